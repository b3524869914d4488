// Shared declarations of the libibert sources: error plumbing, device-side integer helpers,
// internal launcher prototypes.  gfx950 only.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ibert.h"

namespace ibert {

// Records the text of a failed HIP call for ibert_last_hip_error().
int hip_failed(hipError_t e, const char* what);

#define IBERT_HIP_CHECK(expr)                                         \
    do {                                                              \
        hipError_t _e = (expr);                                       \
        if (_e != hipSuccess) return ::ibert::hip_failed(_e, #expr);  \
    } while (0)

// Launch check: kernels are enqueued asynchronously, so only launch-time errors show up here.
#define IBERT_LAUNCH_CHECK(name)                                        \
    do {                                                                \
        hipError_t _e = hipGetLastError();                              \
        if (_e != hipSuccess) return ::ibert::hip_failed(_e, name);     \
    } while (0)

inline bool dyadic_ok(const ibert_dyadic& d) { return d.s >= 0 && d.s <= 62; }
inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// ---- device helpers -------------------------------------------------------------------------
// Requantization: round-half-up of x*m/2^s, exact in 64 bits (|x|,|m| < 2^31, s <= 62).
__device__ __forceinline__ int64_t dyadic64(int32_t x, int32_t m, int32_t s)
{
    int64_t p = (int64_t)x * (int64_t)m;
    if (s > 0) p = (p + ((int64_t)1 << (s - 1))) >> s;
    return p;
}

__device__ __forceinline__ int32_t clamp_i64_to_i32(int64_t v, int32_t lim)
{
    const int64_t l = lim;
    v = v < -l ? -l : v;
    v = v > l ? l : v;
    return (int32_t)v;
}

__device__ __forceinline__ int32_t clamp_i32(int32_t v, int32_t lo, int32_t hi)
{
    return v < lo ? lo : (v > hi ? hi : v);
}

// Packs four values already inside [-128,127] into one little-endian dword.
__device__ __forceinline__ uint32_t pack4_i8(int32_t a, int32_t b, int32_t c, int32_t d)
{
    return (uint32_t)(a & 0xff) | ((uint32_t)(b & 0xff) << 8) | ((uint32_t)(c & 0xff) << 16) |
           ((uint32_t)(d & 0xff) << 24);
}

// clamp(v, lo, hi) for lo <= hi in one instruction.
__device__ __forceinline__ int32_t med3_i32(int32_t v, int32_t lo, int32_t hi)
{
    int32_t r;
    asm("v_med3_i32 %0, %1, %2, %3" : "=v"(r) : "v"(v), "v"(lo), "v"(hi));
    return r;
}

// Full-rate 24-bit multiplies (low 32 bits of the product of the operands' low 24 bits), with explicit types.
__device__ __forceinline__ uint32_t umul24(uint32_t a, uint32_t b) { return (uint32_t)__umul24(a, b); }
__device__ __forceinline__ int32_t smul24(int32_t a, int32_t b) { return (int32_t)__mul24(a, b); }

// a*b + c with 24-bit operands in one full-rate instruction (the compiler otherwise tends to pick a 64-bit
// multiply-add for this pattern).
__device__ __forceinline__ uint32_t umad24(uint32_t a, uint32_t b, uint32_t c)
{
    uint32_t r;
    asm("v_mad_u32_u24 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}
__device__ __forceinline__ int32_t smad24(int32_t a, int32_t b, int32_t c)
{
    int32_t r;
    asm("v_mad_i32_i24 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// Four values already inside [-128,127] -> one dword, three byte permutes.
__device__ __forceinline__ uint32_t pack4_perm(int32_t a, int32_t b, int32_t c, int32_t d)
{
    const uint32_t lo = __builtin_amdgcn_perm((uint32_t)b, (uint32_t)a, 0x0c0c0400u);   // a.b0, b.b0, 0, 0
    const uint32_t hi = __builtin_amdgcn_perm((uint32_t)d, (uint32_t)c, 0x0c0c0400u);
    return __builtin_amdgcn_perm(hi, lo, 0x05040100u);
}

// Cross-lane moves inside a row of 16 lanes (DPP): butterfly partners for all-reduce.
//   0xB1 quad_perm(1,0,3,2)  0x4E quad_perm(2,3,0,1)  0x141 row_half_mirror  0x140 row_mirror
template <int CTRL>
__device__ __forceinline__ int32_t dpp_mov(int32_t v)
{
    return __builtin_amdgcn_update_dpp(v, v, CTRL, 0xF, 0xF, false);
}

// All-reduce over groups of LPR consecutive lanes (LPR = 16, 32 or 64; groups are aligned).
template <int LPR, typename Op>
__device__ __forceinline__ int32_t group_allreduce(int32_t v, Op op)
{
    v = op(v, dpp_mov<0xB1>(v));
    v = op(v, dpp_mov<0x4E>(v));
    v = op(v, dpp_mov<0x141>(v));
    v = op(v, dpp_mov<0x140>(v));
    if (LPR > 16) v = op(v, __shfl_xor(v, 16, 64));
    if (LPR > 32) v = op(v, __shfl_xor(v, 32, 64));
    return v;
}

// Name of the kernel family chosen by the most recent launch_* call (for the optional profile).
extern const char* g_last_kernel;

// ---- internal launchers (validated arguments) -----------------------------------------------
int launch_gemm(const ibert_gemm_desc& d, const int8_t* A, const int8_t* W, const int32_t* bias,
                const int32_t* mult, const int32_t* shift, const int8_t* residual, void* C,
                hipStream_t stream, const ibert_gelu_params* gelu = nullptr);
int launch_gemm_gelu(const ibert_gemm_desc& d, const int8_t* A, const int8_t* W, const int32_t* bias,
                     const int32_t* mult, const int32_t* shift, const ibert_gelu_params& gelu, int8_t* C,
                     int32_t* scratch, hipStream_t stream);
bool attention_fused_ok(const int8_t* qkv, const int8_t* ctx, int32_t seq, int32_t hidden, int32_t heads);
int launch_attention(const int8_t* qkv, int8_t* ctx, int32_t batch, int32_t seq, int32_t hidden, int32_t heads,
                     ibert_dyadic scores_dy, const ibert_softmax_params& sp, ibert_dyadic ctx_dy, hipStream_t stream,
                     const int32_t* key_lens = nullptr);
// key_lens (device, optional): row r keeps its first key_lens[r / rows_per_len] columns
int launch_softmax(const int32_t* x, void* y, int64_t rows, int32_t cols, int64_t ldx, int64_t ldy,
                   const ibert_softmax_params& p, hipStream_t stream, const int32_t* key_lens = nullptr,
                   int64_t rows_per_len = 0);
int launch_gelu(const int32_t* x, int8_t* y, int64_t n, const ibert_gelu_params& p, hipStream_t stream);
int launch_hgelu(const int32_t* x, int8_t* y, int64_t n, const ibert_hgelu_params& p, hipStream_t stream);
int launch_layernorm(const int32_t* x, int8_t* y, int64_t rows, int32_t C, int64_t ldx, int64_t ldy,
                     const int32_t* gamma_q, const int32_t* beta_q, int32_t shift, hipStream_t stream);
int launch_layernorm16(const int16_t* x, int8_t* y, int64_t rows, int32_t C, int64_t ldx, int64_t ldy,
                       const int32_t* gamma_q, const int32_t* beta_q, int32_t shift, hipStream_t stream);
int launch_embedding(const int32_t* ids, const int8_t* tok, const int8_t* pos, int64_t tokens, int32_t seq, int32_t C,
                     int32_t vocab, ibert_dyadic tok_dy, ibert_dyadic pos_dy, const int32_t* gamma_q,
                     const int32_t* beta_q, int32_t shift, int8_t* y, int64_t ldy, hipStream_t stream);

// Parameter validation shared by the public entry points and the layer.
int check_gemm(const ibert_gemm_desc& d, const void* A, const void* W, const void* mult,
               const void* shift, const void* residual, const void* C);
int check_softmax(const ibert_softmax_params& p, int32_t cols);
int check_gelu(const ibert_gelu_params& p);
int check_hgelu(const ibert_hgelu_params& p);
int check_layernorm(int32_t C, int32_t shift);

}  // namespace ibert
