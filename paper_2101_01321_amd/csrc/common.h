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

// Name of the kernel family chosen by the most recent launch_* call (for the optional profile).
extern const char* g_last_kernel;

// ---- internal launchers (validated arguments) -----------------------------------------------
int launch_gemm(const ibert_gemm_desc& d, const int8_t* A, const int8_t* W, const int32_t* bias,
                const int32_t* mult, const int32_t* shift, const int8_t* residual, void* C,
                hipStream_t stream);
int launch_softmax(const int32_t* x, void* y, int64_t rows, int32_t cols, int64_t ldx, int64_t ldy,
                   const ibert_softmax_params& p, hipStream_t stream);
int launch_gelu(const int32_t* x, int8_t* y, int64_t n, const ibert_gelu_params& p, hipStream_t stream);
int launch_layernorm(const int32_t* x, int8_t* y, int64_t rows, int32_t C, int64_t ldx, int64_t ldy,
                     const int32_t* gamma_q, const int32_t* beta_q, int32_t shift, hipStream_t stream);

// Parameter validation shared by the public entry points and the layer.
int check_gemm(const ibert_gemm_desc& d, const void* A, const void* W, const void* mult,
               const void* shift, const void* residual, const void* C);
int check_softmax(const ibert_softmax_params& p, int32_t cols);
int check_gelu(const ibert_gelu_params& p);
int check_layernorm(int32_t C, int32_t shift);

}  // namespace ibert
