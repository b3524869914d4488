// Integer-only LayerNorm (Sec. 3.6, Eq. 15, Alg. 4).  HBM-bound: 4 bytes in, 1 byte out per element.
//
// A row (C <= 1024 int32) is owned by LPR lanes of one wavefront and kept in registers, so HBM is
// read once.  Sum and sum of squared deviations are butterfly reductions inside the lane group; the
// per-row scalar work (mean, variance, Newton integer square root, reciprocal factor) is done
// redundantly by the lanes of the group, which is why short groups (16 lanes, 4 rows per wave) are
// preferred when there are enough rows to fill the chip.
#include "common.h"

namespace ibert {

struct LayerNormArgs {
    const int32_t* x;
    int8_t* y;
    int64_t rows;
    int32_t C;
    int64_t ldx, ldy;
    const int32_t* gamma_q;
    const int32_t* beta_q;
    int32_t shift;
};

// Alg. 4: Newton iteration for floor(sqrt(n)) from x0 = 2^ceil(Bits(n)/2); stops when the iterate
// no longer decreases.  The loop runs to the stop rule (some inputs need more than four passes).
__device__ __forceinline__ uint32_t isqrt_newton(uint32_t n)
{
    if (n == 0) return 0;
    const int bits = 32 - __clz((int)n);
    uint32_t x = 1u << ((bits + 1) >> 1);            // <= 2^16
    for (;;) {
        const uint32_t y = (x + n / x) >> 1;
        if (y >= x) return x;
        x = y;
    }
}

template <int LPR>
__device__ __forceinline__ int32_t group_sum_i32(int32_t v)
{
#pragma unroll
    for (int off = 1; off < LPR; off <<= 1) v += __shfl_xor(v, off, 64);
    return v;
}

template <int LPR>
__device__ __forceinline__ uint64_t group_sum_u64(uint64_t v)
{
#pragma unroll
    for (int off = 1; off < LPR; off <<= 1) {
        const uint32_t lo = (uint32_t)__shfl_xor((int32_t)(uint32_t)v, off, 64);
        const uint32_t hi = (uint32_t)__shfl_xor((int32_t)(uint32_t)(v >> 32), off, 64);
        v += ((uint64_t)hi << 32) | lo;
    }
    return v;
}

constexpr int LN_THREADS = 256;

template <int LPR, int NCH, bool ALIGNED>
__global__ __launch_bounds__(LN_THREADS) void layernorm_rows_kernel(LayerNormArgs a)
{
    constexpr int ROWS_PER_BLOCK = LN_THREADS / LPR;
    const int lane = threadIdx.x % LPR;
    const int64_t row = (int64_t)blockIdx.x * ROWS_PER_BLOCK + threadIdx.x / LPR;
    const bool live = row < a.rows;
    const int32_t* xr = a.x + (live ? row : 0) * a.ldx;
    const int32_t C = a.C;

    int32_t v[NCH][4];
    int32_t sum = 0;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int col = (c * LPR + lane) * 4;
        if (ALIGNED && live && col + 3 < C) {
            const int4 t = *reinterpret_cast<const int4*>(xr + col);
            v[c][0] = t.x; v[c][1] = t.y; v[c][2] = t.z; v[c][3] = t.w;
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) v[c][e] = (live && col + e < C) ? xr[col + e] : 0;
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            v[c][e] = clamp_i32(v[c][e], -32767, 32767);
            sum += v[c][e];                            // |sum| <= 1024 * 32767 < 2^25
        }
    }
    sum = group_sum_i32<LPR>(sum);

    // mu = floor((sum + floor(C/2)) / C)
    const int32_t num = sum + (C >> 1);
    int32_t mu = num / C;
    if (num - mu * C < 0) mu -= 1;

    // ss = sum d^2 (each d^2 < 2^32, the total < 2^42)
    uint64_t ss = 0;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int col = (c * LPR + lane) * 4;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int32_t d = v[c][e] - mu;
            v[c][e] = d;
            const uint32_t ad = (uint32_t)(d < 0 ? -d : d);
            if (col + e < C) ss += (uint64_t)ad * ad;
        }
    }
    ss = group_sum_u64<LPR>(ss);

    // var = floor(ss / C) < 2^32, with two 32-bit divisions: ss = (t << 11) + low, t < 2^31.
    const uint32_t Cu = (uint32_t)C;
    const uint32_t t = (uint32_t)(ss >> 11);
    const uint32_t qa = t / Cu;
    const uint32_t rem = (uint32_t)(ss - (((uint64_t)qa * Cu) << 11));   // < C * 2^11 + 2^11
    const uint32_t var = (qa << 11) + rem / Cu;

    uint32_t sigma = isqrt_newton(var);
    sigma = sigma < 1u ? 1u : sigma;
    const int32_t f = (int32_t)((1u << 24) / sigma);
    if (!live) return;

    int8_t* yr = a.y + row * a.ldy;
    const int32_t rnd = 1 << (a.shift - 1);
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int col = (c * LPR + lane) * 4;
        if (col >= C) continue;
        int32_t o[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int ce = col + e < C ? col + e : C - 1;
            const int32_t n = (v[c][e] * f) >> 14;                     // |d*f| < 2^30
            const int32_t acc = n * a.gamma_q[ce] + a.beta_q[ce] + rnd;  // < 2^31 by the preconditions
            o[e] = clamp_i32(acc >> a.shift, -127, 127);
        }
        if (ALIGNED && col + 3 < C) {
            *reinterpret_cast<uint32_t*>(yr + col) = pack4_i8(o[0], o[1], o[2], o[3]);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (col + e < C) yr[col + e] = (int8_t)o[e];
        }
    }
}

int check_layernorm(int32_t C, int32_t shift)
{
    if (C < 1 || C > 1024) return IBERT_ERR_PARAM_RANGE;
    if (shift < 1 || shift > 30) return IBERT_ERR_PARAM_RANGE;
    return IBERT_OK;
}

template <int LPR, int NCH>
static void launch_rows(const LayerNormArgs& a, bool al, hipStream_t stream)
{
    constexpr int rpb = LN_THREADS / LPR;
    const unsigned blocks = (unsigned)((a.rows + rpb - 1) / rpb);
    if (al) hipLaunchKernelGGL((layernorm_rows_kernel<LPR, NCH, true>), dim3(blocks), dim3(LN_THREADS), 0, stream, a);
    else hipLaunchKernelGGL((layernorm_rows_kernel<LPR, NCH, false>), dim3(blocks), dim3(LN_THREADS), 0, stream, a);
}

int launch_layernorm(const int32_t* x, int8_t* y, int64_t rows, int32_t C, int64_t ldx, int64_t ldy,
                     const int32_t* gamma_q, const int32_t* beta_q, int32_t shift, hipStream_t stream)
{
    if (rows == 0) return IBERT_OK;
    if (rows > 0x7fffffffLL) return IBERT_ERR_SHAPE;
    LayerNormArgs a{x, y, rows, C, ldx, ldy, gamma_q, beta_q, shift};
    const bool al = aligned(x, 16) && ldx % 4 == 0 && aligned(y, 4) && ldy % 4 == 0;
    // Few rows: spread each row over a whole wavefront; many rows: 16 lanes per row.
    const bool wide = rows < 2048;
    if (wide) {
        if (C <= 256) launch_rows<64, 1>(a, al, stream);
        else if (C <= 512) launch_rows<64, 2>(a, al, stream);
        else launch_rows<64, 4>(a, al, stream);
    } else {
        if (C <= 256) launch_rows<16, 4>(a, al, stream);
        else if (C <= 512) launch_rows<16, 8>(a, al, stream);
        else if (C <= 768) launch_rows<16, 12>(a, al, stream);
        else launch_rows<16, 16>(a, al, stream);
    }
    IBERT_LAUNCH_CHECK("layernorm kernel");
    g_last_kernel = "layernorm_rows_kernel";
    return IBERT_OK;
}

}  // namespace ibert

extern "C" int ibert_layernorm_i(const int32_t* x, int8_t* y, int64_t rows, int32_t C, int64_t ldx, int64_t ldy,
                                 const int32_t* gamma_q, const int32_t* beta_q, int32_t shift, void* stream)
{
    if (rows < 0 || C < 1 || ldx < C || ldy < C) return IBERT_ERR_SHAPE;
    const int rc = ibert::check_layernorm(C, shift);
    if (rc) return rc;
    if (rows == 0) return IBERT_OK;
    if (!x || !y || !gamma_q || !beta_q) return IBERT_ERR_NULL;
    return ibert::launch_layernorm(x, y, rows, C, ldx, ldy, gamma_q, beta_q, shift, (hipStream_t)stream);
}
