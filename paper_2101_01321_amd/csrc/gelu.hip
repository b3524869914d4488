// Integer-only GELU (Alg. 2, Eq. 8-9) fused with the requantization to INT8.
// Element-wise and HBM-bound: 4 bytes in, 1 byte out per element.  Each lane streams 16-byte
// chunks (four int32), several in flight, and writes one packed dword per chunk.
#include "common.h"
#include "gelu_math.h"

namespace ibert {

struct GeluArgs {
    const int32_t* x;
    int8_t* y;
    int64_t n;
    GeluConst c;
    HGeluConst h;       // read by the h-GELU instantiations only
};

constexpr int GELU_THREADS = 256;
constexpr int GELU_UNROLL = 4;                        // 16-byte chunks per lane

// HG: h-GELU (Eq. 6) instead of i-GELU (Alg. 2); the streaming skeleton is the same.
template <bool VEC, bool FAST, bool HG = false>
__global__ __launch_bounds__(GELU_THREADS) void gelu_kernel(GeluArgs a)
{
    const int64_t block_base = (int64_t)blockIdx.x * (GELU_THREADS * GELU_UNROLL * 4);
    const int32_t out_s = HG ? a.h.s : a.c.s;
    const int32_t rnd = 1 << ((out_s - 33) & 31), sh = (out_s - 32) & 31;
    auto one = [&](int32_t q) {
        if (HG) return FAST ? hgelu_one_fast(q, a.h, rnd, sh) : hgelu_one(q, a.h);
        return FAST ? gelu_one_fast(q, a.c, rnd, sh) : gelu_one(q, a.c);
    };
    if (VEC) {
        int4 v[GELU_UNROLL];
        int64_t base[GELU_UNROLL];
#pragma unroll
        for (int u = 0; u < GELU_UNROLL; ++u) {
            base[u] = block_base + ((int64_t)u * GELU_THREADS + threadIdx.x) * 4;
            if (base[u] + 3 < a.n) v[u] = *reinterpret_cast<const int4*>(a.x + base[u]);
        }
#pragma unroll
        for (int u = 0; u < GELU_UNROLL; ++u) {
            if (base[u] + 3 < a.n) {
                *reinterpret_cast<uint32_t*>(a.y + base[u]) = pack4_perm(one(v[u].x), one(v[u].y), one(v[u].z), one(v[u].w));
            } else {
                for (int64_t i = base[u]; i < a.n; ++i) a.y[i] = (int8_t)one(a.x[i]);
            }
        }
    } else {
#pragma unroll
        for (int u = 0; u < GELU_UNROLL * 4; ++u) {
            const int64_t i = block_base + (int64_t)u * GELU_THREADS + threadIdx.x;
            if (i < a.n) a.y[i] = (int8_t)one(a.x[i]);
        }
    }
}

int check_gelu(const ibert_gelu_params& p)
{
    if (p.q_b > 0 || p.q_max < 0 || !dyadic_ok(p.out)) return IBERT_ERR_PARAM_RANGE;
    const int64_t top = (int64_t)p.q_b * p.q_b + p.q_c;          // I-Poly at u = 0
    const int64_t a1 = top < 0 ? -top : top;
    const int64_t a2 = p.q_c < 0 ? -(int64_t)p.q_c : p.q_c;      // I-Poly at u = -q_b
    const int64_t a = a1 > a2 ? a1 : a2;
    const int64_t q1 = p.q_1 < 0 ? -(int64_t)p.q_1 : p.q_1;
    if (a > 2147483647LL) return IBERT_ERR_PARAM_RANGE;
    if ((__int128)p.q_max * (a + q1) > 2147483647LL) return IBERT_ERR_PARAM_RANGE;
    return IBERT_OK;
}

int check_hgelu(const ibert_hgelu_params& p)
{
    if (!dyadic_ok(p.slope) || !dyadic_ok(p.out)) return IBERT_ERR_PARAM_RANGE;
    if (p.q_3 < 0 || p.q_6 < p.q_3 || p.q_max < 0) return IBERT_ERR_PARAM_RANGE;
    if ((__int128)p.q_max * p.q_6 > 2147483647LL) return IBERT_ERR_PARAM_RANGE;
    return IBERT_OK;
}

int launch_hgelu(const int32_t* x, int8_t* y, int64_t n, const ibert_hgelu_params& p, hipStream_t stream)
{
    if (n == 0) return IBERT_OK;
    GeluArgs a{x, y, n, GeluConst{}, HGeluConst{p.slope.m, p.slope.s, p.q_3, p.q_6, p.q_max, p.out.m, p.out.s}};
    const int64_t per_block = (int64_t)GELU_THREADS * GELU_UNROLL * 4;
    const int64_t blocks = (n + per_block - 1) / per_block;
    if (blocks > 0x7fffffffLL) return IBERT_ERR_SHAPE;
    const bool vec = aligned(x, 16) && aligned(y, 4);
    const bool fast = hgelu_fast_ok(p);
    const dim3 grid((unsigned)blocks), block(GELU_THREADS);
    if (vec && fast) hipLaunchKernelGGL((gelu_kernel<true, true, true>), grid, block, 0, stream, a);
    else if (vec) hipLaunchKernelGGL((gelu_kernel<true, false, true>), grid, block, 0, stream, a);
    else if (fast) hipLaunchKernelGGL((gelu_kernel<false, true, true>), grid, block, 0, stream, a);
    else hipLaunchKernelGGL((gelu_kernel<false, false, true>), grid, block, 0, stream, a);
    IBERT_LAUNCH_CHECK("gelu_kernel<h-GELU>");
    g_last_kernel = "gelu_kernel<h-GELU>";
    return IBERT_OK;
}

int launch_gelu(const int32_t* x, int8_t* y, int64_t n, const ibert_gelu_params& p, hipStream_t stream)
{
    if (n == 0) return IBERT_OK;
    GeluArgs a{x, y, n, GeluConst{p.q_b, p.q_c, p.q_1, p.q_max, p.out.m, p.out.s}, HGeluConst{}};
    const int64_t per_block = (int64_t)GELU_THREADS * GELU_UNROLL * 4;
    const int64_t blocks = (n + per_block - 1) / per_block;
    if (blocks > 0x7fffffffLL) return IBERT_ERR_SHAPE;
    const bool vec = aligned(x, 16) && aligned(y, 4);
    const bool fast = gelu_fast_ok(p);                 // 24-bit fast path
    const dim3 grid((unsigned)blocks), block(GELU_THREADS);
    if (vec && fast) hipLaunchKernelGGL((gelu_kernel<true, true>), grid, block, 0, stream, a);
    else if (vec) hipLaunchKernelGGL((gelu_kernel<true, false>), grid, block, 0, stream, a);
    else if (fast) hipLaunchKernelGGL((gelu_kernel<false, true>), grid, block, 0, stream, a);
    else hipLaunchKernelGGL((gelu_kernel<false, false>), grid, block, 0, stream, a);
    IBERT_LAUNCH_CHECK("gelu_kernel");
    g_last_kernel = "gelu_kernel";
    return IBERT_OK;
}

}  // namespace ibert

extern "C" int ibert_gelu_i(const int32_t* x, int8_t* y, int64_t n, const ibert_gelu_params* params, void* stream)
{
    if (!params) return IBERT_ERR_NULL;
    if (n < 0) return IBERT_ERR_SHAPE;
    const int rc = ibert::check_gelu(*params);
    if (rc) return rc;
    if (n == 0) return IBERT_OK;
    if (!x || !y) return IBERT_ERR_NULL;
    return ibert::launch_gelu(x, y, n, *params, (hipStream_t)stream);
}

extern "C" int ibert_hgelu_i(const int32_t* x, int8_t* y, int64_t n, const ibert_hgelu_params* params, void* stream)
{
    if (!params) return IBERT_ERR_NULL;
    if (n < 0) return IBERT_ERR_SHAPE;
    const int rc = ibert::check_hgelu(*params);
    if (rc) return rc;
    if (n == 0) return IBERT_OK;
    if (!x || !y) return IBERT_ERR_NULL;
    return ibert::launch_hgelu(x, y, n, *params, (hipStream_t)stream);
}
