// Integer LayerNorm (Sec. 3.6, Eq. 15, Alg. 4): the per-row scalar steps, shared by the row kernel and by the MatMul
// epilogue that normalizes its own output.
#pragma once
#include "common.h"

namespace ibert {

// floor(u / C) for u < 2^31: est = mulhi(u, magic) is the quotient or one more (the excess is below
// u / 2^32 < 1); one fix-up step from the sign of the remainder.
__device__ __forceinline__ uint32_t udiv_c(uint32_t u, uint32_t C, uint32_t magic)
{
    if (magic == 0) return u;
    const uint32_t q = __umulhi(u, magic);
    const int32_t r = (int32_t)(u - q * C);
    return r < 0 ? q - 1 : q;
}

// floor(sqrt(n)), the value the Newton iteration of Alg. 4 ends on (started at or above the root, its integer
// iterates decrease to exactly the floor of the root).  Here: a single-precision estimate -- n rounded to 24 bits
// and a correctly rounded root are together less than 0.01 away from the true root, so the truncated estimate is
// off by at most one -- and one exact correction step in integers.
__device__ __forceinline__ uint32_t isqrt_floor(uint32_t n)
{
    uint32_t x = (uint32_t)__fsqrt_rn((float)n);
    x = x > 65535u ? 65535u : x;                       // keeps the squares below inside 32 bits
    if (x * x > n) return x - 1;
    if (x < 65535u && (x + 1) * (x + 1) <= n) return x + 1;
    return x;
}

// mu = floor((sum + floor(C/2)) / C) for |sum| <= 1024 * 32767, computed on the non-negative number sum + C/2 + 32768 C.
__device__ __forceinline__ int32_t ln_row_mean(int32_t sum, uint32_t C, uint32_t magic)
{
    return (int32_t)udiv_c((uint32_t)(sum + (int32_t)(C >> 1) + (int32_t)(C << 15)), C, magic) - 32768;
}

// f = floor(2^24 / max(1, floor(sqrt(floor(ss / C))))) for ss = sum of squared deviations < 2^42 (C <= 1024).
// var = floor(ss / C) < 2^32 with two 32-bit divisions: ss = (t << 11) + low, t < 2^31.
__device__ __forceinline__ int32_t ln_row_factor(uint64_t ss, uint32_t C, uint32_t magic)
{
    const uint32_t t = (uint32_t)(ss >> 11);
    const uint32_t qa = udiv_c(t, C, magic);
    const uint32_t rem = (uint32_t)(ss - (((uint64_t)qa * C) << 11));   // < C * 2^11 + 2^11
    const uint32_t var = (qa << 11) + udiv_c(rem, C, magic);
    uint32_t sigma = isqrt_floor(var);
    sigma = sigma < 1u ? 1u : sigma;
    return (int32_t)((1u << 24) / sigma);
}

inline uint32_t ln_magic_for(int32_t C) { return C == 1 ? 0u : (uint32_t)((((uint64_t)1 << 32) / (uint32_t)C) + 1); }

}  // namespace ibert
