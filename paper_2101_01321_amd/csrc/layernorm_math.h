// Integer LayerNorm (Sec. 3.6, Eq. 15, Alg. 4): the per-row scalar steps of the row kernel.  Integer instructions only.
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

// floor(sqrt(n)) for any 32-bit n -- the integer Alg. 4 returns (its Newton iterates start at 2^ceil(Bits(n)/2), at or
// above the root, and decrease to exactly the floor of the root; Sec. 3.6).  The row kernel has the LPR lanes of a row
// at hand, all holding the same n, so it finds that integer by a radix-LPR search instead of a chain of up to six
// dependent divisions: the root r is the number of c in [1, 65535] with c^2 <= n, a monotone predicate, and in each
// round lane l tests c = r + (l + 1) << s, the lanes that pass are counted (they are the first ones), and r grows by
// count << s.  After the round with shift s: r <= root < r + 2^s (candidates at or past r + 2^s_previous fail by
// themselves), so s = 0 ends it.  Three rounds of a shift, a multiply, two compares and a population count for 64
// lanes, four for 32.  `lane_in_row` = the lane's index inside its group of LPR consecutive lanes; every lane of the
// wavefront must call this together.
template <int LPR>
__device__ __forceinline__ uint32_t isqrt_floor_rowwise(uint32_t n, int lane_in_row)
{
    static_assert(LPR == 16 || LPR == 32 || LPR == 64, "lanes per row");
    // shifts of the rounds: 6, 5 or 4 bits of the root per round
    constexpr int NR = LPR == 64 ? 3 : 4;
    constexpr int SH[4] = {LPR == 64 ? 10 : (LPR == 32 ? 11 : 12), LPR == 64 ? 4 : (LPR == 32 ? 6 : 8),
                           LPR == 64 ? 0 : (LPR == 32 ? 1 : 4), 0};
    uint32_t r = 0;
#pragma unroll
    for (int k = 0; k < NR; ++k) {
        const uint32_t c = r + ((uint32_t)(lane_in_row + 1) << SH[k]);
        const bool pass = c <= 65535u && c * c <= n;                 // c < 2^16: the square fits 32 bits
        const unsigned long long b = __builtin_amdgcn_ballot_w64(pass);
        uint32_t cnt;
        if (LPR == 64) cnt = (uint32_t)__popcll(b);
        else if (LPR == 32) cnt = (uint32_t)__popc((threadIdx.x & 32) ? (uint32_t)(b >> 32) : (uint32_t)b);
        else cnt = (uint32_t)__popc((uint32_t)(b >> (threadIdx.x & 48)) & 0xffffu);
        r += cnt << SH[k];
    }
    return r;
}

// The same integer for a lane on its own (every lane its own n): the shift-and-subtract square root, sixteen steps of
// an add, a compare and a conditional subtract, no division and no multiplication.  Invariant after the step with
// bit b: res = floor(sqrt(n0 >> 2b)) << b (in the shifted representation below) and n = n0 - res^2 on the bits
// looked at so far.
__device__ __forceinline__ uint32_t isqrt_floor_lane(uint32_t n)
{
    uint32_t res = 0;
#pragma unroll
    for (uint32_t bit = 1u << 30; bit != 0; bit >>= 2) {
        const uint32_t t = res + bit;
        const bool ge = n >= t;
        n = ge ? n - t : n;
        res = ge ? (res >> 1) + bit : res >> 1;
    }
    return res;
}

// mu = floor((sum + floor(C/2)) / C) for |sum| <= 1024 * 32767, computed on the non-negative number sum + C/2 + 32768 C.
__device__ __forceinline__ int32_t ln_row_mean(int32_t sum, uint32_t C, uint32_t magic)
{
    return (int32_t)udiv_c((uint32_t)(sum + (int32_t)(C >> 1) + (int32_t)(C << 15)), C, magic) - 32768;
}

// var = floor(ss / C) < 2^32 for ss = sum of squared deviations < 2^42 (C <= 1024), with two 32-bit divisions:
// ss = (t << 11) + low, t < 2^31.
__device__ __forceinline__ uint32_t ln_row_variance(uint64_t ss, uint32_t C, uint32_t magic)
{
    const uint32_t t = (uint32_t)(ss >> 11);
    const uint32_t qa = udiv_c(t, C, magic);
    const uint32_t rem = (uint32_t)(ss - (((uint64_t)qa * C) << 11));   // < C * 2^11 + 2^11
    return (qa << 11) + udiv_c(rem, C, magic);
}

// f = floor(2^24 / max(1, sigma)).
__device__ __forceinline__ int32_t ln_factor_of_sigma(uint32_t sigma)
{
    sigma = sigma < 1u ? 1u : sigma;
    return (int32_t)((1u << 24) / sigma);
}

inline uint32_t ln_magic_for(int32_t C) { return C == 1 ? 0u : (uint32_t)((((uint64_t)1 << 32) / (uint32_t)C) + 1); }

}  // namespace ibert
