// Integer-only Softmax arithmetic of one element (Alg. 3; Eq. 11-14): shared by the row kernels and by the
// attention kernel that keeps a score row in registers.
#pragma once
#include "common.h"

namespace ibert {

struct SoftmaxConst {
    uint32_t q_ln2, q_b, q_c;
    uint32_t magic;      // floor(2^32 / q_ln2) + 1  (0 stands for 2^32, i.e. q_ln2 == 1)
    uint32_t d_cap;      // 31 * q_ln2: differences at or beyond it contribute e = 0
    uint32_t magic27;    // floor(2^27 / q_ln2) + 1, used by the 24-bit path
    int32_t k;           // output fractional bits
};

// Host: derived constants, and whether the 24-bit forms apply (see iexp_from_diff_fast).
inline SoftmaxConst softmax_const(const ibert_softmax_params& p)
{
    SoftmaxConst a;
    a.q_ln2 = (uint32_t)p.q_ln2; a.q_b = (uint32_t)p.q_b; a.q_c = (uint32_t)p.q_c;
    a.magic = p.q_ln2 == 1 ? 0u : (uint32_t)((((uint64_t)1 << 32) / (uint32_t)p.q_ln2) + 1);
    a.d_cap = 31u * (uint32_t)p.q_ln2;                 // q_ln2 <= q_b < 2^16 by the preconditions
    a.magic27 = (uint32_t)((1u << 27) / (uint32_t)p.q_ln2) + 1u;
    a.k = p.out_frac_bits;
    return a;
}
inline bool softmax_fast_ok(const ibert_softmax_params& p)
{
    const int64_t poly_max = (int64_t)p.q_b * p.q_b + p.q_c;
    return p.q_ln2 > 8 && p.q_ln2 < 2080 && poly_max >= 256 && poly_max < (1 << 24);
}

// e = I-Exp(-(d)) for a non-negative difference d = max - q (Alg. 3):
//   z = floor(d / q_ln2), r = d - z q_ln2, e = ((q_b - r)^2 + q_c) >> z.
// d is first capped at 31*q_ln2 (z = 31 already shifts every 31-bit polynomial value to zero).
// floor(d/q_ln2) uses a reciprocal multiply: est = mulhi(d, magic) is z or z+1; one fix-up step.
__device__ __forceinline__ uint32_t iexp_from_diff(uint32_t d, const SoftmaxConst& a)
{
    d = d < a.d_cap ? d : a.d_cap;
    uint32_t z = a.magic ? __umulhi(d, a.magic) : d;
    int32_t r = (int32_t)(d - z * a.q_ln2);
    if (r < 0) { r += (int32_t)a.q_ln2; z -= 1; }
    const uint32_t v = a.q_b - (uint32_t)r;            // may be "negative": squared below, mod 2^32 is exact
    const uint32_t poly = v * v + a.q_c;               // I-Poly, Alg. 1 (true value < 2^31)
    return poly >> z;                                  // z <= 31
}

// The same value with full-rate 24-bit multiplies, valid when 8 < q_ln2 < 2080 and q_b^2 + q_c < 2^24
// (host-checked): d <= 31 q_ln2 < 2^16, so with M = floor(2^27/q_ln2) + 1 the product d*M stays below 2^32 and
// floor(d*M / 2^27) = floor(d / q_ln2) exactly (the excess d/2^27 is below 1/q_ln2 because 31 q_ln2^2 < 2^27);
// q_b - r = q_b - d + z q_ln2 is one multiply-add; (q_b - r)^2 + q_c another.
__device__ __forceinline__ uint32_t iexp_from_diff_fast(uint32_t d, const SoftmaxConst& a)
{
    d = d < a.d_cap ? d : a.d_cap;
    const uint32_t z = umul24(d, a.magic27) >> 27;
    const uint32_t v = umad24(z, a.q_ln2, a.q_b - d);           // q_b - r, in (0, q_b]
    const uint32_t poly = umad24(v, v, a.q_c);                  // I-Poly, Alg. 1
    return poly >> z;
}

// y = min(cap, (e*Fz + 2^(30-k)) >> (31-k)),  Fz = floor(2^31 / sum)
__device__ __forceinline__ uint32_t normalise(uint32_t e, uint32_t Fz, int32_t k)
{
    return (e * Fz + (1u << (30 - k))) >> (31 - k);
}

}  // namespace ibert
