// Integer-only GELU of one value (Alg. 2, Eq. 8-9) followed by the requantization to INT8: shared by the
// element-wise kernel and by the MatMul epilogue that applies GELU to its own output.
#pragma once
#include "common.h"

namespace ibert {

struct GeluConst {
    int32_t q_b, q_c, q_1, q_max;
    int32_t m, s;          // output requantization
};

// General parameters.  All products stay inside 32 bits by the host-checked preconditions
// ((u+q_b)^2 + q_c and q*(erf+q_1) are bounded by q_max * (|poly| + |q_1|) < 2^31).
__device__ __forceinline__ int32_t gelu_one(int32_t q, const GeluConst& a)
{
    q = clamp_i32(q, -a.q_max, a.q_max);
    int32_t u = q < 0 ? -q : q;
    u = u > -a.q_b ? -a.q_b : u;                      // clip(|q|, max = -q_b)
    const int32_t v = u + a.q_b;
    // I-Poly, Alg. 1.  Unsigned arithmetic: the true values fit 32 bits, partial terms may wrap.
    const uint32_t poly = (uint32_t)v * (uint32_t)v + (uint32_t)a.q_c;
    const uint32_t erf = q < 0 ? 0u - poly : (q == 0 ? 0u : poly);          // sgn(q) * poly
    const int32_t t = (int32_t)((uint32_t)q * (erf + (uint32_t)a.q_1));
    return clamp_i64_to_i32(dyadic64(t, a.m, a.s), 127);
}

// When q_max, |q_b| and max|erf + q_1| are below 2^23 and the output shift is in [33, 62]: every product is a
// full-rate 24-bit multiply, and the requantization is a multiply-high, an add and a shift
// (floor((t m + 2^(s-1)) / 2^s) = (hi32(t m) + 2^(s-33)) >> (s-32), exact for s >= 33).
// sgn(q)*poly needs no special case at q = 0 because t = q * (...) is zero there anyway.
// rnd = 2^(s-33), sh = s - 32.
__device__ __forceinline__ int32_t gelu_one_fast(int32_t q, const GeluConst& a, int32_t rnd, int32_t sh)
{
    q = med3_i32(q, -a.q_max, a.q_max);
    const int32_t aq = max(q, -q);
    const int32_t v = min(aq, -a.q_b) + a.q_b;        // in [q_b, 0]
    const int32_t poly = smad24(v, v, a.q_c);         // I-Poly, Alg. 1
    const int32_t sg = q >> 31;
    const int32_t erf = (poly ^ sg) - sg;             // -poly for q < 0
    const int32_t t = smul24(q, erf + a.q_1);
    return med3_i32((__mulhi(t, a.m) + rnd) >> sh, -127, 127);
}

// Host: do the parameters allow gelu_one_fast?
inline bool gelu_fast_ok(const ibert_gelu_params& p)
{
    const int64_t top = (int64_t)p.q_b * p.q_b + p.q_c;
    const int64_t a1 = top < 0 ? -top : top, a2 = p.q_c < 0 ? -(int64_t)p.q_c : p.q_c;
    const int64_t wmax = (a1 > a2 ? a1 : a2) + (p.q_1 < 0 ? -(int64_t)p.q_1 : p.q_1);
    const int64_t lim = 1 << 23;
    return p.q_max < lim && -(int64_t)p.q_b < lim && wmax < lim && p.out.s >= 33 && p.out.s <= 62;
}

// ---- h-GELU (Eq. 6): x ReLU6(1.702 x + 3) / 6 on integers ----------------------------------------------------
struct HGeluConst {
    int32_t slope_m, slope_s;      // ~1.702
    int32_t q_3, q_6, q_max;
    int32_t m, s;                  // output requantization (carries the 1/6)
};

// General parameters: 64-bit throughout; q*u fits 32 bits by the host-checked precondition q_max * q_6 < 2^31.
__device__ __forceinline__ int32_t hgelu_one(int32_t q, const HGeluConst& a)
{
    q = clamp_i32(q, -a.q_max, a.q_max);
    int64_t u = dyadic64(q, a.slope_m, a.slope_s) + a.q_3;
    u = u < 0 ? 0 : (u > a.q_6 ? a.q_6 : u);
    const int32_t t = q * (int32_t)u;
    return clamp_i64_to_i32(dyadic64(t, a.m, a.s), 127);
}

// When the slope shift is in [1, 31], |q_max * slope| + q_3 < 2^31 - 1, q_max and q_6 are below 2^23 and the output
// shift is in [33, 62]: the gate is bits [s, s+32) of the 64-bit sum q m + 2^(s-1) (one funnel shift), q*u a 24-bit
// multiply, and the requantization the multiply-high form of gelu_one_fast.
__device__ __forceinline__ int32_t hgelu_one_fast(int32_t q, const HGeluConst& a, int32_t rnd, int32_t sh)
{
    q = med3_i32(q, -a.q_max, a.q_max);
    const int64_t p = (int64_t)q * a.slope_m + ((int64_t)1 << (a.slope_s - 1));
    const int32_t g = (int32_t)__builtin_amdgcn_alignbit((uint32_t)(p >> 32), (uint32_t)p, (uint32_t)(a.slope_s & 31));
    const int32_t u = med3_i32(g + a.q_3, 0, a.q_6);
    const int32_t t = smul24(q, u);
    return med3_i32((__mulhi(t, a.m) + rnd) >> sh, -127, 127);
}

inline bool hgelu_fast_ok(const ibert_hgelu_params& p)
{
    if (p.slope.s < 1 || p.slope.s > 31 || p.out.s < 33 || p.out.s > 62) return false;
    const int64_t lim = 1 << 23;
    if (p.q_max >= lim || p.q_6 >= lim) return false;
    const __int128 top = (((__int128)p.q_max * (p.slope.m < 0 ? -(int64_t)p.slope.m : p.slope.m)) >> p.slope.s) + 1 + p.q_3;
    return top < 2147483647LL;
}

}  // namespace ibert
