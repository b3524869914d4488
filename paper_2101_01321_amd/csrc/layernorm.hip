// Integer-only LayerNorm (Sec. 3.6, Eq. 15, Alg. 4).  HBM-bound: 4 bytes in, 1 byte out per element.
//
// A row (C <= 1024 int32) is owned by LPR lanes of one wavefront and kept in registers, so HBM is
// read once.  Sum and sum of squares are butterfly reductions inside the lane group; mean, variance and the
// reciprocal factor are worked out redundantly by the lanes of the group, the integer square root (the value
// Alg. 4 returns) by the lanes of the group together, each testing one candidate per round.  No floating point.
//
// The same kernel also serves the INT8 embedding (Sec. 1, contribution 3; App. C.1): there the row is not read from
// an INT32 buffer but made on the fly from one row of the INT8 token table and one of the INT8 position table, each
// rescaled by a dyadic number to the common INT32 scale of the sum, and then normalized as above.
#include "common.h"
#include "layernorm_math.h"

namespace ibert {

struct EmbedArgs {
    const int32_t* ids;  // [rows] token ids, clamped into [0, vocab)
    const int8_t* tok;   // [vocab, C]
    const int8_t* pos;   // [>= seq, C]; row r takes position r mod seq
    int32_t seq, vocab;
    int32_t tok_m, tok_s, pos_m, pos_s;
};

struct LayerNormArgs {
    const int32_t* x;    // rows of int32, or of int16 (X16 instantiations: same values in half the bytes)
    int8_t* y;
    int64_t rows;
    int32_t C;
    int64_t ldx, ldy;
    const int32_t* gamma_q;
    const int32_t* beta_q;
    int32_t shift;
    uint32_t magic_c;    // floor(2^32 / C) + 1 (0 for C == 1): reciprocal multiply for the divisions by C
    EmbedArgs emb;       // only read by the embedding instantiations
};

template <int LPR>
__device__ __forceinline__ int32_t group_sum_i32(int32_t v)
{
    return group_allreduce<LPR>(v, [](int32_t a, int32_t b) { return a + b; });
}

// 64-bit all-reduce built from 32-bit ones.
template <int LPR>
__device__ __forceinline__ uint64_t group_sum_u64(uint64_t v)
{
    // every lane value is below 2^35 here (at most 32 squares below 2^30); split at bit 19 so that both parts,
    // summed over 64 lanes, stay below 2^25 and plain 32-bit all-reduces are exact
    const int32_t l0 = (int32_t)(v & 0x7ffff), l1 = (int32_t)(v >> 19);
    const uint64_t s0 = (uint32_t)group_sum_i32<LPR>(l0), s1 = (uint32_t)group_sum_i32<LPR>(l1);
    return s0 + (s1 << 19);
}

constexpr int LN_THREADS = 256;

// ALIGNED: rows 16-byte (x) / 4-byte (y) aligned, C % 4 == 0, gamma/beta 16-byte aligned: every 4-element
// chunk is either entirely inside the row or entirely outside, and moves as one vector.
// EMB: the row is DY(tok[id]) + DY(pos[row mod seq]) instead of x[row] (ALIGNED then means 4-byte aligned table rows).
// FULL: C == NCH * LPR * 4 (and ALIGNED), so no chunk lies outside the row and the column masks fold away.
// X16: the row is int16 (8-byte aligned rows when ALIGNED).
// WIDE (X16, ALIGNED, NCH even, C % 8 == 0, 16-byte aligned x rows, 8-byte aligned y rows): a lane's chunks 2k and 2k+1
// are neighbours, eight columns that come in with one 16-byte load and leave with one 8-byte store.
template <int LPR, int NCH, bool ALIGNED, bool EMB = false, bool FULL = false, bool X16 = false, bool WIDE = false>
__global__ __launch_bounds__(LN_THREADS) void layernorm_rows_kernel(LayerNormArgs a)
{
    constexpr int ROWS_PER_BLOCK = LN_THREADS / LPR;
    static_assert(NCH * 4 <= 32, "a lane's sum of squares must stay below 2^35");
    static_assert(!WIDE || (X16 && ALIGNED && NCH % 2 == 0), "wide chunks: pairs of int16 chunks");
    const int lane = threadIdx.x % LPR;
    auto col_of = [&](int c) { return WIDE ? ((c >> 1) * LPR + lane) * 8 + (c & 1) * 4 : (c * LPR + lane) * 4; };
    const int64_t row = (int64_t)blockIdx.x * ROWS_PER_BLOCK + threadIdx.x / LPR;
    const bool live = row < a.rows;
    const int32_t C = a.C;
    const int32_t* xr = (EMB || X16) ? nullptr : a.x + (live ? row : 0) * a.ldx;
    const int16_t* xh = X16 ? reinterpret_cast<const int16_t*>(a.x) + (live ? row : 0) * a.ldx : nullptr;
    const int8_t *tr = nullptr, *pr = nullptr;
    if (EMB) {
        const int64_t r0 = live ? row : 0;
        int32_t id = a.emb.ids[r0];
        id = id < 0 ? 0 : (id >= a.emb.vocab ? a.emb.vocab - 1 : id);
        tr = a.emb.tok + (int64_t)id * C;
        pr = a.emb.pos + (r0 % a.emb.seq) * C;
    }
    const int32_t rnd = 1 << (a.shift - 1);

    int32_t v[NCH][4], gm[NCH][4], bt[NCH][4];
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int col = col_of(c);
        if (EMB) {
            int32_t tv[4], pv[4];
            if (ALIGNED) {
                const int cc = (FULL || col < C) ? col : 0;
                const uint32_t t4 = *reinterpret_cast<const uint32_t*>(tr + cc), p4 = *reinterpret_cast<const uint32_t*>(pr + cc);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    tv[e] = (int8_t)(t4 >> (8 * e));
                    pv[e] = (int8_t)(p4 >> (8 * e));
                }
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int ce = col + e < C ? col + e : 0;
                    tv[e] = tr[ce];
                    pv[e] = pr[ce];
                }
            }
            // the sum is taken in 64 bits and clamped once, as the definition has it
#pragma unroll
            for (int e = 0; e < 4; ++e)
                v[c][e] = clamp_i64_to_i32(dyadic64(tv[e], a.emb.tok_m, a.emb.tok_s) + dyadic64(pv[e], a.emb.pos_m, a.emb.pos_s), 32767);
        } else if (ALIGNED) {
            const int cc = (FULL || col < C) ? col : 0; // out-of-row chunks re-read chunk 0 and are masked below
            if (WIDE) {
                if ((c & 1) == 0) {
                    const int4 t = *reinterpret_cast<const int4*>(xh + cc);
                    v[c][0] = (int16_t)(t.x & 0xffff); v[c][1] = t.x >> 16; v[c][2] = (int16_t)(t.y & 0xffff); v[c][3] = t.y >> 16;
                    v[c + (NCH > 1 ? 1 : 0)][0] = (int16_t)(t.z & 0xffff); v[c + (NCH > 1 ? 1 : 0)][1] = t.z >> 16;
                    v[c + (NCH > 1 ? 1 : 0)][2] = (int16_t)(t.w & 0xffff); v[c + (NCH > 1 ? 1 : 0)][3] = t.w >> 16;
                }
            } else if (X16) {
                const int2 t = *reinterpret_cast<const int2*>(xh + cc);
                v[c][0] = (int16_t)(t.x & 0xffff); v[c][1] = t.x >> 16; v[c][2] = (int16_t)(t.y & 0xffff); v[c][3] = t.y >> 16;
            } else {
                const int4 t = *reinterpret_cast<const int4*>(xr + cc);
                v[c][0] = t.x; v[c][1] = t.y; v[c][2] = t.z; v[c][3] = t.w;
            }
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) v[c][e] = (live && col + e < C) ? (X16 ? (int32_t)xh[col + e] : xr[col + e]) : 0;
        }
    }
    // gamma and beta after the row itself, so that the row is the first thing in flight; every wavefront of a
    // compute unit reads the same few KB, which the vector cache serves after the first
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int col = col_of(c);
        if (ALIGNED) {
            const int cc = (FULL || col < C) ? col : 0;
            const int4 g4 = *reinterpret_cast<const int4*>(a.gamma_q + cc);
            const int4 b4 = *reinterpret_cast<const int4*>(a.beta_q + cc);
            gm[c][0] = g4.x; gm[c][1] = g4.y; gm[c][2] = g4.z; gm[c][3] = g4.w;
            bt[c][0] = b4.x + rnd; bt[c][1] = b4.y + rnd; bt[c][2] = b4.z + rnd; bt[c][3] = b4.w + rnd;
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int ce = col + e < C ? col + e : C - 1;
                gm[c][e] = a.gamma_q[ce];
                bt[c][e] = a.beta_q[ce] + rnd;
            }
        }
    }

    // clamp on load; the sum and the sum of squares in one sweep, so that their reductions overlap
    int32_t sum = 0;
    uint64_t sq = 0;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int col = col_of(c);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int32_t keep = (FULL || (ALIGNED ? col < C : col + e < C)) ? -1 : 0;
            v[c][e] = med3_i32(v[c][e], -32767, 32767) & keep;
            sum += v[c][e];                            // |sum| <= 1024 * 32767 < 2^25
            sq += (uint32_t)smul24(v[c][e], v[c][e]);  // |v| < 2^15: a 24-bit multiply; the total is below 2^40
        }
    }
    sum = group_sum_i32<LPR>(sum);
    sq = group_sum_u64<LPR>(sq);

    // mu = floor((sum + floor(C/2)) / C), computed on the non-negative number sum + C/2 + 32768 C
    const uint32_t Cu = (uint32_t)C;
    const int32_t mu = ln_row_mean(sum, Cu, a.magic_c);

    // sum of squared deviations from the two totals: sum (v - mu)^2 = sq - 2 mu sum + C mu^2, exact in 64 bits
    // (|2 mu sum| < 2^42, C mu^2 <= 2^40)
    const uint64_t ss = (uint64_t)((int64_t)sq - 2 * (int64_t)mu * sum + (int64_t)C * ((int64_t)mu * mu));

    const uint32_t var = ln_row_variance(ss, Cu, a.magic_c);
    const int32_t f = ln_factor_of_sigma(isqrt_floor_rowwise<LPR>(var, lane));
    if (!live) return;
    // d*f: |d| < 2^17 always; f < 2^23 unless sigma <= 2, where the full 32-bit multiply is used instead
    const bool f24 = __builtin_amdgcn_ballot_w64(f >= (1 << 23)) == 0;

    int8_t* yr = a.y + row * a.ldy;
    uint32_t even_pack = 0;                                    // WIDE: the packed bytes of the pair's first chunk
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int col = col_of(c);
        if (!FULL && col >= C) continue;
        int32_t o[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int32_t d = v[c][e] - mu;                                        // |d| < 2^17
            const int32_t n = (f24 ? smul24(d, f) : d * f) >> 14;                  // |d*f| < 2^30; |n| < 2^16
            const int32_t acc = smad24(n, gm[c][e], bt[c][e]);                     // |gamma_q| < 2^14: 24-bit multiply
            o[e] = med3_i32(acc >> a.shift, -127, 127);
        }
        if (WIDE) {
            const uint32_t pk = pack4_perm(o[0], o[1], o[2], o[3]);
            if ((c & 1) == 0) even_pack = pk;
            else *reinterpret_cast<uint2*>(yr + col - 4) = uint2{even_pack, pk};
        } else if (ALIGNED) {
            *reinterpret_cast<uint32_t*>(yr + col) = pack4_perm(o[0], o[1], o[2], o[3]);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (col + e < C) yr[col + e] = (int8_t)o[e];
        }
    }
}

// Alg. 4's integer square root on its own.  METHOD 0: a value per lane.  METHOD 1-3: the LPR = 64, 32, 16 lanes of a
// group take the group's values one after the other, all lanes working on one value, as the row kernel does with its
// one variance per row.
template <int METHOD>
__global__ __launch_bounds__(256) void isqrt_kernel(const uint32_t* n, uint32_t* root, int64_t count)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const uint32_t v = n[i < count ? i : count - 1];               // (every lane stays for the cross-lane rounds)
    uint32_t r;
    if (METHOD == 0) {
        r = isqrt_floor_lane(v);
    } else {
        constexpr int LPR = METHOD == 1 ? 64 : (METHOD == 2 ? 32 : 16);
        const int lane = threadIdx.x & 63, lir = lane % LPR, base = lane - lir;
        r = 0;
        for (int k = 0; k < LPR; ++k) {
            const uint32_t vk = (uint32_t)__shfl((int32_t)v, base + k, 64);
            const uint32_t rk = isqrt_floor_rowwise<LPR>(vk, lir);
            r = lir == k ? rk : r;
        }
    }
    if (i < count) root[i] = r;
}

int check_layernorm(int32_t C, int32_t shift)
{
    if (C < 1 || C > 1024) return IBERT_ERR_PARAM_RANGE;
    if (shift < 1 || shift > 30) return IBERT_ERR_PARAM_RANGE;
    return IBERT_OK;
}

template <int LPR, int NCH>
static void launch_rows(const LayerNormArgs& a, bool al, bool x16, bool wide, hipStream_t stream)
{
    constexpr int rpb = LN_THREADS / LPR;
    const dim3 grid((unsigned)((a.rows + rpb - 1) / rpb)), block(LN_THREADS);
    const bool full = al && a.C == NCH * LPR * 4;
#define IBERT_LN_LAUNCH(...) hipLaunchKernelGGL((layernorm_rows_kernel<LPR, NCH, __VA_ARGS__>), grid, block, 0, stream, a)
    if (a.emb.ids) {
        if (full) IBERT_LN_LAUNCH(true, true, true);
        else if (al) IBERT_LN_LAUNCH(true, true);
        else IBERT_LN_LAUNCH(false, true);
    } else if (x16) {
        if constexpr (NCH % 2 == 0) {
            if (wide && full) { IBERT_LN_LAUNCH(true, false, true, true, true); return; }
            if (wide) { IBERT_LN_LAUNCH(true, false, false, true, true); return; }
        }
        if (full) IBERT_LN_LAUNCH(true, false, true, true);
        else if (al) IBERT_LN_LAUNCH(true, false, false, true);
        else IBERT_LN_LAUNCH(false, false, false, true);
    } else if (full) IBERT_LN_LAUNCH(true, false, true);
    else if (al) IBERT_LN_LAUNCH(true);
    else IBERT_LN_LAUNCH(false);
#undef IBERT_LN_LAUNCH
}

static int dispatch_rows(const LayerNormArgs& a, bool al, bool x16, bool wide, hipStream_t stream)
{
    const int32_t C = a.C;
    // One wavefront per row (two rows for short ones): the per-row scalar work (mean, variance, square root,
    // reciprocal) is repeated by every lane of a row, but few registers per lane let many rows be in flight on a
    // compute unit, which is what hides the memory latency; shorter groups measured slower at every size.
    // int16 rows with wide chunks: the same bytes per lane (two rows per wavefront up to 768 columns).
    if (x16 && wide) {
        if (C <= 256) launch_rows<32, 2>(a, al, x16, true, stream);
        else if (C <= 512) launch_rows<64, 2>(a, al, x16, true, stream);
        else if (C <= 768) launch_rows<32, 6>(a, al, x16, true, stream);
        else launch_rows<64, 4>(a, al, x16, true, stream);
    } else if (C <= 256) launch_rows<32, 2>(a, al, x16, false, stream);
    else if (C <= 512) launch_rows<64, 2>(a, al, x16, false, stream);
    else if (C <= 768) launch_rows<64, 3>(a, al, x16, false, stream);
    else launch_rows<64, 4>(a, al, x16, false, stream);
    IBERT_LAUNCH_CHECK("layernorm kernel");
    g_last_kernel = a.emb.ids ? "layernorm_rows_kernel<embedding>" : "layernorm_rows_kernel";
    return IBERT_OK;
}

int launch_layernorm(const int32_t* x, int8_t* y, int64_t rows, int32_t C, int64_t ldx, int64_t ldy,
                     const int32_t* gamma_q, const int32_t* beta_q, int32_t shift, hipStream_t stream)
{
    if (rows == 0) return IBERT_OK;
    if (rows > 0x7fffffffLL) return IBERT_ERR_SHAPE;
    LayerNormArgs a{x, y, rows, C, ldx, ldy, gamma_q, beta_q, shift, ln_magic_for(C), EmbedArgs{}};
    const bool al = aligned(x, 16) && ldx % 4 == 0 && aligned(y, 4) && ldy % 4 == 0 && C % 4 == 0 &&
                    aligned(gamma_q, 16) && aligned(beta_q, 16);
    return dispatch_rows(a, al, false, false, stream);
}

// The same on int16 rows (the 16-bit form the MatMul can store its clamped LayerNorm input in).
int launch_layernorm16(const int16_t* x, int8_t* y, int64_t rows, int32_t C, int64_t ldx, int64_t ldy,
                       const int32_t* gamma_q, const int32_t* beta_q, int32_t shift, hipStream_t stream)
{
    if (rows == 0) return IBERT_OK;
    if (rows > 0x7fffffffLL) return IBERT_ERR_SHAPE;
    LayerNormArgs a{reinterpret_cast<const int32_t*>(x), y, rows, C, ldx, ldy, gamma_q, beta_q, shift, ln_magic_for(C), EmbedArgs{}};
    const bool al = aligned(x, 8) && ldx % 4 == 0 && aligned(y, 4) && ldy % 4 == 0 && C % 4 == 0 &&
                    aligned(gamma_q, 16) && aligned(beta_q, 16);
    // (wide chunks pay from about 8192 rows on: [32768,768] 19.3 -> 17.2 us; a few hundred rows lose half a microsecond)
    const bool wide = rows >= 8192 && al && aligned(x, 16) && ldx % 8 == 0 && aligned(y, 8) && ldy % 8 == 0 && C % 8 == 0;
    return dispatch_rows(a, al, true, wide, stream);
}

int launch_embedding(const int32_t* ids, const int8_t* tok, const int8_t* pos, int64_t tokens, int32_t seq, int32_t C,
                     int32_t vocab, ibert_dyadic tok_dy, ibert_dyadic pos_dy, const int32_t* gamma_q,
                     const int32_t* beta_q, int32_t shift, int8_t* y, int64_t ldy, hipStream_t stream)
{
    if (tokens == 0) return IBERT_OK;
    if (tokens > 0x7fffffffLL) return IBERT_ERR_SHAPE;
    LayerNormArgs a{nullptr, y, tokens, C, 0, ldy, gamma_q, beta_q, shift, ln_magic_for(C),
                    EmbedArgs{ids, tok, pos, seq, vocab, tok_dy.m, tok_dy.s, pos_dy.m, pos_dy.s}};
    const bool al = aligned(tok, 4) && aligned(pos, 4) && aligned(y, 4) && ldy % 4 == 0 && C % 4 == 0 &&
                    aligned(gamma_q, 16) && aligned(beta_q, 16);
    return dispatch_rows(a, al, false, false, stream);
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

extern "C" int ibert_isqrt_i(const uint32_t* n, uint32_t* root, int64_t count, int32_t method, void* stream_)
{
    using namespace ibert;
    if (count < 0) return IBERT_ERR_SHAPE;
    if (method < 0 || method > 3) return IBERT_ERR_PARAM_RANGE;
    if (count == 0) return IBERT_OK;
    if (!n || !root) return IBERT_ERR_NULL;
    const int64_t blocks = (count + 255) / 256;
    if (blocks > 0x7fffffffLL) return IBERT_ERR_SHAPE;
    hipStream_t stream = (hipStream_t)stream_;
    const dim3 grid((unsigned)blocks), block(256);
    switch (method) {
        case 0: hipLaunchKernelGGL(isqrt_kernel<0>, grid, block, 0, stream, n, root, count); break;
        case 1: hipLaunchKernelGGL(isqrt_kernel<1>, grid, block, 0, stream, n, root, count); break;
        case 2: hipLaunchKernelGGL(isqrt_kernel<2>, grid, block, 0, stream, n, root, count); break;
        default: hipLaunchKernelGGL(isqrt_kernel<3>, grid, block, 0, stream, n, root, count); break;
    }
    IBERT_LAUNCH_CHECK("isqrt_kernel");
    return IBERT_OK;
}

extern "C" int ibert_layernorm_i16(const int16_t* x, int8_t* y, int64_t rows, int32_t C, int64_t ldx, int64_t ldy,
                                   const int32_t* gamma_q, const int32_t* beta_q, int32_t shift, void* stream)
{
    if (rows < 0 || C < 1 || ldx < C || ldy < C) return IBERT_ERR_SHAPE;
    const int rc = ibert::check_layernorm(C, shift);
    if (rc) return rc;
    if (rows == 0) return IBERT_OK;
    if (!x || !y || !gamma_q || !beta_q) return IBERT_ERR_NULL;
    return ibert::launch_layernorm16(x, y, rows, C, ldx, ldy, gamma_q, beta_q, shift, (hipStream_t)stream);
}

extern "C" int ibert_embedding_i(const int32_t* ids, const int8_t* tok, const int8_t* pos, int64_t tokens, int32_t seq,
                                 int32_t hidden, int32_t vocab, int32_t max_pos, const ibert_dyadic* tok_dy,
                                 const ibert_dyadic* pos_dy, const int32_t* gamma_q, const int32_t* beta_q,
                                 int32_t ln_shift, int8_t* y, int64_t ldy, void* stream)
{
    if (!tok_dy || !pos_dy) return IBERT_ERR_NULL;
    if (tokens < 0 || seq < 1 || hidden < 1 || vocab < 1 || max_pos < seq || ldy < hidden) return IBERT_ERR_SHAPE;
    if (!ibert::dyadic_ok(*tok_dy) || !ibert::dyadic_ok(*pos_dy)) return IBERT_ERR_PARAM_RANGE;
    const int rc = ibert::check_layernorm(hidden, ln_shift);
    if (rc) return rc;
    if (tokens == 0) return IBERT_OK;
    if (!ids || !tok || !pos || !gamma_q || !beta_q || !y) return IBERT_ERR_NULL;
    return ibert::launch_embedding(ids, tok, pos, tokens, seq, hidden, vocab, *tok_dy, *pos_dy, gamma_q, beta_q, ln_shift, y,
                                   ldy, (hipStream_t)stream);
}
