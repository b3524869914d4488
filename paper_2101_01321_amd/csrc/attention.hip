// Self-attention core of one encoder layer in one kernel: scores = DY(Q_h K_h^T), integer Softmax over the
// keys (Alg. 3; Eq. 11-14), context = clamp(DY(P V_h)) -- steps 2, 3 and 4 of the layer (Fig. 1 right;
// Sec. 4.1), bit-identical to running them one after the other.  The INT32 scores and the INT8
// probabilities never leave the CU.
//
// Shape: head width 64, sequence length L = 128, 256, 384 or 512 (a whole score row, L/4 values per lane, stays in
// registers; the integer exponent cannot be rescaled exactly, so the row maximum must be known before the first
// exponent is taken).  One workgroup of four wavefronts owns 64 queries of one (batch, head); a wavefront owns 16.
//   * K_h (L x 64) and the 64 Q_h rows go to LDS row-major (64-byte rows, chunk index swizzled by the row);
//     V_h goes to LDS transposed, one L-byte row per output channel, with the keys of a row ordered so that a
//     lane's MFMA operand (16 keys) is one 16-byte read -- see `vt_offset`.
//   * Scores: L/16 MFMAs (16x16x64) per wavefront; lane l then holds, for query l%16, the L/4 keys
//     {16 i + 4 (l/16) + r}.  Row maximum and row sum finish with two cross-lane steps over the four lanes
//     that share a query.
//   * The probabilities are packed four to a dword as they are produced; the four dwords i = 4kb..4kb+3 are
//     exactly the lane's MFMA operand for key block kb under the key order above, so P never moves.
//   * Context: L/16 MFMAs per wavefront, requantized and stored as 4 bytes per lane.
//   * Padded sequences: the keys from key_lens[b] on take the logit INT32_MIN before the row maximum is taken (the
//     paper does not treat padding; this is the integer form of adding minus infinity to a masked logit).
#include "common.h"
#include "softmax_math.h"

namespace ibert {

typedef int v4i __attribute__((ext_vector_type(4)));

struct AttentionArgs {
    const int8_t* qkv;     // [batch*seq, 3*hidden]: Q | K | V, heads side by side
    int8_t* ctx;           // [batch*seq, hidden]
    int32_t heads;
    int32_t xcd_chunk;     // workgroups per XCD when the grid divides by 8, else 0
    int64_t ld_qkv, ld_ctx;
    int32_t s_m, s_s;      // scores requantization
    int32_t c_m, c_s;      // context requantization
    SoftmaxConst sm;
    const int32_t* key_lens;   // optional [batch]: sequence b attends to its first key_lens[b] keys only
};

constexpr int ATT_DH = 64, ATT_QB = 64, ATT_THREADS = 256;

// LDS byte offset inside the transposed V tile of (channel c, key n): row c (L bytes), 16-byte chunk
// (n/64)*4 + (n%16)/4 swizzled by c, byte 4*((n%64)/16) + n%4 inside the chunk.
template <int L>
__device__ __forceinline__ int vt_offset(int c, int n)
{
    const int kb = n >> 6, ip = (n >> 4) & 3, q = (n >> 2) & 3, r = n & 3;
    return c * L + ((((kb << 2) | q) ^ (c & 7)) << 4) + (ip << 2) + r;
}

__device__ __forceinline__ int swz64(int row) { return (row >> 1) & 3; }      // chunk swizzle of 64-byte rows

// DY(x; m, s) for |x| < 2^b when b <= s <= 62 (b <= 23): x m + 2^(s-1) fits 63 bits and the result fits 32 (it is
// below 2^(b+31-s)), so the floor-division by 2^s is bits [s, s+32) of the 64-bit sum: the high dword shifted by
// s - 32, or for s < 32 a funnel shift of the two dwords.  rnd = 2^(s-1).
// FORM 1: the shift is known to be at least 32 (a scale ratio below 1/2), FORM 2: known to be below 32 -- only that
// form is computed, two instructions a value; FORM 0: both and a select.
template <int FORM>
__device__ __forceinline__ int32_t dyadic_hi(int32_t x, int32_t m, int64_t rnd, int32_t sh)
{
    const int64_t p = (int64_t)x * m + rnd;
    const int32_t hi = (int32_t)(p >> 32);
    const int32_t a = hi >> ((sh - 32) & 31);
    if (FORM == 1) return a;
    const int32_t b = (int32_t)__builtin_amdgcn_alignbit((uint32_t)hi, (uint32_t)p, (uint32_t)(sh & 31));
    if (FORM == 2) return b;
    return sh >= 32 ? a : b;
}

// FAST: the 24-bit Softmax forms apply.  RQ: the scores shift is in [21, 62] and the context shift in [23, 62]
// (accumulators: 64 products of INT8 pairs, below 2^21; up to 512 products of a probability and an INT8 value,
// below 2^23), so dyadic_hi applies; |scores| then stays below 2^31 and needs no clamp.  RQ = 2 .. 5 say in addition on
// which side of 32 each shift lies: RQ - 2 = (scores shift >= 32) + 2 (context shift >= 32).
template <int NKB, bool FAST, int RQ>                     // NKB: key blocks of 64 (L = 64 NKB)
__global__ __launch_bounds__(ATT_THREADS) void attention_kernel(AttentionArgs a)
{
    constexpr int ATT_L = 64 * NKB, QBLKS = ATT_L / ATT_QB, NI = ATT_L / 16;
    constexpr int S_FORM = RQ < 2 ? 0 : (((RQ - 2) & 1) ? 1 : 2), C_FORM = RQ < 2 ? 0 : (((RQ - 2) & 2) ? 1 : 2);
    extern __shared__ __attribute__((aligned(16))) int8_t att_lds[];
    int8_t* const ks = att_lds;                                               // K_h, row-major [L][64]
    int8_t* const qs = att_lds + ATT_L * ATT_DH;                              // the block's queries [64][64]
    int8_t* const vt = qs + ATT_QB * ATT_DH;                                  // V_h transposed [64][L]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // Workgroups are dealt round-robin to the 8 XCDs.  The two halves of a head's queries read the same K and V,
    // and neighbouring heads share 128-byte lines of the packed QKV rows: give each XCD a contiguous run of
    // (batch, head, half) so that those re-reads hit its own L2.
    int bid = blockIdx.x;
    if (a.xcd_chunk > 0) bid = (bid & 7) * a.xcd_chunk + (bid >> 3);
    const int qblk = bid % QBLKS;                          // which 64 of the queries
    const int bh = bid / QBLKS;
    const int b = bh / a.heads, h = bh - b * a.heads;
    const int hidden = a.heads * ATT_DH;
    const int8_t* base = a.qkv + (int64_t)b * ATT_L * a.ld_qkv + h * ATT_DH;

    // ---- global -> LDS -------------------------------------------------------------------------
    {
        const int row = tid >> 2, ch = tid & 3;            // 64 rows x 4 chunks of 16 bytes per pass
        const v4i q0 = *reinterpret_cast<const v4i*>(base + (int64_t)(qblk * ATT_QB + row) * a.ld_qkv + ch * 16);
        v4i kk[NKB];
#pragma unroll
        for (int p = 0; p < NKB; ++p)
            kk[p] = *reinterpret_cast<const v4i*>(base + hidden + (int64_t)(row + 64 * p) * a.ld_qkv + ch * 16);
        *reinterpret_cast<v4i*>(qs + row * 64 + ((ch ^ swz64(row)) << 4)) = q0;
#pragma unroll
        for (int p = 0; p < NKB; ++p)
            *reinterpret_cast<v4i*>(ks + (row + 64 * p) * 64 + ((ch ^ swz64(row + 64 * p)) << 4)) = kk[p];
        // V: 4 keys x 4 channels per item, 4 L items, L/64 per lane (two at a time); item t: key group t/16, channel quad t%16
#pragma unroll
        for (int u0 = 0; u0 < NKB; u0 += 2) {
            uint32_t vv[2][4];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int t = (u0 + u) * ATT_THREADS + tid;
                const int g = t >> 4, cq = t & 15;
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    vv[u][r] = *reinterpret_cast<const uint32_t*>(base + 2 * hidden + (int64_t)(4 * g + r) * a.ld_qkv + 4 * cq);
            }
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int t = (u0 + u) * ATT_THREADS + tid;
                const int g = t >> 4, cq = t & 15;
                // 4x4 byte transpose: x01/y01 interleave rows 0,1; x23/y23 rows 2,3; tt[e] = bytes (r = 0..3) of channel e
                const uint32_t x01 = __builtin_amdgcn_perm(vv[u][1], vv[u][0], 0x05010400u);
                const uint32_t y01 = __builtin_amdgcn_perm(vv[u][1], vv[u][0], 0x07030602u);
                const uint32_t x23 = __builtin_amdgcn_perm(vv[u][3], vv[u][2], 0x05010400u);
                const uint32_t y23 = __builtin_amdgcn_perm(vv[u][3], vv[u][2], 0x07030602u);
                uint32_t tt[4];
                tt[0] = __builtin_amdgcn_perm(x23, x01, 0x05040100u);
                tt[1] = __builtin_amdgcn_perm(x23, x01, 0x07060302u);
                tt[2] = __builtin_amdgcn_perm(y23, y01, 0x05040100u);
                tt[3] = __builtin_amdgcn_perm(y23, y01, 0x07060302u);
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    *reinterpret_cast<uint32_t*>(vt + vt_offset<ATT_L>(4 * cq + e, 4 * g)) = tt[e];
            }
        }
    }
    __syncthreads();

    // ---- scores --------------------------------------------------------------------------------
    const int frow = lane & 15, fch = lane >> 4;
    const int qrow = wave * 16 + frow;                     // query row inside the block
    const v4i qf = *reinterpret_cast<const v4i*>(qs + qrow * 64 + ((fch ^ swz64(qrow)) << 4));
    const int64_t s_rnd = (int64_t)1 << ((a.s_s - 1) & 63), c_rnd = (int64_t)1 << ((a.c_s - 1) & 63);
    int32_t sc[NI][4];                                     // sc[i][r]: key 16 i + 4 fch + r
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int krow = 16 * i + frow;
        const v4i kf = *reinterpret_cast<const v4i*>(ks + krow * 64 + ((fch ^ swz64(krow)) << 4));
        const v4i acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(kf, qf, v4i{0, 0, 0, 0}, 0, 0, 0);
#pragma unroll
        for (int r = 0; r < 4; ++r)
            sc[i][r] = RQ ? dyadic_hi<S_FORM>(acc[r], a.s_m, s_rnd, a.s_s) : clamp_i64_to_i32(dyadic64(acc[r], a.s_m, a.s_s), 2147483647);
    }
    if (a.key_lens) {                                      // uniform over the workgroup
        int32_t nk = a.key_lens[b];
        nk = nk < 1 ? 1 : nk;
        if (nk < ATT_L) {
#pragma unroll
            for (int i = 0; i < NI; ++i)
#pragma unroll
                for (int r = 0; r < 4; ++r) sc[i][r] = 16 * i + 4 * fch + r < nk ? sc[i][r] : INT32_MIN;
        }
    }

    // ---- softmax over the L keys of the lane's query (four lanes share a query) ---------------
    int32_t mx = sc[0][0];
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) mx = sc[i][r] > mx ? sc[i][r] : mx;
    {
        const int32_t o1 = __shfl_xor(mx, 16, 64);
        mx = o1 > mx ? o1 : mx;
        const int32_t o2 = __shfl_xor(mx, 32, 64);
        mx = o2 > mx ? o2 : mx;
    }
    uint32_t ex[NI][4];
    uint32_t sum = 0;
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const uint32_t d = (uint32_t)mx - (uint32_t)sc[i][r];
            ex[i][r] = FAST ? iexp_from_diff_fast(d, a.sm) : iexp_from_diff(d, a.sm);
            sum += ex[i][r];
        }
    sum += (uint32_t)__shfl_xor((int32_t)sum, 16, 64);
    sum += (uint32_t)__shfl_xor((int32_t)sum, 32, 64);
    const uint32_t Fz = 0x80000000u / sum;                 // sum >= q_b^2 + q_c >= 1 (the maximum itself)

    v4i pf[NKB];                                           // probabilities as MFMA operands, one per key block
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        uint32_t o[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            // FAST: e < 2^24 and Fz <= 2^23 (sum >= q_b^2 + q_c >= 2^8), so the 24-bit multiply is exact
            o[r] = FAST ? umad24(ex[i][r], Fz, 1u << (30 - a.sm.k)) >> (31 - a.sm.k) : normalise(ex[i][r], Fz, a.sm.k);
            o[r] = o[r] > 127u ? 127u : o[r];
        }
        pf[i >> 2][i & 3] = (int32_t)(o[0] | (o[1] << 8) | (o[2] << 16) | (o[3] << 24));
    }

    // ---- context -------------------------------------------------------------------------------
    int8_t* out = a.ctx + (int64_t)(b * ATT_L + qblk * ATT_QB + qrow) * a.ld_ctx + h * ATT_DH + 4 * fch;
#pragma unroll
    for (int cb = 0; cb < 4; ++cb) {
        const int c = 16 * cb + frow;
        v4i acc = {0, 0, 0, 0};
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb) {
            const v4i vf = *reinterpret_cast<const v4i*>(vt + c * ATT_L + ((((kb << 2) | fch) ^ (c & 7)) << 4));
            acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(vf, pf[kb], acc, 0, 0, 0);
        }
        int32_t o[4];
#pragma unroll
        for (int r = 0; r < 4; ++r)
            o[r] = RQ ? med3_i32(dyadic_hi<C_FORM>(acc[r], a.c_m, c_rnd, a.c_s), -127, 127) : clamp_i64_to_i32(dyadic64(acc[r], a.c_m, a.c_s), 127);
        *reinterpret_cast<uint32_t*>(out + 16 * cb) = pack4_i8(o[0], o[1], o[2], o[3]);
    }
}

// Is the one-kernel form available for this shape and these pointers?
bool attention_fused_ok(const int8_t* qkv, const int8_t* ctx, int32_t seq, int32_t hidden, int32_t heads)
{
    return (seq == 128 || seq == 256 || seq == 384 || seq == 512) && heads >= 1 && hidden == heads * ATT_DH &&
           aligned(qkv, 16) && aligned(ctx, 4);
}

template <int NKB>
static int launch_attention_l(const AttentionArgs& a, int64_t blocks, bool fast, int rq, hipStream_t stream)
{
    constexpr int L = 64 * NKB;
    constexpr size_t lds_bytes = (size_t)L * ATT_DH + ATT_QB * ATT_DH + (size_t)ATT_DH * L;
    const dim3 grid((unsigned)blocks), block(ATT_THREADS);
#define IBERT_ATT_LAUNCH(F_, R_)                                                                                  \
    do {                                                                                                          \
        auto kern = attention_kernel<NKB, F_, R_>;                                                                \
        static bool attr_done = false;                                                                            \
        if (!attr_done && lds_bytes > 65536) {                                                                    \
            IBERT_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                              \
                                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes));     \
            attr_done = true;                                                                                     \
        }                                                                                                         \
        hipLaunchKernelGGL(kern, grid, block, lds_bytes, stream, a);                                              \
    } while (0)
    if (fast) {
        switch (rq) {
            case 0: IBERT_ATT_LAUNCH(true, 0); break;
            case 2: IBERT_ATT_LAUNCH(true, 2); break;
            case 3: IBERT_ATT_LAUNCH(true, 3); break;
            case 4: IBERT_ATT_LAUNCH(true, 4); break;
            default: IBERT_ATT_LAUNCH(true, 5); break;
        }
    } else {
        if (rq) IBERT_ATT_LAUNCH(false, 1); else IBERT_ATT_LAUNCH(false, 0);      // (the general Softmax forms dominate there)
    }
#undef IBERT_ATT_LAUNCH
    return IBERT_OK;
}

int launch_attention(const int8_t* qkv, int8_t* ctx, int32_t batch, int32_t seq, int32_t hidden, int32_t heads,
                     ibert_dyadic scores_dy, const ibert_softmax_params& sp, ibert_dyadic ctx_dy, hipStream_t stream,
                     const int32_t* key_lens)
{
    if (!attention_fused_ok(qkv, ctx, seq, hidden, heads)) return IBERT_ERR_NOT_IMPLEMENTED;
    const int64_t blocks = (int64_t)batch * heads * (seq / ATT_QB);
    if (blocks == 0) return IBERT_OK;
    if (blocks > 0x7fffffffLL) return IBERT_ERR_SHAPE;
    AttentionArgs a;
    a.qkv = qkv; a.ctx = ctx; a.heads = heads;
    a.xcd_chunk = blocks % 8 == 0 ? (int32_t)(blocks / 8) : 0;
    a.ld_qkv = 3 * (int64_t)hidden; a.ld_ctx = hidden;
    a.s_m = scores_dy.m; a.s_s = scores_dy.s; a.c_m = ctx_dy.m; a.c_s = ctx_dy.s;
    a.sm = softmax_const(sp);
    a.key_lens = key_lens;
    // register-only requantization: accumulators are below 64*127^2 (scores) and L*127*127 (context) < 2^23
    const int rq = (a.s_s >= 21 && a.s_s <= 62 && a.c_s >= 23 && a.c_s <= 62) ? 2 + (a.s_s >= 32 ? 1 : 0) + (a.c_s >= 32 ? 2 : 0) : 0;
    const bool fast = softmax_fast_ok(sp);
    int rc;
    switch (seq) {
        case 128: rc = launch_attention_l<2>(a, blocks, fast, rq, stream); break;
        case 256: rc = launch_attention_l<4>(a, blocks, fast, rq, stream); break;
        case 384: rc = launch_attention_l<6>(a, blocks, fast, rq, stream); break;
        default: rc = launch_attention_l<8>(a, blocks, fast, rq, stream); break;
    }
    if (rc) return rc;
    IBERT_LAUNCH_CHECK("attention_kernel");
    g_last_kernel = "attention_kernel";
    return IBERT_OK;
}

}  // namespace ibert
