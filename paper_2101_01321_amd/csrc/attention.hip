// Self-attention core of one encoder layer in one kernel: scores = DY(Q_h K_h^T), integer Softmax over the
// keys (Alg. 3; Eq. 11-14), context = clamp(DY(P V_h)) -- steps 2, 3 and 4 of the layer (Fig. 1 right;
// Sec. 4.1), bit-identical to running them one after the other.  The INT32 scores and the INT8
// probabilities never leave the CU.
//
// Shape: sequence length 128, head width 64 (RoBERTa-Base/Large at sequence length 128).  One workgroup of four
// wavefronts owns 64 queries of one (batch, head); a wavefront owns 16 queries.
//   * K_h (128 x 64) and the 64 Q_h rows go to LDS row-major (64-byte rows, chunk index swizzled by the row);
//     V_h goes to LDS transposed, one 128-byte row per output channel, with the keys of a row ordered so that a
//     lane's MFMA operand (16 keys) is one 16-byte read -- see `vt_offset`.
//   * Scores: 8 MFMAs (16x16x64) per wavefront; lane l then holds, for query l%16, the 32 keys
//     {16 i + 4 (l/16) + r}.  Row maximum and row sum finish with two cross-lane steps over the four lanes
//     that share a query.
//   * The probabilities are packed four to a dword as they are produced; the four dwords i = 4kb..4kb+3 are
//     exactly the lane's MFMA operand for key block kb under the key order above, so P never moves.
//   * Context: 8 MFMAs per wavefront, requantized and stored as 4 bytes per lane.
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
};

constexpr int ATT_L = 128, ATT_DH = 64, ATT_QB = 64, ATT_THREADS = 256;

// LDS byte offset inside the transposed V tile of (channel c, key n): row c (128 bytes), 16-byte chunk
// (n/64)*4 + (n%16)/4 swizzled by c, byte 4*((n%64)/16) + n%4 inside the chunk.
__device__ __forceinline__ int vt_offset(int c, int n)
{
    const int kb = n >> 6, ip = (n >> 4) & 3, q = (n >> 2) & 3, r = n & 3;
    return c * 128 + ((((kb << 2) | q) ^ (c & 7)) << 4) + (ip << 2) + r;
}

__device__ __forceinline__ int swz64(int row) { return (row >> 1) & 3; }      // chunk swizzle of 64-byte rows

// DY(x; m, s) for |x| < 2^21 when 21 <= s <= 62: x m + 2^(s-1) fits 63 bits and the result fits 32 (it is below
// 2^(52-s)), so the floor-division by 2^s is bits [s, s+32) of the 64-bit sum: the high dword shifted by s - 32, or
// for s < 32 a funnel shift of the two dwords.  rnd = 2^(s-1).
__device__ __forceinline__ int32_t dyadic_hi(int32_t x, int32_t m, int64_t rnd, int32_t sh)
{
    const int64_t p = (int64_t)x * m + rnd;
    const int32_t hi = (int32_t)(p >> 32);
    const int32_t a = hi >> ((sh - 32) & 31);
    const int32_t b = (int32_t)__builtin_amdgcn_alignbit((uint32_t)hi, (uint32_t)p, (uint32_t)(sh & 31));
    return sh >= 32 ? a : b;
}

// FAST: the 24-bit Softmax forms apply.  RQ: both requantization shifts are in [21, 62] (accumulators are below
// 2^21 in magnitude: 64 or 128 products of INT8 pairs), so dyadic_hi applies; |scores| then stays below 2^31 and
// needs no clamp.
template <bool FAST, bool RQ>
__global__ __launch_bounds__(ATT_THREADS) void attention_kernel(AttentionArgs a)
{
    __shared__ __attribute__((aligned(16))) int8_t ks[ATT_L * ATT_DH];        // K_h, row-major
    __shared__ __attribute__((aligned(16))) int8_t qs[ATT_QB * ATT_DH];       // the block's queries
    __shared__ __attribute__((aligned(16))) int8_t vt[ATT_DH * ATT_L];        // V_h transposed

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // Workgroups are dealt round-robin to the 8 XCDs.  The two halves of a head's queries read the same K and V,
    // and neighbouring heads share 128-byte lines of the packed QKV rows: give each XCD a contiguous run of
    // (batch, head, half) so that those re-reads hit its own L2.
    int bid = blockIdx.x;
    if (a.xcd_chunk > 0) bid = (bid & 7) * a.xcd_chunk + (bid >> 3);
    const int qblk = bid & 1;                              // which half of the queries
    const int bh = bid >> 1;
    const int b = bh / a.heads, h = bh - b * a.heads;
    const int hidden = a.heads * ATT_DH;
    const int8_t* base = a.qkv + (int64_t)b * ATT_L * a.ld_qkv + h * ATT_DH;

    // ---- global -> LDS -------------------------------------------------------------------------
    {
        const int row = tid >> 2, ch = tid & 3;            // 64 rows x 4 chunks of 16 bytes per pass
        const v4i q0 = *reinterpret_cast<const v4i*>(base + (int64_t)(qblk * ATT_QB + row) * a.ld_qkv + ch * 16);
        const v4i k0 = *reinterpret_cast<const v4i*>(base + hidden + (int64_t)row * a.ld_qkv + ch * 16);
        const v4i k1 = *reinterpret_cast<const v4i*>(base + hidden + (int64_t)(row + 64) * a.ld_qkv + ch * 16);
        // V: 4 keys x 4 channels per item, 512 items, two per lane; item t: key group t/16, channel quad t%16
        uint32_t vv[2][4];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int t = u * ATT_THREADS + tid;
            const int g = t >> 4, cq = t & 15;
#pragma unroll
            for (int r = 0; r < 4; ++r)
                vv[u][r] = *reinterpret_cast<const uint32_t*>(base + 2 * hidden + (int64_t)(4 * g + r) * a.ld_qkv + 4 * cq);
        }
        *reinterpret_cast<v4i*>(qs + row * 64 + ((ch ^ swz64(row)) << 4)) = q0;
        *reinterpret_cast<v4i*>(ks + row * 64 + ((ch ^ swz64(row)) << 4)) = k0;
        *reinterpret_cast<v4i*>(ks + (row + 64) * 64 + ((ch ^ swz64(row + 64)) << 4)) = k1;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int t = u * ATT_THREADS + tid;
            const int g = t >> 4, cq = t & 15;
            // 4x4 byte transpose: x01/y01 interleave rows 0,1; x23/y23 rows 2,3; t[e] = bytes (r = 0..3) of channel e
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
                *reinterpret_cast<uint32_t*>(vt + vt_offset(4 * cq + e, 4 * g)) = tt[e];
        }
    }
    __syncthreads();

    // ---- scores --------------------------------------------------------------------------------
    const int frow = lane & 15, fch = lane >> 4;
    const int qrow = wave * 16 + frow;                     // query row inside the block
    const v4i qf = *reinterpret_cast<const v4i*>(qs + qrow * 64 + ((fch ^ swz64(qrow)) << 4));
    const int64_t s_rnd = (int64_t)1 << ((a.s_s - 1) & 63), c_rnd = (int64_t)1 << ((a.c_s - 1) & 63);
    int32_t sc[8][4];                                      // sc[i][r]: key 16 i + 4 fch + r
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int krow = 16 * i + frow;
        const v4i kf = *reinterpret_cast<const v4i*>(ks + krow * 64 + ((fch ^ swz64(krow)) << 4));
        const v4i acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(kf, qf, v4i{0, 0, 0, 0}, 0, 0, 0);
#pragma unroll
        for (int r = 0; r < 4; ++r)
            sc[i][r] = RQ ? dyadic_hi(acc[r], a.s_m, s_rnd, a.s_s) : clamp_i64_to_i32(dyadic64(acc[r], a.s_m, a.s_s), 2147483647);
    }

    // ---- softmax over the 128 keys of the lane's query (four lanes share a query) ---------------
    int32_t mx = sc[0][0];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) mx = sc[i][r] > mx ? sc[i][r] : mx;
    {
        const int32_t o1 = __shfl_xor(mx, 16, 64);
        mx = o1 > mx ? o1 : mx;
        const int32_t o2 = __shfl_xor(mx, 32, 64);
        mx = o2 > mx ? o2 : mx;
    }
    uint32_t ex[8][4];
    uint32_t sum = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const uint32_t d = (uint32_t)mx - (uint32_t)sc[i][r];
            ex[i][r] = FAST ? iexp_from_diff_fast(d, a.sm) : iexp_from_diff(d, a.sm);
            sum += ex[i][r];
        }
    sum += (uint32_t)__shfl_xor((int32_t)sum, 16, 64);
    sum += (uint32_t)__shfl_xor((int32_t)sum, 32, 64);
    const uint32_t Fz = 0x80000000u / sum;                 // sum >= q_b^2 + q_c >= 1 (the maximum itself)

    v4i pf[2];                                             // probabilities as MFMA operands, one per key block
#pragma unroll
    for (int i = 0; i < 8; ++i) {
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
        for (int kb = 0; kb < 2; ++kb) {
            const v4i vf = *reinterpret_cast<const v4i*>(vt + c * 128 + ((((kb << 2) | fch) ^ (c & 7)) << 4));
            acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(vf, pf[kb], acc, 0, 0, 0);
        }
        int32_t o[4];
#pragma unroll
        for (int r = 0; r < 4; ++r)
            o[r] = RQ ? med3_i32(dyadic_hi(acc[r], a.c_m, c_rnd, a.c_s), -127, 127) : clamp_i64_to_i32(dyadic64(acc[r], a.c_m, a.c_s), 127);
        *reinterpret_cast<uint32_t*>(out + 16 * cb) = pack4_i8(o[0], o[1], o[2], o[3]);
    }
}

// Is the one-kernel form available for this shape and these pointers?
bool attention_fused_ok(const int8_t* qkv, const int8_t* ctx, int32_t seq, int32_t hidden, int32_t heads)
{
    return seq == ATT_L && heads >= 1 && hidden == heads * ATT_DH && aligned(qkv, 16) && aligned(ctx, 4);
}

int launch_attention(const int8_t* qkv, int8_t* ctx, int32_t batch, int32_t seq, int32_t hidden, int32_t heads,
                     ibert_dyadic scores_dy, const ibert_softmax_params& sp, ibert_dyadic ctx_dy, hipStream_t stream)
{
    if (!attention_fused_ok(qkv, ctx, seq, hidden, heads)) return IBERT_ERR_NOT_IMPLEMENTED;
    const int64_t blocks = (int64_t)batch * heads * (ATT_L / ATT_QB);
    if (blocks == 0) return IBERT_OK;
    if (blocks > 0x7fffffffLL) return IBERT_ERR_SHAPE;
    AttentionArgs a;
    a.qkv = qkv; a.ctx = ctx; a.heads = heads;
    a.xcd_chunk = blocks % 8 == 0 ? (int32_t)(blocks / 8) : 0;
    a.ld_qkv = 3 * (int64_t)hidden; a.ld_ctx = hidden;
    a.s_m = scores_dy.m; a.s_s = scores_dy.s; a.c_m = ctx_dy.m; a.c_s = ctx_dy.s;
    a.sm = softmax_const(sp);
    const bool rq = a.s_s >= 21 && a.s_s <= 62 && a.c_s >= 21 && a.c_s <= 62;
    const dim3 grid((unsigned)blocks), block(ATT_THREADS);
    if (softmax_fast_ok(sp)) {
        if (rq) hipLaunchKernelGGL((attention_kernel<true, true>), grid, block, 0, stream, a);
        else hipLaunchKernelGGL((attention_kernel<true, false>), grid, block, 0, stream, a);
    } else {
        if (rq) hipLaunchKernelGGL((attention_kernel<false, true>), grid, block, 0, stream, a);
        else hipLaunchKernelGGL((attention_kernel<false, false>), grid, block, 0, stream, a);
    }
    IBERT_LAUNCH_CHECK("attention_kernel");
    g_last_kernel = "attention_kernel";
    return IBERT_OK;
}

}  // namespace ibert
