// INT8 x INT8 -> INT32 MatMul (Sec. 1 third contribution, App. C.1) with bias, dyadic requantization,
// optional residual and clamp fused into the epilogue.
//
// Fast path (W is [N,K], rows 16-byte aligned): LDS-staged tiles feeding v_mfma_i32_16x16x64_i8.
//   * The weight rows are fed as the first MFMA operand and the activation rows as the second, so that
//     each lane ends up with four consecutive output channels n of one token m: the epilogue packs
//     them into one dword (INT8 out) or one 16-byte store (INT32 out).
//   * Both operands are K-contiguous in memory; a lane's MFMA operand is 16 consecutive K bytes, one
//     ds_read_b128.  LDS rows are BK bytes (64 or 128) with the 16-byte chunk index XOR-swizzled by the row
//     so that the rows a group of lanes reads in one cycle fall into distinct banks.
//   * Two tile loaders: global memory straight into LDS (whole tiles, K a multiple of 128), or through a ring
//     of registers (everything else that is 16-byte aligned, and W given as [K,N] with aligned rows).
//   * Integer accumulation is exact, so any consistent K order gives the oracle's bits.
//   * The epilogue can also apply integer GELU (Alg. 2) to its own INT8 output.
//   * Four wavefronts per workgroup, or eight (two per SIMD) for the big INT8 tiles.
// Generic path (unaligned operands): one output element per lane, byte loads.
#pragma once
#include <cstdio>
#include <type_traits>

#include "common.h"
#include "gelu_math.h"
#include "ibert_testing.h"

namespace ibert {

typedef int v4i __attribute__((ext_vector_type(4)));

struct GemmArgs {
    const int8_t* A;
    const int8_t* W;
    const int32_t* bias;
    const int32_t* mult;
    const int32_t* shift;
    const int8_t* R;
    void* C;
    int32_t M, N, K;
    int32_t batch_inner, nbatch;
    int32_t tiles_m, tiles_n;
    int64_t lda, ldw, ldc, ldr;
    int64_t sA_o, sA_i, sW_o, sW_i, sC_o, sC_i, sR_o, sR_i;
    int32_t per_channel;
    int32_t dy_m, dy_s;
    int32_t out_clamp;
    int32_t res_m, res_s;
    int32_t c_vec;     // output rows allow one vector store per lane (4 bytes INT8, 16 bytes INT32)
    int32_t r_vec;     // residual rows allow 16-byte loads
    int32_t c_vec16;   // INT8 output rows allow 16-byte stores
    int32_t c16;       // the INT32 kernels store 16-bit elements (IBERT_I16: |value| <= out_clamp <= 32767)
    int32_t res_fast;  // residual absent, or its shift is in [8, 62]: its requantized value fits 32 bits
    int64_t res_rnd;   // 2^(res_s - 1), or 0 when res_s == 0
    int32_t xcd_chunk; // tiles per XCD when the grid divides by 8, else 0 (no remap)
    int32_t xcd_xn;    // >= 1: each XCD works on a block of the tile grid, xcd_xn (a power of two) blocks side by side
    int32_t xcd_xs;    // log2(xcd_xn)
    int32_t xcd_bm, xcd_bn;   // tile rows and tile columns of such a block
    int32_t gelu_fast; // GELU epilogue: the 24-bit form applies
    int32_t gelu_lut_lo, gelu_lut_n;   // GELU epilogue: table of the values at lo .. lo + n - 1 behind the tile's LDS (n = 0: none)
    GeluConst gelu;    // GELU epilogue: constants (the clamp before it is out_clamp = q_max)
    uint32_t* path_word;   // tests only (may be null): workgroup 0 records which epilogue form it ran
};

// Requantize one accumulator and finish the output value (before the store).
__device__ __forceinline__ int32_t finish(int32_t acc, int32_t m, int32_t s, bool has_res, int32_t res,
                                          const GemmArgs& g)
{
    int64_t v = dyadic64(acc, m, s);
    if (has_res) v += dyadic64(res, g.res_m, g.res_s);
    return clamp_i64_to_i32(v, g.out_clamp);
}

// ---------------------------------------------------------------------------------------------
// MFMA kernel, W = [N,K].
//
// One workgroup = 4 wavefronts (2 x 2) computes a BM x BN tile; each wavefront owns (BM/2) x (BN/2),
// i.e. (BM/32) x (BN/32) MFMA blocks of 16x16, accumulators in registers.
// K is walked in steps of BK bytes.  Register-ring loader: global loads for step s are issued RING steps
// ahead into a ring of register slots; one step before use they are written to the other half of a
// double-buffered LDS tile; inside a step the operand fragments of the next 64-wide K slice are read from
// LDS while the MFMAs of the current slice issue.  The direct-to-LDS loader is described at the kernel.
// ---------------------------------------------------------------------------------------------
constexpr int GEMM_THREADS = 256;

// XOR swizzle of the 16-byte chunk index by the LDS row, so that the 16 rows whose same logical chunk the lanes
// of an operand read fetch (row stride = BK bytes) land on 16 distinct 16-byte bank groups of the 256-byte bank cycle:
// two 128-byte rows (or four 64-byte rows) share a bank cycle, so the chunk is XORed with row / 2 -- rows 2r and 2r+1
// sit in different halves of the cycle, and the eight values of row / 2 spread the rest.  (chunk ^ row, which repeats
// after eight rows, leaves rows r and r + 8 on the same banks: 106 B/clk measured on the LDS of this chip against 118
// for this one and 128 for a linear read.)  CPR = chunks per row.
template <int CPR>
__device__ __forceinline__ int swz(int row)
{
    if (CPR == 16) return row & 15;
    if (CPR == 8) return (row >> 1) & 7;
    return (row >> 1) & 3;
}

// One 16-byte chunk of a tile row.  p points at the chunk (column k of the row).
//   KMODE 0: K is a multiple of BK, every chunk is in range.
//   KMODE 1: K is a multiple of 16: a chunk at or past K is fetched from column K-16 instead (in range)
//            and replaced by zeros, without a branch.
//   KMODE 2: any K >= 1: the chunk that straddles K is assembled bytewise (slow, rare).
template <int KMODE>
__device__ __forceinline__ v4i load_chunk(const int8_t* p, int k, int K)
{
    if (KMODE == 0) return *reinterpret_cast<const v4i*>(p);
    if (KMODE == 1) {
        const bool in = k < K;
        const int back = in ? 0 : k - (K - 16);
        v4i r = *reinterpret_cast<const v4i*>(p - back);
        r.x = in ? r.x : 0; r.y = in ? r.y : 0; r.z = in ? r.z : 0; r.w = in ? r.w : 0;
        return r;
    }
    v4i r = {0, 0, 0, 0};
    if (k >= K) return r;
    if (k + 16 <= K) return *reinterpret_cast<const v4i*>(p);
    union { v4i v; int8_t b[16]; } u;
    u.v = r;
    for (int i = 0; i < 16; ++i)
        if (k + i < K) u.b[i] = p[i];
    return u.v;
}

// LDS layout of the epilogue: a staging tile of 32*JC rows (padded stride), the per-channel constants and the
// residual tile.  JC (MFMA block rows per chunk) is the largest power-of-two divisor of BM/32 that fits the
// budget: the main loop's own allocation for small tiles (several workgroups share a CU), up to 160 KB
// for big ones (one workgroup per CU anyway).
template <int BM, int BN, int BK, int NSTG = 2>
struct EpiLayout {
    static constexpr int SP = BN + 4;
    static constexpr int FM = BM / 32;
    static constexpr int FIXED = 3 * BN + BM * BN / 4;
    static constexpr int MAIN = NSTG * (BM + BN) * BK / 4;
    static constexpr int BUDGET = MAIN * 4 >= 65536 ? 40000 : MAIN;
    static constexpr int fit(int jc) { return 32 * jc * SP + FIXED <= BUDGET; }
    static constexpr int JC = fit(FM) ? FM : (FM >= 2 && fit(FM / 2) ? FM / 2 : (FM >= 4 && fit(FM / 4) ? FM / 4 : 1));
    static constexpr int EPI = 32 * JC * SP + FIXED;
    static constexpr int LDS_BYTES = 4 * (MAIN > EPI ? MAIN : EPI);
};

// TW = true: W is [K,N] (N contiguous).  Only the W loader differs: each lane fetches a 4 (k) x 4 (n) byte
// block as four dwords, transposes it in registers with byte permutes and writes four dwords (4 consecutive
// k of one n) into the same K-contiguous LDS layout the MFMA loop reads.
//
// DMA = true (whole tiles only, BK = 128): the tiles go from global memory straight into LDS
// (global_load_lds_dwordx4: lane l of a wavefront writes bytes [16 l, 16 l + 16) of a 1 KB LDS block, so a
// block is 8 tile rows and the lane fetches the chunk that the swizzle puts at its position).  No register
// ring and no LDS write instructions; a K step is two phases of MFMAs, each of which also issues the
// fragment reads of the next phase and (second phase) the loads of the step after next, one barrier per step.
// GELU = true (INT8 output): the requantized, clamped value is the GELU input; integer GELU (Alg. 2) and its
// requantization to INT8 are applied before the store, so the INT32 tensor between the two never exists.
// NLD > 0 (direct-to-LDS loader): NLD further wavefronts that only request tiles.  A wavefront whose request waits for
// the address unit issues nothing else, so requests issued between MFMAs cost the MFMA wavefronts time (without any tile
// request the loop of the 128x96 tile runs in three quarters of its time); a wavefront of their own takes that wait
// instead.  They join every barrier of the loop and end before the epilogue (a barrier waits for the surviving
// wavefronts only).
template <int BM, int BN, int BK, int RING, bool OUT_I8, int KMODE, bool TW = false, bool DMA = false, bool GELU = false,
          int NW = 4, int NLD = 0>
__global__ __launch_bounds__(64 * (NW + NLD)) void gemm_nt_mfma_kernel(GemmArgs g)
{
    // NW wavefronts in two rows of NW/2: wavefront w owns rows [(w%2) BM/2, +BM/2) and columns [(w/2) WN, +WN) of the tile.
    // (Eight wavefronts on a tile whose width does not divide into four strips of whole MFMA blocks -- 128x96 -- stand in
    // four rows of two instead: rows [(w%4) BM/4, +BM/4), columns [(w/4) BN/2, +BN/2).)
    // Eight (two per SIMD) pay for INT8 tiles of 256x192: the second wavefront hides what the first waits for in the loop
    // and in the packing epilogue (inside the encoder: S1 of Large 21.4 -> 19.9 us, S7+S8 of Base 20.6 -> 19.3 us).
    constexpr int NT = 64 * NW;
    static_assert(NW == 4 || (NW == 8 && DMA), "four wavefronts, or eight for the direct-to-LDS loader");
    static_assert(!GELU || OUT_I8, "the GELU epilogue writes INT8");
    static_assert(NLD == 0 || (NLD == 4 && DMA && !GELU), "loader wavefronts: four, direct-to-LDS tiles");
    constexpr int CPR = BK / 16;                       // 16-byte chunks per tile row
    constexpr int RPP = NT / CPR;            // tile rows loaded per pass of the workgroup
    constexpr int LA = BM / RPP, LW = BN / RPP;        // chunks per lane per K step
    constexpr bool R4 = NW == 8 && (BN / 4) % 16 != 0;  // four rows of two wavefronts
    constexpr int WR = R4 ? 4 : 2;                      // rows of wavefronts
    constexpr int WM = BM / WR, WN = BN / (NW / WR);    // wavefront tile
    constexpr int FM = WM / 16, FN = WN / 16;
    constexpr int NS = BK / 64;                        // 64-wide K slices per step
    static_assert((DMA || (BM % RPP == 0 && BN % RPP == 0)) && WM % 16 == 0 && WN % 16 == 0, "tile shape");
    static_assert(!TW || (BK / 4) * (BN / 4) == LW * NT, "transposing loader covers the W tile exactly");

    // The argument block spans five 64-byte lines of a scalar cache that is cold when a kernel starts, and the compiler
    // fetches each argument where it is first used, one dependent wait after the other -- each a trip to memory.  Touch
    // every line now, back to back, so that those later fetches hit.
    {
        static_assert(sizeof(GemmArgs) <= 384, "argument block: six lines at most");
#if defined(__HIP_DEVICE_COMPILE__)
        typedef const __attribute__((address_space(4))) uint32_t* kernarg_words;
        kernarg_words kp = (kernarg_words)__builtin_amdgcn_kernarg_segment_ptr();
        const uint32_t k0 = kp[0], k1 = kp[16], k2 = kp[32], k3 = kp[48], k4 = kp[64], k5 = kp[(sizeof(GemmArgs) - 4) / 4];
        asm volatile("" :: "s"(k0), "s"(k1), "s"(k2), "s"(k3), "s"(k4), "s"(k5));
        // ... and have what the start of the kernel needs in registers after one wait
        asm volatile("" :: "s"(g.A), "s"(g.W), "s"(g.bias), "s"(g.mult), "s"(g.shift), "s"(g.R), "s"(g.C), "s"(g.M), "s"(g.N),
                     "s"(g.K), "s"(g.nbatch), "s"(g.lda), "s"(g.ldw), "s"(g.xcd_xn), "s"(g.xcd_xs), "s"(g.xcd_bm), "s"(g.xcd_bn),
                     "s"(g.per_channel), "s"(g.gelu_lut_n), "s"(g.gelu_lut_lo));
#endif
    }
    extern __shared__ __attribute__((aligned(16))) int8_t lds[];
    constexpr int STAGE = (BM + BN) * BK;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave & (WR - 1)) * WM, wn0 = (wave / WR) * WN;

    // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous run of tiles so that
    // the A panels and W panels it touches stay in its own L2.
    // One problem whose tile grid divides suitably (xcd_xn >= 1, the launcher's choice): the run is a rectangular block
    // of the tile grid -- xcd_bm tile rows by xcd_bn tile columns, xcd_xn such blocks side by side, 8 / xcd_xn above each
    // other -- so that an XCD fetches only its rows of A and its columns of W over the fabric: 8 (M K / XM + N K / XN)
    // bytes in all, least for near-square blocks.  The launch grid is then (8 xcd_bn, xcd_bm): the XCD is blockIdx.x % 8
    // and the tile's place inside the block comes from the block indices without a division.
    int z, tm, tn;
    if (g.xcd_xn >= 1) {
        const int x = blockIdx.x & 7, ln = blockIdx.x >> 3, lm = blockIdx.y;
        const int xm = x >> g.xcd_xs, xn = x & (g.xcd_xn - 1);
        z = 0;
        tm = xm * g.xcd_bm + lm;
        tn = xn * g.xcd_bn + ln;
    } else {
        int bid = blockIdx.x;
        if (g.xcd_chunk > 0) bid = (bid & 7) * g.xcd_chunk + (bid >> 3);
        const int tiles = g.tiles_m * g.tiles_n;
        z = bid / tiles;
        bid -= z * tiles;
        tm = bid / g.tiles_n;
        tn = bid - tm * g.tiles_n;
    }
    const int m0 = tm * BM, n0 = tn * BN;
    const int zo = g.nbatch == 1 ? 0 : z / g.batch_inner, zi = z - zo * g.batch_inner;

    const int8_t* A = g.A + zo * g.sA_o + zi * g.sA_i;
    const int8_t* W = g.W + zo * g.sW_o + zi * g.sW_i;

    const int lrow = tid / CPR, lch = tid % CPR;
    // rows past the edge are clamped to the last valid row: they load real memory and are never stored
    const int8_t* pa[LA];
    const int8_t* pw[LW];
#pragma unroll
    for (int i = 0; i < LA; ++i) {
        const int row = m0 + i * RPP + lrow;
        pa[i] = A + (int64_t)(row < g.M ? row : g.M - 1) * g.lda + lch * 16;
    }
    // TW: block q = i*256 + tid of the BK x BN tile covers k in [4*kb4, 4*kb4+4), n in [4*nb4, 4*nb4+4)
    constexpr int NB4 = BN / 4;
    int tw_k[LW], tw_n[LW];
#pragma unroll
    for (int i = 0; i < LW; ++i) {
        if (TW) {
            const int q = i * NT + tid;
            tw_k[i] = (q / NB4) * 4;
            tw_n[i] = (q % NB4) * 4;
            const int ncol = n0 + tw_n[i];
            pw[i] = W + (ncol + 3 < g.N ? ncol : g.N - 4);        // N % 4 == 0, N >= 4: clamped columns are never stored
        } else {
            const int row = n0 + i * RPP + lrow;
            pw[i] = W + (int64_t)(row < g.N ? row : g.N - 1) * g.ldw + lch * 16;
        }
    }
    const int wr_off = lrow * BK + ((lch ^ swz<CPR>(lrow)) << 4);   // RPP is a multiple of 16: swizzle depends on lrow only

    v4i ring[RING][LA + LW];
    auto load_global = [&](int kt, int slot) {
        const int kb = kt * BK;
#pragma unroll
        for (int i = 0; i < LA; ++i) ring[slot][i] = load_chunk<KMODE>(pa[i] + kb, kb + lch * 16, g.K) ;
#pragma unroll
        for (int i = 0; i < LW; ++i) {
            if (TW) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int k = kb + tw_k[i] + r;
                    const int d = *reinterpret_cast<const int*>(pw[i] + (int64_t)(k < g.K ? k : g.K - 1) * g.ldw);
                    ring[slot][LA + i][r] = k < g.K ? d : 0;
                }
            } else {
                ring[slot][LA + i] = load_chunk<KMODE>(pw[i] + kb, kb + lch * 16, g.K);
            }
        }
    };
    auto store_lds = [&](int slot, int buf) {
        int8_t* base = lds + buf * STAGE + wr_off;
#pragma unroll
        for (int i = 0; i < LA; ++i) *reinterpret_cast<v4i*>(base + i * RPP * BK) = ring[slot][i];
#pragma unroll
        for (int i = 0; i < LW; ++i) {
            if (TW) {
                const v4i d = ring[slot][LA + i];
                const uint32_t x01 = __builtin_amdgcn_perm((uint32_t)d[1], (uint32_t)d[0], 0x05010400u);
                const uint32_t y01 = __builtin_amdgcn_perm((uint32_t)d[1], (uint32_t)d[0], 0x07030602u);
                const uint32_t x23 = __builtin_amdgcn_perm((uint32_t)d[3], (uint32_t)d[2], 0x05010400u);
                const uint32_t y23 = __builtin_amdgcn_perm((uint32_t)d[3], (uint32_t)d[2], 0x07030602u);
                uint32_t t[4];
                t[0] = __builtin_amdgcn_perm(x23, x01, 0x05040100u);
                t[1] = __builtin_amdgcn_perm(x23, x01, 0x07060302u);
                t[2] = __builtin_amdgcn_perm(y23, y01, 0x05040100u);
                t[3] = __builtin_amdgcn_perm(y23, y01, 0x07060302u);
                int8_t* wb = lds + buf * STAGE + BM * BK;
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const int nrow = tw_n[i] + c;
                    *reinterpret_cast<uint32_t*>(wb + nrow * BK + (((tw_k[i] >> 4) ^ swz<CPR>(nrow)) << 4) + (tw_k[i] & 15)) = t[c];
                }
            } else {
                *reinterpret_cast<v4i*>(base + BM * BK + i * RPP * BK) = ring[slot][LA + i];
            }
        }
    };

    v4i acc[FN][FM];
#pragma unroll
    for (int i = 0; i < FN; ++i)
#pragma unroll
        for (int j = 0; j < FM; ++j) acc[i][j] = v4i{0, 0, 0, 0};

    const int nk = (g.K + BK - 1) / BK;
    const int frow = lane & 15, fch = lane >> 4;       // MFMA operand: row within the 16-block, K chunk
    const int rd_swz = swz<CPR>(frow);                 // block rows are multiples of 16: depends on frow only
    const int rd_a = (wm0 + frow) * BK, rd_w = BM * BK + (wn0 + frow) * BK;

    auto read_frags = [&](int buf, int s, v4i (&xa)[FM], v4i (&wb)[FN]) {
        const int8_t* base = lds + buf * STAGE + (((s * 4 + fch) ^ rd_swz) << 4);
#pragma unroll
        for (int j = 0; j < FM; ++j) xa[j] = *reinterpret_cast<const v4i*>(base + rd_a + j * 16 * BK);
#pragma unroll
        for (int i = 0; i < FN; ++i) wb[i] = *reinterpret_cast<const v4i*>(base + rd_w + i * 16 * BK);
    };

    using EL = EpiLayout<BM, BN, BK, (DMA ? RING : 2)>;
    const int64_t c_off = zo * g.sC_o + zi * g.sC_i;
    const int8_t* R = g.R ? g.R + zo * g.sR_o + zi * g.sR_i : nullptr;
    const bool interior = m0 + BM <= g.M && n0 + BN <= g.N && g.c_vec && (!R || g.r_vec) && g.ldc < (1 << 22);

    // Per-channel constants of this tile's BN columns, one or two columns per lane; used after the main loop.
    // (register-ring kernels; the direct-to-LDS kernels fetch them straight into LDS, see below)
    constexpr int PPT = (BN + NT - 1) / NT;
    int32_t pb[PPT], pm[PPT], ps[PPT];
    if constexpr (!DMA) {
#pragma unroll
        for (int q = 0; q < PPT; ++q) {
            int nn = n0 + q * NT + tid;
            nn = nn < g.N ? nn : g.N - 1;
            pb[q] = 0; pm[q] = g.dy_m; ps[q] = g.dy_s;
            if (g.bias) pb[q] = g.bias[nn];
            if (g.per_channel) {
                pm[q] = g.mult[nn];
                ps[q] = g.shift[nn];
            }
        }
    }
    // Direct-to-LDS kernels with small tiles also fetch their residual tile now, 16 bytes per lane and round, and park
    // it in registers until the main loop is over (the tile's LDS home is inside the stages): after the loop it would
    // be a full trip to memory with nothing to hide it behind.  (Requested before the tile loads: loads complete in
    // order, and the waits of the main loop count the tile loads as the youngest.)
    constexpr int RCH = BM * BN / 16;                              // 16-byte chunks of the residual tile
    constexpr int RPRE = DMA && !OUT_I8 && RCH <= 6 * NT ? (RCH + NT - 1) / NT : 0;
    v4i rpre[RPRE > 0 ? RPRE : 1];
    const bool res_early = RPRE > 0 && R && interior;
    if (RPRE > 0 && res_early && (NLD == 0 || tid < NT)) {
#pragma unroll
        for (int u = 0; u < RPRE; ++u) {
            const int q = u * NT + tid;
            const int qq = q < RCH ? q : 0;
            const int row = qq / (BN / 16), c16 = qq - row * (BN / 16);
            rpre[u] = *reinterpret_cast<const v4i*>(R + (int64_t)(m0 + row) * g.ldr + n0 + c16 * 16);
        }
    }
    // (direct-to-LDS kernels: the constants live in LDS behind the stages, requested before the loop starts, see below)
    int32_t* const par_early = reinterpret_cast<int32_t*>(lds + EL::LDS_BYTES);
    constexpr int PAR_BYTES = (3 * BN * 4 + 255) & ~255;
    bool fast_early = false, fold_early = false;

    if constexpr (DMA) {
        // With eight wavefronts (two per SIMD) only the first four request tiles: a wavefront whose request waits for the
        // address unit issues nothing else meanwhile, and when both wavefronts of a SIMD ask in the same phase (they run
        // in step, from barrier to barrier) its MFMA pipe idles -- a phase with requests took twice the time of one
        // without.  This way the second wavefront of each SIMD keeps the pipe busy while the first one asks.
        constexpr int ND = NLD > 0 ? NLD : (NW == 8 ? 4 : NW);        // wavefronts that request tiles
        constexpr int RG = 8 * ND;                                    // tile rows they fetch together

        static_assert(BK == 128 && !TW && KMODE == 0 && BM % RG == 0 && BN % RG == 0, "DMA loader: whole 1 KB blocks");
        constexpr int NLA = BM / RG, NLW = BN / RG, NL = NLA + NLW;   // 1 KB blocks per wavefront and step
        constexpr int NMF = FM * FN, NR = FM + FN;
        constexpr int SPC = NMF / NR > 0 ? NMF / NR : 1;              // MFMAs between two fragment reads
        static_assert(NL <= 2 * NR && (NMF + SPC - 1) / SPC >= NR, "one read and at most two loads per slot");
        static_assert(RG % 32 == 0, "the swizzle of a lane's row must not depend on the block");
        const int wave_u = __builtin_amdgcn_readfirstlane(wave);
        const bool loader = NLD > 0 && wave_u >= NW;                  // (uniform: scalar branches, not exec masks)
        const int wv = NLD > 0 ? (loader ? wave_u - NW : wave_u) : wave_u;   // index among the requesting wavefronts
        const bool asker = NLD > 0 ? loader : wv < ND;
        const int lr8 = lane >> 3, lp = lane & 7;
        // swz<8> of the lane's row: the row is RG i + 8 wave + lr8 with RG a multiple of 32, so (row >> 1) & 7 depends on
        // the wavefront's parity and the lane only
        const int lsw = ((wv & 1) << 2) | (lr8 >> 1);
        const uint32_t voff_a = (uint32_t)lr8 * (uint32_t)g.lda + (uint32_t)((lp ^ lsw) << 4);
        const uint32_t voff_w = (uint32_t)lr8 * (uint32_t)g.ldw + (uint32_t)((lp ^ lsw) << 4);
        const int8_t* ga = A + (int64_t)(m0 + wv * 8) * g.lda;
        const int8_t* gw = W + (int64_t)(n0 + wv * 8) * g.ldw;
        const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) int8_t*)lds + (uint32_t)wv * 1024u;

        // block q of the step: rows [RG i + 8 wave, +8) of A (q < NLA) or of W
        auto dma_one = [&](int q, int kt, int buf) {
            const bool is_a = q < NLA;
            const int i = is_a ? q : q - NLA;
            const int8_t* sb = (is_a ? ga + (int64_t)i * RG * g.lda : gw + (int64_t)i * RG * g.ldw) + (int64_t)kt * BK;
            const uint32_t la = lds0 + (uint32_t)(buf * STAGE + (is_a ? 0 : BM * BK) + i * (RG * BK));
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                         :: "s"(la), "v"(is_a ? voff_a : voff_w), "s"(sb) : "memory", "m0");
        };
        auto read_one = [&](int q, int buf, int s, v4i (&xa)[FM], v4i (&wb)[FN]) {
            const int8_t* base = lds + buf * STAGE + (((s * 4 + fch) ^ rd_swz) << 4);
            if (q < FM) xa[q] = *reinterpret_cast<const v4i*>(base + rd_a + q * 16 * BK);
            else wb[q - FM] = *reinterpret_cast<const v4i*>(base + rd_w + (q - FM) * 16 * BK);
        };
        // One phase: the MFMAs of one 64-wide K slice (operands xa, wb); every SPC MFMAs one fragment of
        // the next phase is read (into nxa, nwb) and one block of a later step is requested.
        // The blocks requested are [Q0, Q1) of step dkt (if dm), one per slot.
        auto phase = [&](v4i (&xa)[FM], v4i (&wb)[FN], v4i (&nxa)[FM], v4i (&nwb)[FN], int rbuf, int rs,
                         auto read_tag, int dkt, int dbuf, bool dm, auto q0_tag, auto q1_tag) {
            constexpr bool RD = decltype(read_tag)::value;
            constexpr int Q0 = decltype(q0_tag)::value, Q1 = decltype(q1_tag)::value;
#pragma unroll
            for (int i = 0; i < FN; ++i)
#pragma unroll
                for (int jj = 0; jj < FM; ++jj) {
                    const int idx = i * FM + jj;
                    if (idx % SPC == 0 && idx / SPC < NR) {
                        if (RD) read_one(idx / SPC, rbuf, rs, nxa, nwb);
                        if (Q0 + idx / SPC < Q1 && dm) dma_one(Q0 + idx / SPC, dkt, dbuf);
                        if (Q0 + NR + idx / SPC < Q1 && dm) dma_one(Q0 + NR + idx / SPC, dkt, dbuf);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    acc[i][jj] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wb[i], xa[jj], acc[i][jj], 0, 0, 0);
                }
            __builtin_amdgcn_sched_barrier(0);
        };

        // RING = LDS stages.  Steps 0 .. RING-1 are requested up front; step kt+RING is requested into the stage
        // step kt has just left: all of it in the second phase of step kt with two stages, and with three or more
        // (there is time) half there and half in the first phase of step kt+1, because a wavefront that waits
        // for the address unit to take a request issues no MFMA meanwhile, and the four wavefronts ask at once.
        // Loads complete in order, so "step s has landed" is a wait that leaves the loads of the younger steps
        // outstanding.
        constexpr int NSTG = RING;
        static_assert(NSTG >= 2 && NSTG <= 4, "stage count");
        constexpr auto vm = [](int n) { return ((n > 63 ? 63 : n) & 15) | (7 << 4) | (15 << 8) | (((n > 63 ? 63 : n) >> 4) << 14); };
        auto wait_landed = [&](int younger) {                          // younger: steps requested after the awaited one
            if (younger <= 0) __builtin_amdgcn_s_waitcnt(vm(0));
            else if (younger == 1) __builtin_amdgcn_s_waitcnt(vm(NL));
            else if (younger == 2) __builtin_amdgcn_s_waitcnt(vm(2 * NL));
            else __builtin_amdgcn_s_waitcnt(vm(3 * NL));               // RING <= 4: never more than three
        };
        // With two stages only the first step is requested up front and the second during the first MFMA phase: the
        // address unit takes as long over a stage's requests as the MFMAs of a phase take, so asking for both first
        // would only delay the first MFMA by that much.
        constexpr bool DEFER = NSTG == 2;
        const int npro = DEFER ? 1 : (nk < NSTG ? nk : NSTG);
        {
            // The per-channel constants (bias, mult, shift: 3 x BN dwords) go from global memory straight into LDS behind
            // the stages, 64 dwords per request, the requests dealt round the wavefronts -- before the tile requests, so
            // that they have landed when the first stage has (loads complete in order) and nothing but the epilogue
            // itself is left to do after the loop.  Missing arrays are filled in by hand.
            constexpr int CPA = (BN + 63) / 64;                        // requests per array
            const uint32_t par0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) int8_t*)lds + (uint32_t)EL::LDS_BYTES;
            const uint32_t voff4 = (uint32_t)lane * 4u;
#pragma unroll
            for (int a = 0; a < 3; ++a) {
                const int32_t* src = a == 0 ? g.bias : (a == 1 ? g.mult : g.shift);
                const bool have = a == 0 ? g.bias != nullptr : g.per_channel != 0;
                if (have) {
#pragma unroll
                    for (int c = 0; c < CPA; ++c) {
                        if ((a * CPA + c) % ND == wv && asker && (BN % 64 == 0 || c * 64 + lane < BN)) {
                            const uint32_t la = par0 + (uint32_t)((a * BN + c * 64) * 4);
                            if constexpr (NLD > 0) {
                                // (the address is the same in every lane; say so: behind the loaders' branch the compiler
                                // no longer sees it)
                                const uint64_t sbv = (uint64_t)(uintptr_t)(src + n0 + c * 64);
                                const uint64_t sb = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int32_t)(sbv >> 32)) << 32) |
                                                    (uint32_t)__builtin_amdgcn_readfirstlane((int32_t)(uint32_t)sbv);
                                asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2"
                                             :: "s"(la), "v"(voff4), "s"(sb) : "memory", "m0");
                            } else {
                                const int32_t* sb = src + n0 + c * 64;
                                asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2"
                                             :: "s"(la), "v"(voff4), "s"(sb) : "memory", "m0");
                            }
                        }
                    }
                } else {
                    const int32_t fill = a == 0 ? 0 : (a == 1 ? g.dy_m : g.dy_s);
                    for (int c = tid; c < BN; c += NT) par_early[a * BN + c] = fill;
                }
            }
        }
#pragma unroll
        for (int st = 0; st < NSTG; ++st)
            if (st < npro && asker) {
#pragma unroll
                for (int q = 0; q < NL; ++q) dma_one(q, st, st);
            }
        if constexpr (GELU) {
            // Likewise: tabulate GELU (with its output requantization) over the interval
            // outside of which it is constant -- below q_b the result is DY(0), from the first saturated value up
            // it stays saturated -- so that the epilogue replaces ~17 instructions per value by a clamp and a byte
            // read.  Every workgroup builds its own copy with the very function the table stands for.
            // (by the wavefronts that request no tiles, where there are such: the others are busy asking)
            int8_t* lut = lds + EL::LDS_BYTES + PAR_BYTES;
            const int32_t rnd = 1 << ((g.gelu.s - 33) & 31), sh = (g.gelu.s - 32) & 31;
            constexpr int NB = ND < NW ? NT - 64 * ND : NT;            // threads that build
            if (ND == NW || !asker) {
                for (int e = ND < NW ? tid - 64 * ND : tid; e < g.gelu_lut_n; e += NB) {
                    const int32_t q = g.gelu_lut_lo + e;
                    lut[e] = (int8_t)(g.gelu_fast ? gelu_one_fast(q, g.gelu, rnd, sh) : gelu_one(q, g.gelu));
                }
            }
        }
        if (NLD == 0 || asker) wait_landed(npro - 1);
        asm volatile("s_barrier" ::: "memory");
        if (NLD > 0 && loader) {
            // the loop of a loader wavefront: the requests of the MFMA wavefronts' two phases, the same waits and barriers
            constexpr int QHL = NSTG >= 3 ? (NL + 1) / 2 : NL;
            int lbuf = 0;
            for (int kt = 0; kt < nk; ++kt) {
                const int nbuf = lbuf + 1 == NSTG ? 0 : lbuf + 1, pbuf = lbuf == 0 ? NSTG - 1 : lbuf - 1;
                if (DEFER && kt == 0) {
                    if (nk > 1) {
#pragma unroll
                        for (int q = 0; q < NL; ++q) dma_one(q, 1, 1);
                    }
                } else if (kt >= 1 && kt - 1 + NSTG < nk) {
#pragma unroll
                    for (int q = QHL; q < NL; ++q) dma_one(q, kt - 1 + NSTG, pbuf);
                }
                const int hi = kt + NSTG - 1 < nk - 1 ? kt + NSTG - 1 : nk - 1;
                wait_landed(hi - (kt + 1));
                asm volatile("s_barrier" ::: "memory");
                if (kt + NSTG < nk) {
#pragma unroll
                    for (int q = 0; q < QHL; ++q) dma_one(q, kt + NSTG, lbuf);
                }
                lbuf = nbuf;
            }
            return;
        }
        v4i xa0[FM], wb0[FN], xa1[FM], wb1[FN];
#pragma unroll
        for (int q = 0; q < NR; ++q) read_one(q, 0, 0, xa0, wb0);
        {
            // The constants have landed with the first stage.  Every wavefront looks at all BN channels itself and decides
            // whether they allow the register-direct epilogue (see "Fast path" below): the same answer in all of
            // them without another barrier, and nothing but the epilogue itself is left to do after the loop.
            int badc = 0, bigs = 0;
            for (int c = lane; c < BN; c += 64) {
                const int32_t pbc = par_early[c], psc = par_early[2 * BN + c];
                const int32_t ab = pbc < 0 ? -pbc : pbc;
                badc |= (psc < 33 || psc > 62 || ab < 0 || ab >= (1 << 30)) ? 1 : 0;
                bigs |= psc > 43 ? 1 : 0;
            }
            fast_early = __builtin_amdgcn_ballot_w64(badc != 0) == 0 && g.res_fast && (int64_t)g.K * 16129 < (1 << 30);
            fold_early = __builtin_amdgcn_ballot_w64(bigs != 0) == 0;  // every shift at most 43
        }
        // One K step.  Phase 1: slice 0 (fragments already in registers) while slice 1 is read.  Then this
        // wavefront's share of step kt+1 has landed and its reads of stage `buf` are done; after the barrier
        // that holds for the whole workgroup, so `buf` may be refilled and the next stage read.  Phase 2:
        // slice 1, while slice 0 of step kt+1 is read and step kt+RING is requested (uniform test per request).
        int buf = 0;
        for (int kt = 0; kt < nk; ++kt) {
            const int nbuf = buf + 1 == NSTG ? 0 : buf + 1;
            constexpr int QH = NSTG >= 3 ? (NL + 1) / 2 : NL;          // blocks requested in the second phase
            const int pbuf = buf == 0 ? NSTG - 1 : buf - 1;
            if (DEFER && kt == 0)
                phase(xa0, wb0, xa1, wb1, buf, 1, std::true_type{}, 1, 1, asker && nk > 1,
                      std::integral_constant<int, 0>{}, std::integral_constant<int, NL>{});
            else
                phase(xa0, wb0, xa1, wb1, buf, 1, std::true_type{}, kt - 1 + NSTG, pbuf, asker && kt >= 1 && kt - 1 + NSTG < nk,
                      std::integral_constant<int, QH>{}, std::integral_constant<int, NL>{});
            // steps requested after kt+1 so far: kt+2 .. min(kt+RING-1, nk-1)
            const int hi = kt + NSTG - 1 < nk - 1 ? kt + NSTG - 1 : nk - 1;
            if (NLD == 0 || asker) wait_landed(hi - (kt + 1));
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
            // (the fragment reads past the last step fetch stale LDS bytes that nothing uses)
            phase(xa1, wb1, xa0, wb0, nbuf, 0, std::true_type{}, kt + NSTG, buf, asker && kt + NSTG < nk,
                  std::integral_constant<int, 0>{}, std::integral_constant<int, QH>{});
            buf = nbuf;
        }
    } else {
    // The loop body is branch-free apart from one uniform test around the MFMAs, so that the compiler can
    // count outstanding loads exactly (vmcnt) instead of draining them: loads past the last step re-read
    // the last step (never used), and the LDS write of a step past the end lands in the idle buffer.
    const int last = nk - 1;                           // nk >= 1 (K == 0 never reaches this kernel)
#pragma unroll
    for (int s = 0; s < RING; ++s) load_global(s < last ? s : last, s);
    store_lds(0, 0);
    load_global(RING < last ? RING : last, 0);
    __syncthreads();

    for (int kt0 = 0; kt0 < nk; kt0 += RING) {
#pragma unroll
        for (int j = 0; j < RING; ++j) {
            const int kt = kt0 + j;
            const int buf = kt & 1;
            const int slot = (j + 1) % RING;           // slot of step kt + 1 (kt0 is a multiple of RING)
            store_lds(slot, buf ^ 1);
            const int nxt = kt + 1 + RING;
            load_global(nxt < last ? nxt : last, slot);
            if (kt < nk) {
                v4i xa[2][FM], wb[2][FN];
                read_frags(buf, 0, xa[0], wb[0]);
#pragma unroll
                for (int s = 0; s < NS; ++s) {
                    if (s + 1 < NS) read_frags(buf, s + 1, xa[(s + 1) & 1], wb[(s + 1) & 1]);
#pragma unroll
                    for (int i = 0; i < FN; ++i)
#pragma unroll
                        for (int jj = 0; jj < FM; ++jj)
                            acc[i][jj] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wb[s & 1][i], xa[s & 1][jj], acc[i][jj], 0, 0, 0);
                }
            }
            __syncthreads();
        }
    }

    }

    // ---- Epilogue -------------------------------------------------------------------------------
    // acc[i][j][r] = C[m0 + wm0 + 16 j + lane%16][n0 + wn0 + 16 i + 4 (lane/16) + r].
    // The accumulators go through LDS (free now), a chunk of rows at a time, so that a short loop can
    // requantize them and write whole rows: a lane finishes 4 consecutive channels of one token per step and
    // consecutive lanes are consecutive in memory.  Only the accumulator indices have to be unrolled, which
    // keeps the code small.  The finishing loop must never wait on memory -- a wait for a load would also
    // wait for the previous store to be acknowledged (one counter covers both), a full round trip per row --
    // so per-channel constants sit in registers and the residual tile is parked in LDS beforehand.
    // (The direct-to-LDS loop reads nothing it still needs from LDS after the barrier of its last step, so the stages
    // are free from here on without another barrier.)
    constexpr int SP = EL::SP, JC = EL::JC;
    constexpr int G4 = BN / 4;                                     // 4-channel groups per row
    constexpr int RPS = NT / G4;                         // rows finished per pass of the workgroup
    // JCW: MFMA block rows of a wavefront per staged chunk (with four rows of wavefronts the chunk is the whole tile)
    constexpr int JCW = R4 ? FM : JC;
    static_assert(FM % JCW == 0 && RPS >= 1 && 16 * WR * JCW == 32 * JC, "epilogue layout");
    int32_t* stage = reinterpret_cast<int32_t*>(lds);              // [32 * JC][SP]
    // [3][BN]: bias, mult, shift -- behind the stages for the direct-to-LDS kernels (written before the loop), else
    // behind the staging tile
    int32_t* par = DMA ? par_early : stage + 32 * JC * SP;
    uint32_t* resl = reinterpret_cast<uint32_t*>(stage + 32 * JC * SP + 3 * BN);   // [BM][BN / 4]: residual tile, 4 channels per dword

    int bad = 0;
    if constexpr (!DMA) {
#pragma unroll
        for (int q = 0; q < PPT; ++q) {
            const int c = q * NT + tid;
            if (c < BN) {
                par[c] = pb[q];
                par[BN + c] = pm[q];
                par[2 * BN + c] = ps[q];
                const int32_t ab = pb[q] < 0 ? -pb[q] : pb[q];
                bad |= (ps[q] < 33 || ps[q] > 62 || ab < 0 || ab >= (1 << 30)) ? 1 : 0;
            }
        }
    }
    if (RPRE > 0 && res_early) {
#pragma unroll
        for (int u = 0; u < RPRE; ++u) {
            const int q = u * NT + tid;
            if (q < RCH) *reinterpret_cast<v4i*>(resl + q * 4) = rpre[u];
        }
    } else if (R && interior) {
        // residual tile -> LDS, 16 bytes per lane, rows of BN bytes
        constexpr int CH = BM * BN / 16;                           // 16-byte chunks in the tile
#pragma unroll 1
        for (int q0 = 0; q0 < CH; q0 += 4 * NT) {
            v4i t[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int q = q0 + u * NT + tid;
                const int qq = q < CH ? q : 0;
                const int row = qq / (BN / 16), c16 = qq - row * (BN / 16);
                t[u] = *reinterpret_cast<const v4i*>(R + (int64_t)(m0 + row) * g.ldr + n0 + c16 * 16);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int q = q0 + u * NT + tid;
                if (q < CH) *reinterpret_cast<v4i*>(resl + q * 4) = t[u];
            }
        }
    }
    // Fast path: every shift of the tile is in [33, 62] (multipliers of magnitude below a quarter), every
    // |bias| and the largest possible |accumulator| (K * 127^2) are below 2^30, and the residual shift is in
    // [8, 62].  Then (acc + bias) m + 2^(s-1) fits 63 bits, its floor-division by 2^s equals the high dword
    // shifted by s-32, every term fits 32 bits, and an element costs one 64-bit multiply-add, a shift and a
    // three-operand clamp.
    bool fast;
    if constexpr (DMA) {
        fast = fast_early;
        if (R && interior) __syncthreads();                        // the residual tile is complete
    } else {
        fast = !__syncthreads_or(bad) && g.res_fast && (int64_t)g.K * 16129 < (1 << 30);
    }

    const int wrow = wave & (WR - 1);
    const int c4 = tid % G4, r0 = tid / G4;                        // lane = (row of the pass, 4-channel group)
    const int col = c4 * 4, n = n0 + col;
    const v4i b4 = *reinterpret_cast<const v4i*>(par + col);
    const v4i m4 = *reinterpret_cast<const v4i*>(par + BN + col);
    const v4i s4 = *reinterpret_cast<const v4i*>(par + 2 * BN + col);

    auto tile_row = [&](int jc0, int lr) {                         // row inside the BM x BN tile of chunk row lr
        const int w = lr / (16 * JCW), rem = lr - w * 16 * JCW;    // rem = 16 * jj + row-in-block
        return w * WM + 16 * jc0 + rem;
    };
    // Fast-path constants of the lane's four channels: c0 = bias*m + 2^(s-1) (64 bits), so that one
    // multiply-add gives (acc + bias)*m + 2^(s-1); the high dword shifted by s-32 is the requantized value.
    int64_t c0[4];
    int32_t sh32[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        c0[e] = (int64_t)b4[e] * m4[e] + ((int64_t)1 << ((s4[e] - 1) & 63));
        sh32[e] = (s4[e] - 32) & 31;
    }
    const int32_t clamp_lo = -g.out_clamp, clamp_hi = g.out_clamp;
    const int32_t gelu_rnd = 1 << ((g.gelu.s - 33) & 31), gelu_sh = (g.gelu.s - 32) & 31;
    auto post = [&](int32_t v) {                                   // v is already clamped to +-out_clamp
        if constexpr (GELU) return g.gelu_fast ? gelu_one_fast(v, g.gelu, gelu_rnd, gelu_sh) : gelu_one(v, g.gelu);
        else return v;
    };
    auto post_fast = [&](int32_t v) {                              // same, the caller has tested g.gelu_fast
        if constexpr (GELU) return gelu_one_fast(v, g.gelu, gelu_rnd, gelu_sh);
        else return v;
    };
    auto requant4 = [&](const v4i& a4, const int32_t (&res)[4], bool has_res, auto fast_tag, int32_t (&o)[4]) {
        constexpr bool FAST = decltype(fast_tag)::value;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (FAST) {
                const int64_t p = (int64_t)a4[e] * m4[e] + c0[e];                                       // |p| < 2^63
                int32_t v = (int32_t)(p >> 32) >> sh32[e];                                              // |v| <= 2^30
                if (has_res) v += (int32_t)(((int64_t)res[e] * g.res_m + g.res_rnd) >> g.res_s);       // |.| < 2^30
                o[e] = post(med3_i32(v, clamp_lo, clamp_hi));
            } else {
                const int32_t a = a4[e] + b4[e];
                const int sh = s4[e] & 63;
                int64_t v = ((int64_t)a * m4[e] + (sh > 0 ? (int64_t)1 << (sh - 1) : 0)) >> sh;
                if (has_res) v += ((int64_t)res[e] * g.res_m + g.res_rnd) >> g.res_s;
                o[e] = post(clamp_i64_to_i32(v, g.out_clamp));
            }
        }
    };
    // Output pointer of the lane's channel group in tile row 0; row offsets inside a tile fit 32 bits.
    const uint32_t esz = OUT_I8 ? 1u : (g.c16 ? 2u : 4u);          // bytes per output element
    char* const c_lane = reinterpret_cast<char*>(g.C) + (c_off + (int64_t)m0 * g.ldc + n) * (int64_t)esz;
    const uint32_t c_pitch = (uint32_t)g.ldc * esz;
    auto pack2_i16 = [](int32_t a, int32_t b) { return ((uint32_t)a & 0xffffu) | ((uint32_t)b << 16); };
    auto finish_interior = [&](int jc0, auto fast_tag) {
        if (tid >= RPS * G4) return;
        constexpr int U = 4;                                       // rows in flight: LDS reads first, then math and stores
#pragma unroll 1
        for (int lr0 = r0; lr0 < 32 * JC; lr0 += U * RPS) {
            v4i a4[U];
            uint32_t pk[U];
            int tr[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int lr = lr0 + u * RPS;
                const int lrc = lr < 32 * JC ? lr : r0;
                tr[u] = tile_row(jc0, lrc);
                a4[u] = *reinterpret_cast<const v4i*>(stage + lrc * SP + col);
                pk[u] = R ? resl[tr[u] * G4 + c4] : 0u;
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (lr0 + u * RPS < 32 * JC) {
                    int32_t res[4];
                    res[0] = (int8_t)(pk[u] & 0xff); res[1] = (int8_t)((pk[u] >> 8) & 0xff);
                    res[2] = (int8_t)((pk[u] >> 16) & 0xff); res[3] = (int8_t)(pk[u] >> 24);
                    int32_t o[4];
                    requant4(a4[u], res, R != nullptr, fast_tag, o);
                    char* cp = c_lane + (uint32_t)tr[u] * c_pitch;
                    if (OUT_I8) *reinterpret_cast<uint32_t*>(cp) = pack4_i8(o[0], o[1], o[2], o[3]);
                    else if (g.c16) *reinterpret_cast<uint2*>(cp) = uint2{pack2_i16(o[0], o[1]), pack2_i16(o[2], o[3])};
                    else *reinterpret_cast<v4i*>(cp) = v4i{o[0], o[1], o[2], o[3]};
                }
            }
        }
    };
    auto finish_edge = [&](int jc0) {                              // tiles on an edge or with unaligned rows
        if (tid >= RPS * G4 || n >= g.N) return;
        for (int lr = r0; lr < 32 * JC; lr += RPS) {
            const int m = m0 + tile_row(jc0, lr);
            if (m >= g.M) continue;
            const v4i a4 = *reinterpret_cast<const v4i*>(stage + lr * SP + col);
            int32_t res[4] = {0, 0, 0, 0};
            if (R) {
                const int8_t* rp = R + (int64_t)m * g.ldr + n;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (n + e < g.N) res[e] = rp[e];
            }
            int32_t o[4];
            requant4(a4, res, R != nullptr, std::false_type{}, o);
            const int64_t off = c_off + (int64_t)m * g.ldc + n;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (n + e < g.N) {
                    if (OUT_I8) (reinterpret_cast<int8_t*>(g.C) + off)[e] = (int8_t)o[e];
                    else if (g.c16) (reinterpret_cast<int16_t*>(g.C) + off)[e] = (int16_t)o[e];
                    else (reinterpret_cast<int32_t*>(g.C) + off)[e] = o[e];
                }
            }
        }
    };

    // Whole tiles on the fast path skip the staging: a lane already holds four consecutive channels of one
    // token per accumulator, so it requantizes them in place and stores them itself (4 bytes INT8, 16 bytes
    // INT32; the four lanes that share a token write 16 or 64 contiguous bytes).  The chain per value is
    // register-only -- constants of the lane's channel group are re-read from LDS once per MFMA block column.
    // The function is straight-line code: every choice that does not depend on the value itself (how the tile is
    // stored, which form of GELU) is a template tag, so that the compiler can keep many values of many blocks in flight
    // -- one block column's 4 FM values go through requantization together, then (table form of GELU) their table reads
    // are issued back to back, then they are packed and stored.
    // SM = how a lane's four values leave: 0 the lane's own store, 1 through LDS as whole row pieces (INT8: 16 bytes;
    // int16: 8 bytes).  ES = bytes per stored element (1, 2, 4).
    // FOLD (table form of GELU with every shift at most 43): the table's LDS address is folded into the requantization
    // constant -- (acc m + c - (lo - base) 2^s) >> s = v - lo + base exactly, the subtrahend being a multiple of 2^s, and
    // below 2^62 in magnitude, so the sum stays inside 64 bits -- which leaves a multiply-add, a shift, a clamp and a
    // byte read per value.  (Byte loads into register halves would pack four values with one instruction, but with
    // ECC on the register file they clear the other half instead of keeping it.)
    auto finish_direct = [&](auto res_tag, auto gf_tag, auto lut_tag, auto sm_tag, auto es_tag, auto fold_tag) {
        constexpr bool RES = decltype(res_tag)::value, GF = decltype(gf_tag)::value, LUT = decltype(lut_tag)::value;
        constexpr int SM = decltype(sm_tag)::value, ES = decltype(es_tag)::value;
        constexpr bool FOLD = decltype(fold_tag)::value;
        static_assert(!FOLD || (LUT && ES == 1 && !RES), "folding belongs to the table form");
        static_assert((ES == 1) == OUT_I8, "INT8 kernels store bytes");
        const int8_t* const lut = lds + EL::LDS_BYTES + PAR_BYTES;
        const uint32_t lut_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) int8_t*)lds + (uint32_t)(EL::LDS_BYTES + PAR_BYTES);
        const int32_t lut_hi = g.gelu_lut_n - 1;
        // staged row pitch in bytes (16-byte aligned rows): padded by one piece, or -- where only the bare tile fits and
        // a row is a whole number of 256-byte bank cycles -- unpadded with the pieces of a row permuted by the row
        // number, so that the 16 rows a wavefront writes at once still land on 16 different bank groups
        constexpr bool OST_PAD = BM * (BN + 16) <= 32 * JC * SP * 4;
        constexpr bool OST_SWZ = !OST_PAD && BN == 256 && BM * BN <= 32 * JC * SP * 4;
        constexpr int SPB = OST_PAD ? BN + 16 : BN;
        auto ost_at = [&](int row, int col) {                      // byte offset of column col (a multiple of 4) of a staged row
            const int piece = OST_SWZ ? ((col >> 4) ^ (row & 15)) : (col >> 4);
            return row * SPB + (piece << 4) + (col & 15);
        };
        constexpr int SPH = 2 * BN + 8;                            // int16 rows: 8-byte pieces, padded by one
        static_assert(SM == 0 || ES != 2 || BM * SPH <= 32 * JC * SP * 4, "the 16-bit staging tile ends where the constants begin");
        static_assert(SM == 0 || ES != 1 || OST_PAD || OST_SWZ, "the INT8 staging tile fits in front of the constants");
        static_assert(SM == 0 || ES != 4, "INT32 outputs are stored by the lanes themselves");
        int8_t* const ostage = lds;
        char* const c_base = reinterpret_cast<char*>(g.C) +
                             (c_off + (int64_t)(m0 + wm0 + frow) * g.ldc + n0 + wn0 + 4 * fch) * (int64_t)ES;
        const uint32_t pitch = (uint32_t)g.ldc * ES;
        const uint32_t* const r_base = resl + (wm0 + frow) * G4 + (wn0 >> 2) + fch;
        static_assert(SM != 2 || (ES == 1 && FN <= 4), "lane-transposed stores: INT8, at most four block columns a wavefront");
        uint32_t pq[SM == 2 ? 4 : 1][FM];                          // SM 2: the packed dwords, by block column
        if (SM == 2) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < FM; ++j) pq[SM == 2 ? i : 0][j] = 0u;
        }
#pragma clang loop unroll(full)
        for (int i = 0; i < FN; ++i) {
            const int cl = wn0 + 16 * i + 4 * fch;
            const v4i bb = *reinterpret_cast<const v4i*>(par + cl);
            const v4i mm = *reinterpret_cast<const v4i*>(par + BN + cl);
            const v4i ss = *reinterpret_cast<const v4i*>(par + 2 * BN + cl);
            int64_t cc[4];
            int32_t sh[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                cc[e] = (int64_t)bb[e] * mm[e] + ((int64_t)1 << ((ss[e] - 1) & 63));
                if (FOLD) cc[e] -= (int64_t)(g.gelu_lut_lo - (int32_t)lut_lds) << (ss[e] & 63);
                sh[e] = (ss[e] - 32) & 31;
            }
            uint32_t pk[FM];
            if constexpr (FOLD) {
                typedef const __attribute__((address_space(3))) uint8_t* lds_bytes;
                uint32_t by[FM][4];
#pragma unroll
                for (int j = 0; j < FM; ++j)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int64_t p = (int64_t)acc[i][j][e] * mm[e] + cc[e];
                        by[j][e] = (uint32_t)med3_i32((int32_t)(p >> 32) >> sh[e], (int32_t)lut_lds, (int32_t)lut_lds + lut_hi);
                    }
#pragma unroll
                for (int j = 0; j < FM; ++j)
#pragma unroll
                    for (int e = 0; e < 4; ++e) by[j][e] = *(lds_bytes)(uintptr_t)by[j][e];
#pragma unroll
                for (int j = 0; j < FM; ++j) {
                    const uint32_t pk4 = (by[j][0] | (by[j][1] << 8)) | ((by[j][2] | (by[j][3] << 8)) << 16);
                    char* cp = c_base + ((uint32_t)(j * 16) * pitch + (uint32_t)(i * 16) * ES);
                    const int row = wm0 + 16 * j + frow, colb = wn0 + 16 * i + 4 * fch;
                    if (SM == 2) pq[i < 4 ? i : 0][j] = pk4;
                    else if (SM == 1) *reinterpret_cast<uint32_t*>(ostage + ost_at(row, colb)) = pk4;
                    else *reinterpret_cast<uint32_t*>(cp) = pk4;
                }
                continue;
            }
            if (RES) {
#pragma unroll
                for (int j = 0; j < FM; ++j) pk[j] = r_base[j * 16 * G4 + i * 4];
            }
            int32_t o[FM][4];
#pragma unroll
            for (int j = 0; j < FM; ++j)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int64_t p = (int64_t)acc[i][j][e] * mm[e] + cc[e];
                    int32_t v = (int32_t)(p >> 32) >> sh[e];
                    if (RES) {
                        const int32_t r8 = (int32_t)(int8_t)(pk[j] >> (8 * e));
                        v += (int32_t)(((int64_t)r8 * g.res_m + g.res_rnd) >> g.res_s);
                    }
                    if (LUT) {
                        // (the table covers [lo, lo + n) inside [-q_max, q_max] and the function is constant beyond its
                        // ends, so the clamp to the table is the clamp to +-q_max as well; |v| <= 2^30: no wrap)
                        o[j][e] = med3_i32(v - g.gelu_lut_lo, 0, lut_hi);
                    } else {
                        v = med3_i32(v, clamp_lo, clamp_hi);
                        o[j][e] = GF ? post_fast(v) : post(v);
                    }
                }
            if (LUT) {
#pragma unroll
                for (int j = 0; j < FM; ++j)
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[j][e] = lut[o[j][e]];
            }
#pragma unroll
            for (int j = 0; j < FM; ++j) {
                char* cp = c_base + ((uint32_t)(j * 16) * pitch + (uint32_t)(i * 16) * ES);
                const int row = wm0 + 16 * j + frow, colb = wn0 + 16 * i + 4 * fch;
                if (ES == 1) {
                    const uint32_t pk4 = pack4_i8(o[j][0], o[j][1], o[j][2], o[j][3]);
                    if (SM == 2) pq[i < 4 ? i : 0][j] = pk4;
                    else if (SM == 1) *reinterpret_cast<uint32_t*>(ostage + ost_at(row, colb)) = pk4;
                    else *reinterpret_cast<uint32_t*>(cp) = pk4;
                } else if (ES == 2) {
                    const uint2 pk2 = uint2{pack2_i16(o[j][0], o[j][1]), pack2_i16(o[j][2], o[j][3])};
                    if (SM == 1) *reinterpret_cast<uint2*>(ostage + row * SPH + colb * 2) = pk2;
                    else *reinterpret_cast<uint2*>(cp) = pk2;
                } else {
                    *reinterpret_cast<v4i*>(cp) = v4i{o[j][0], o[j][1], o[j][2], o[j][3]};
                }
            }
        }
        if (SM == 2) {
            // A lane holds 4 bytes (its 4 channels) of one token per block column; the four lanes that share the token
            // (16 apart) hold 16 consecutive bytes of it between them.  Transposing the 4 x 4 arrangement (lane group x
            // block column) with the swaps of 32- and 16-lane rows between registers gives lane group b the 16 bytes of
            // block column b, which leave as one 16-byte store -- 16 tokens x 16 FN bytes per instruction, no trip
            // through LDS and no barrier.
            typedef unsigned v2u __attribute__((ext_vector_type(2)));
            char* const c16 = reinterpret_cast<char*>(g.C) + c_off + (int64_t)(m0 + wm0 + frow) * g.ldc + n0 + wn0 + 16 * fch;
#pragma unroll
            for (int j = 0; j < FM; ++j) {
                uint32_t r0 = pq[0][j], r1 = pq[SM == 2 ? 1 : 0][j], r2 = pq[SM == 2 ? 2 : 0][j], r3 = pq[SM == 2 ? 3 : 0][j];
                v2u t = __builtin_amdgcn_permlane32_swap(r0, r2, false, false); r0 = t.x; r2 = t.y;
                t = __builtin_amdgcn_permlane32_swap(r1, r3, false, false); r1 = t.x; r3 = t.y;
                t = __builtin_amdgcn_permlane16_swap(r0, r1, false, false); r0 = t.x; r1 = t.y;
                t = __builtin_amdgcn_permlane16_swap(r2, r3, false, false); r2 = t.x; r3 = t.y;
                if (fch < FN) {
                    *reinterpret_cast<v4i*>(c16 + (uint32_t)(j * 16) * pitch) = v4i{(int)r0, (int)r1, (int)r2, (int)r3};
                }
            }
        }
        if (SM == 1 && ES == 2) {
            __syncthreads();
            constexpr int P8 = BN / 4, CH = BM * P8;               // 8-byte pieces per row, per tile
            char* const ct = reinterpret_cast<char*>(g.C) + (c_off + (int64_t)m0 * g.ldc + n0) * 2;
#pragma unroll 4
            for (int q0 = 0; q0 < CH; q0 += NT) {
                const int q = q0 + tid;
                if (CH % NT == 0 || q < CH) {
                    const int row = q / P8, c8 = q - row * P8;
                    *reinterpret_cast<uint2*>(ct + (uint32_t)row * pitch + c8 * 8) =
                        *reinterpret_cast<const uint2*>(ostage + row * SPH + c8 * 8);
                }
            }
        }
        if (SM == 1 && ES == 1) {
            __syncthreads();
            constexpr int C16 = BN / 16, CH = BM * C16;            // 16-byte chunks per row, per tile
            char* const ct = reinterpret_cast<char*>(g.C) + c_off + (int64_t)m0 * g.ldc + n0;
#pragma unroll
            for (int q0 = 0; q0 < CH; q0 += NT) {
                const int q = q0 + tid;
                if (CH % NT == 0 || q < CH) {
                    const int row = q / C16, c16 = q - row * C16;
                    *reinterpret_cast<v4i*>(ct + (uint32_t)row * pitch + c16 * 16) =
                        *reinterpret_cast<const v4i*>(ostage + ost_at(row, c16 * 16));
                }
            }
        }
    };
    // Which tiles leave through LDS (measured): INT8 tiles without GELU, and with GELU those of eight wavefronts -- a lane's
    // own store would be 4 bytes in each of 16 rows per instruction, which the address unit takes an order of magnitude
    // longer over than whole rows (a gain of 1.5-2 us on the QKV projections; S7+S8 of Base 18.9 -> 17.9 us, of Base at
    // 512 tokens x 64: 133.8 -> 125.5 us; the four-wavefront GELU tiles gain nothing from it and 256x128 loses); int16
    // tiles of eight wavefronts (256x192, [32768,768] outputs: K 768 48.3 -> 43.5 us, K 3072 91.7 -> 89.5 us; the
    // four-wavefront tiles lose by it -- 128x96: 9.6 -> 11.0 us; 256x128: 66.5 -> 76.4 us).
    constexpr bool OST_FITS = BM * (BN + 16) <= 32 * JC * SP * 4 || (BN == 256 && BM * BN <= 32 * JC * SP * 4);
    constexpr bool OST = OUT_I8 && (!GELU || NW == 8) && OST_FITS;
    constexpr bool LTS = OUT_I8 && NW == 8 && FN <= 4;             // lane-transposed 16-byte stores instead
    constexpr bool OST16 = !OUT_I8 && NW == 8 && BM <= 64 * JC;
    using T = std::true_type;
    using F = std::false_type;
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using I2 = std::integral_constant<int, 2>;
    using I4 = std::integral_constant<int, 4>;
    if (g.path_word && blockIdx.x == 0 && blockIdx.y == 0 && tid == 0)
        *g.path_word = !interior ? IBERT_EPILOGUE_EDGE
                                 : (!fast ? IBERT_EPILOGUE_STAGED
                                          : (GELU && g.gelu_lut_n > 0 ? IBERT_EPILOGUE_DIRECT_GELU_TABLE : IBERT_EPILOGUE_DIRECT));
    if (interior && fast) {
        // (GELU excludes a residual; without a table -- it did not fit, or the parameters are unusual -- the
        // arithmetic form runs, with the choice between its two variants made per value)
        using I2s = std::integral_constant<int, 2>;
        bool stored = false;
        if constexpr (LTS) {
            if (g.c_vec16 && !R) {
                if constexpr (GELU) {
                    if (g.gelu_lut_n > 0) if (fold_early) finish_direct(F{}, F{}, T{}, I2s{}, I1{}, T{}); else finish_direct(F{}, F{}, T{}, I2s{}, I1{}, F{});
                    else finish_direct(F{}, F{}, F{}, I2s{}, I1{}, F{});
                } else {
                    finish_direct(F{}, F{}, F{}, I2s{}, I1{}, F{});
                }
                stored = true;
            }
        }
        if (stored) {
        } else if constexpr (OUT_I8) {
            const bool via_lds = OST && g.c_vec16;
            if constexpr (GELU) {
                if (g.gelu_lut_n > 0) {
                    if constexpr (OST) { if (via_lds) if (fold_early) finish_direct(F{}, F{}, T{}, I1{}, I1{}, T{}); else finish_direct(F{}, F{}, T{}, I1{}, I1{}, F{}); else if (fold_early) finish_direct(F{}, F{}, T{}, I0{}, I1{}, T{}); else finish_direct(F{}, F{}, T{}, I0{}, I1{}, F{}); }
                    else if (fold_early) finish_direct(F{}, F{}, T{}, I0{}, I1{}, T{}); else finish_direct(F{}, F{}, T{}, I0{}, I1{}, F{});
                } else {
                    finish_direct(F{}, F{}, F{}, I0{}, I1{}, F{});
                }
            } else {
                if constexpr (OST) {
                    if (via_lds) { if (R) finish_direct(T{}, F{}, F{}, I1{}, I1{}, F{}); else finish_direct(F{}, F{}, F{}, I1{}, I1{}, F{}); }
                    else { if (R) finish_direct(T{}, F{}, F{}, I0{}, I1{}, F{}); else finish_direct(F{}, F{}, F{}, I0{}, I1{}, F{}); }
                } else {
                    if (R) finish_direct(T{}, F{}, F{}, I0{}, I1{}, F{}); else finish_direct(F{}, F{}, F{}, I0{}, I1{}, F{});
                }
            }
        } else {
            if (g.c16) {
                if constexpr (OST16) { if (R) finish_direct(T{}, F{}, F{}, I1{}, I2{}, F{}); else finish_direct(F{}, F{}, F{}, I1{}, I2{}, F{}); }
                else { if (R) finish_direct(T{}, F{}, F{}, I0{}, I2{}, F{}); else finish_direct(F{}, F{}, F{}, I0{}, I2{}, F{}); }
            } else {
                if (R) finish_direct(T{}, F{}, F{}, I0{}, I4{}, F{}); else finish_direct(F{}, F{}, F{}, I0{}, I4{}, F{});
            }
        }
    } else
#pragma unroll
    for (int jc = 0; jc < FM / JCW; ++jc) {
        if (jc > 0) __syncthreads();                               // the previous chunk has been consumed
#pragma unroll
        for (int jj = 0; jj < JCW; ++jj)
#pragma unroll
            for (int i = 0; i < FN; ++i)
                *reinterpret_cast<v4i*>(stage + ((wrow * JCW + jj) * 16 + frow) * SP + wn0 + i * 16 + fch * 4) = acc[i][jc * JCW + jj];
        __syncthreads();
        if (!interior) finish_edge(jc * JCW);
        else if (fast) finish_interior(jc * JCW, std::true_type{});
        else finish_interior(jc * JCW, std::false_type{});
    }
}

// ---------------------------------------------------------------------------------------------
// Launchers.  Each tile configuration is instantiated in exactly one translation unit (gemm_inst_*.hip, which list
// their configurations in gemm_instances_*.inc); gemm.hip sees them as extern templates.
// ---------------------------------------------------------------------------------------------
bool xcd_blocks_enabled();       // (gemm.hip: a switch for A/B measurements, on by default)

template <int BM, int BN, int BK, int RING, bool TW = false, bool DMA = false, bool GELU = false, int NW = 4, int NLD = 0>
int launch_mfma(GemmArgs& g, bool i8, hipStream_t stream)
{
    g.tiles_m = (g.M + BM - 1) / BM;
    g.tiles_n = (g.N + BN - 1) / BN;
    const int64_t blocks = (int64_t)g.tiles_m * g.tiles_n * g.nbatch;
    if (blocks > 0x7fffffffLL) return IBERT_ERR_SHAPE;
    g.xcd_chunk = (blocks % 8 == 0 && blocks >= 16) ? (int32_t)(blocks / 8) : 0;
    g.xcd_xn = g.xcd_xs = 0;
    g.xcd_bm = g.xcd_bn = 0;
    if (g.xcd_chunk > 0 && g.nbatch == 1) {
        // fabric bytes of the operands ~ XN * M + XM * N (times K) for XM x XN blocks, XM * XN = 8
        int best_xn = 0, best_xs = 0;
        int64_t best = 0;
        for (int xs = 0; xs <= (xcd_blocks_enabled() ? 3 : 0); ++xs) {
            const int xn = 1 << xs, xm = 8 >> xs;
            if (g.tiles_m % xm != 0 || g.tiles_n % xn != 0) continue;
            const int64_t cost = (int64_t)xn * g.M + (int64_t)xm * g.N;
            if (best_xn == 0 || cost < best) { best = cost; best_xn = xn; best_xs = xs; }
        }
        if (best_xn > 0) {
            g.xcd_xn = best_xn;
            g.xcd_xs = best_xs;
            g.xcd_bm = g.tiles_m / (8 / best_xn);
            g.xcd_bn = g.tiles_n / best_xn;
        }
    }
    const dim3 grid = g.xcd_xn >= 1 ? dim3(8u * (unsigned)g.xcd_bn, (unsigned)g.xcd_bm) : dim3((unsigned)blocks);
    constexpr size_t lds_tile = EpiLayout<BM, BN, BK, (DMA ? RING : 2)>::LDS_BYTES;
    static_assert(lds_tile <= 163840, "LDS budget");
    // (direct-to-LDS kernels keep the per-channel constants behind the stages)
    constexpr size_t par_bytes = DMA ? (size_t)((3 * BN * 4 + 255) & ~255) : 0;
    static_assert(lds_tile + par_bytes <= 163840, "LDS budget");
    size_t lds_bytes = lds_tile + par_bytes;
    if (GELU) {
        // the GELU table rides behind them if it fits the CU's 160 KB (and, for tiles that share a CU,
        // stays small enough not to cost a resident workgroup)
        const size_t room = lds_bytes >= 81920 ? 163840 - lds_bytes : (163840 / 2 - lds_bytes);
        // (small tiles have fewer values than the table has entries: they take the arithmetic form)
        if (DMA && g.gelu_lut_n > 0 && (size_t)g.gelu_lut_n <= room) lds_bytes += ((size_t)g.gelu_lut_n + 255) & ~(size_t)255;
        else g.gelu_lut_n = 0;
    }
#define IBERT_GEMM_LAUNCH(I8_, KT_)                                                                       \
    do {                                                                                                  \
        auto kern = gemm_nt_mfma_kernel<BM, BN, BK, RING, I8_, KT_, TW, DMA, GELU && I8_, NW, NLD>;          \
        static size_t attr_bytes = 0;                                                                     \
        if (lds_bytes > attr_bytes) {                                                                     \
            IBERT_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                      \
                                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes)); \
            attr_bytes = lds_bytes;                                                                       \
        }                                                                                                 \
        hipLaunchKernelGGL(kern, grid, dim3(64 * (NW + NLD)), lds_bytes, stream, g);                      \
    } while (0)
    if constexpr (GELU) {
        if (!i8 || g.K % BK != 0) return IBERT_ERR_NOT_IMPLEMENTED;
        IBERT_GEMM_LAUNCH(true, 0);
    } else if (g.K % BK == 0) {
        if (i8) IBERT_GEMM_LAUNCH(true, 0); else IBERT_GEMM_LAUNCH(false, 0);
    } else if constexpr (!DMA) {
        if (i8) IBERT_GEMM_LAUNCH(true, 1); else IBERT_GEMM_LAUNCH(false, 1);
    } else {
        return IBERT_ERR_SHAPE;                                    // never chosen for such K
    }
#undef IBERT_GEMM_LAUNCH
    IBERT_LAUNCH_CHECK("gemm_nt_mfma_kernel");
    // the name a profiler shows for this instantiation
    static char label[2][2][96];
    char* l = label[i8 ? 1 : 0][g.K % BK == 0 ? 0 : 1];
    if (!l[0])
        std::snprintf(l, sizeof label[0][0], "gemm_nt_mfma_kernel<%d, %d, %d, %d, %s, %d, %s, %s, %s, %d, %d>", BM, BN, BK, RING,
                      i8 ? "true" : "false", g.K % BK == 0 ? 0 : 1, TW ? "true" : "false", DMA ? "true" : "false",
                      GELU ? "true" : "false", NW, NLD);
    g_last_kernel = l;
    return IBERT_OK;
}

// K not a multiple of 16 (rows still 16-byte aligned): one configuration with the bytewise tail loader (gemm_inst_a.hip).
int launch_tail(GemmArgs& g, bool i8, hipStream_t stream);

}  // namespace ibert
