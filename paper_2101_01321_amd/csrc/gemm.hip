// INT8 x INT8 -> INT32 MatMul with bias, dyadic requantization, optional residual and clamp (Sec. 1 third contribution,
// App. C.1): argument checks, the choice of a tile configuration, the generic kernel for unaligned operands, and the
// C entry points.  The MFMA kernel is in gemm_kernel.h; its tile configurations are compiled in gemm_inst_*.hip.
#include "gemm_kernel.h"

namespace ibert {

#define IBERT_GEMM_INSTANCE(...) extern template int launch_mfma<__VA_ARGS__>(GemmArgs&, bool, hipStream_t);
#include "gemm_instances_a.inc"
#include "gemm_instances_b.inc"
#include "gemm_instances_c.inc"
#include "gemm_instances_d.inc"
#include "gemm_instances_e.inc"
#include "gemm_instances_f.inc"
#undef IBERT_GEMM_INSTANCE

// ---------------------------------------------------------------------------------------------
// Generic kernel: one output element per lane (lanes run along n), any layout and alignment.
// ---------------------------------------------------------------------------------------------
template <bool TRANS_W, bool OUT_I8>
__global__ __launch_bounds__(GEMM_THREADS) void gemm_generic_kernel(GemmArgs g)
{
    const int64_t per = (int64_t)g.M * g.N;
    const int64_t idx = (int64_t)blockIdx.x * GEMM_THREADS + threadIdx.x;
    if (idx >= per * g.nbatch) return;
    const int z = (int)(idx / per);
    const int64_t e = idx - (int64_t)z * per;
    const int i = (int)(e / g.N), n = (int)(e - (int64_t)i * g.N);
    const int zo = z / g.batch_inner, zi = z - zo * g.batch_inner;
    const int8_t* a = g.A + zo * g.sA_o + zi * g.sA_i + (int64_t)i * g.lda;
    const int8_t* w = g.W + zo * g.sW_o + zi * g.sW_i;
    int32_t acc = 0;
    if (TRANS_W) {
        w += n;
        for (int k = 0; k < g.K; ++k) acc += (int32_t)a[k] * (int32_t)w[(int64_t)k * g.ldw];
    } else {
        w += (int64_t)n * g.ldw;
        for (int k = 0; k < g.K; ++k) acc += (int32_t)a[k] * (int32_t)w[k];
    }
    if (g.bias) acc += g.bias[n];
    const int32_t m = g.per_channel ? g.mult[n] : g.dy_m;
    const int32_t s = g.per_channel ? g.shift[n] : g.dy_s;
    int32_t res = 0;
    if (g.R) res = g.R[zo * g.sR_o + zi * g.sR_i + (int64_t)i * g.ldr + n];
    const int32_t o = finish(acc, m, s, g.R != nullptr, res, g);
    const int64_t off = zo * g.sC_o + zi * g.sC_i + (int64_t)i * g.ldc + n;
    if (OUT_I8) reinterpret_cast<int8_t*>(g.C)[off] = (int8_t)o;
    else if (g.c16) reinterpret_cast<int16_t*>(g.C)[off] = (int16_t)o;
    else reinterpret_cast<int32_t*>(g.C)[off] = o;
}

// ---------------------------------------------------------------------------------------------
int check_gemm(const ibert_gemm_desc& d, const void* A, const void* W, const void* mult, const void* shift,
               const void* residual, const void* C)
{
    (void)residual;
    if (d.M < 0 || d.N < 0 || d.K < 0 || d.batch_outer < 0 || d.batch_inner < 0) return IBERT_ERR_SHAPE;
    if (d.K > (1 << 17)) return IBERT_ERR_SHAPE;
    if (d.out_dtype != IBERT_I8 && d.out_dtype != IBERT_I32 && d.out_dtype != IBERT_I16) return IBERT_ERR_PARAM_RANGE;
    if (d.out_clamp < 0 || (d.out_dtype == IBERT_I8 && d.out_clamp > 127)) return IBERT_ERR_PARAM_RANGE;
    if (d.out_dtype == IBERT_I16 && d.out_clamp > 32767) return IBERT_ERR_PARAM_RANGE;
    if (d.trans_w != 0 && d.trans_w != 1) return IBERT_ERR_PARAM_RANGE;
    if (!d.per_channel && !dyadic_ok(d.requant)) return IBERT_ERR_PARAM_RANGE;
    if (residual && !dyadic_ok(d.residual_dy)) return IBERT_ERR_PARAM_RANGE;
    const int64_t nb = (int64_t)d.batch_outer * d.batch_inner;
    if (nb == 0 || d.M == 0 || d.N == 0) return IBERT_OK;
    if (nb > 0x7fffffffLL) return IBERT_ERR_SHAPE;
    if (d.lda < d.K || d.ldc < d.N || (residual && d.ldr < d.N)) return IBERT_ERR_SHAPE;
    if (d.ldw < (d.trans_w ? d.N : d.K)) return IBERT_ERR_SHAPE;
    if (!C) return IBERT_ERR_NULL;
    if (d.K > 0 && (!A || !W)) return IBERT_ERR_NULL;
    if (d.per_channel && (!mult || !shift)) return IBERT_ERR_NULL;
    return IBERT_OK;
}

// Tile configurations of the MFMA kernel.
struct GemmConfig {
    int bm, bn, bk, ring;
    bool direct;          // direct-to-LDS loader (whole tiles only; ring = LDS stages) or register ring
};
static const GemmConfig kConfigs[] = {      // index = configuration number of ibert_gemm_config_override
    {256, 192, 128, 2, false},
    {128, 128, 128, 2, false},
    {128, 128, 64, 2, false},
    {64, 64, 128, 3, false},
    {64, 128, 64, 3, false},
    {128, 96, 128, 2, false},
    {256, 192, 128, 2, true},
    {128, 128, 128, 2, true},
    {256, 256, 128, 2, true},
    {128, 96, 128, 2, true},
    {256, 128, 128, 2, true},
    {128, 96, 128, 3, true},
    {128, 128, 128, 3, true},
    {256, 192, 128, 2, true},       // with eight wavefronts
    {256, 128, 128, 2, true},       // with eight wavefronts
    {32, 32, 128, 4, false},
    {256, 256, 128, 2, true},       // with eight wavefronts
    {64, 96, 128, 3, true},
    {64, 96, 128, 2, true},
    {64, 128, 128, 2, true},
    {128, 96, 128, 3, true},        // with eight wavefronts (four rows of two)
    {128, 96, 128, 3, true},        // the same with four more wavefronts that only request tiles
    {128, 128, 128, 3, true},       // eight wavefronts and four that only request tiles
};
constexpr int kNumConfigs = sizeof(kConfigs) / sizeof(kConfigs[0]);
static int g_config_override = -1;
static bool g_xcd_blocks = true;
bool xcd_blocks_enabled() { return g_xcd_blocks; }
static uint32_t* g_path_word = nullptr;

// GELU with its requantization, on the host (the arithmetic of gelu_one in 64 bits; the preconditions keep every
// value inside 32).  Used only to find where the function saturates.
static int32_t gelu_host(int64_t q, const ibert_gelu_params& p)
{
    q = q < -p.q_max ? -p.q_max : (q > p.q_max ? p.q_max : q);
    int64_t u = q < 0 ? -q : q;
    u = u > -(int64_t)p.q_b ? -(int64_t)p.q_b : u;
    const int64_t v = u + p.q_b, poly = v * v + p.q_c;
    const int64_t erf = q < 0 ? -poly : (q == 0 ? 0 : poly);
    const int64_t t = q * (erf + p.q_1);
    const int sh = p.out.s;
    const __int128 prod = (__int128)t * p.out.m + (sh > 0 ? ((__int128)1 << (sh - 1)) : 0);
    const int64_t y = (int64_t)(prod >> sh);
    return (int32_t)(y < -127 ? -127 : (y > 127 ? 127 : y));
}

// The interval [lo, lo + n) outside of which GELU-with-requantization is constant on [-q_max, q_max]: at and below
// q_b the polynomial argument is clipped, erf = -q_c, and with q_1 = q_c (c = 1 in Eq. 8-9) the product is zero;
// at and above -q_b the product is linear in q, so the clamped output is monotone and constant from its first
// saturated value on.  n = 0 when the parameters do not have that shape.
static void gelu_table_range(const ibert_gelu_params& p, int32_t* lo, int32_t* n)
{
    *lo = 0; *n = 0;
    if (p.q_1 != p.q_c || p.q_b >= 0 || p.q_max < -(int64_t)p.q_b) return;
    const int32_t top = gelu_host(p.q_max, p);
    int64_t a = -(int64_t)p.q_b, b = p.q_max;                     // first q in [a, b] with the value of q_max
    while (a < b) {
        const int64_t mid = a + (b - a) / 2;
        if (gelu_host(mid, p) == top) b = mid; else a = mid + 1;
    }
    const int64_t count = a - p.q_b + 1;
    if (count > (1 << 17)) return;
    *lo = p.q_b;
    *n = (int32_t)count;
}

// The direct-to-LDS loader handles whole tiles only, with row offsets that fit its 32-bit lane offsets.
static bool dma_ok(const ibert_gemm_desc& d, int bm, int bn)
{
    return d.M % bm == 0 && d.N % bn == 0 && d.K % 128 == 0 && d.lda < (1 << 28) && d.ldw < (1 << 28);
}

// Tile choice, measured on MI355X at RoBERTa-Base/Large shapes (256 CUs).
// Whole-tile problems with K a multiple of 128 take the direct-to-LDS loader: the biggest tile that still
// gives (nearly) every CU a workgroup -- big wavefront tiles need fewer LDS bytes per MFMA, which is what
// limits the loop -- and, when the problem is too small for that, 128x96 tiles, several of which share a CU
// so that one workgroup's requantization overlaps another's MFMAs.
// Everything else takes the register-ring loader: 128x128 tiles with a 64-wide K step while that gives every
// CU something to do, below that 64x64 tiles.
static int choose_config(const ibert_gemm_desc& d, int64_t nb, bool gelu)
{
    if (g_config_override >= 0 && g_config_override < kNumConfigs) return g_config_override;
    auto tiles = [&](int bm, int bn) -> int64_t { return dma_ok(d, bm, bn) ? (int64_t)(d.M / bm) * (d.N / bn) * nb : 0; };
    // (256x256 pays only when K is long enough to amortise its 256-value-per-lane epilogue, and never with GELU in it)
    // (with eight wavefronts for 16- and 32-bit outputs from two rounds of tiles on: [32768,1024] x K 4096 154 -> 131 us,
    //  2.1 POP/s; K 1024 67.8 -> 65.2 us)
    if (tiles(256, 256) >= 512 && d.out_dtype != IBERT_I8 && !gelu) return 16;
    // (INT8 outputs without GELU, whose rows leave packed through LDS, when the tiles come in whole rounds:
    //  [32768,3072] x K 1024 134 -> 120 us; with a ragged last round, or GELU in the epilogue, it loses)
    if (tiles(256, 256) >= 512 && tiles(256, 256) % 256 == 0 && d.out_dtype == IBERT_I8 && !gelu) return 16;
    if (tiles(256, 256) >= 512 && d.K >= 8192 && !gelu) return 8;
    // (with eight wavefronts; it pays from three quarters of a wave of tiles on: S1 of Base, 192 tiles, 17.1 -> 15.1 us)
    if (tiles(256, 192) >= (gelu ? 224 : 192)) return 13;
    // (one workgroup per CU and a long K: a third LDS stage lets the requests spread over the whole step)
    if (tiles(128, 96) >= 256) {
        // (exactly one 128x96 tile per CU and a 16- or 32-bit output: 64x96 tiles, three or four of which share a CU, so
        //  that one's epilogue overlaps another's loop -- inside the encoder S5 of Base 9.7 -> 8.9 us, S9 17.9 -> 17.3 us;
        //  a fourth LDS stage leaves room for one workgroup per CU only and loses, 24 us.)
        // (a long K instead: the whole 128x96 tile with eight wavefronts in four rows of two, three stages, and four more
        //  wavefronts that do nothing but request tiles, so that no MFMA wavefront ever waits for the address unit:
        //  [4096,768] x K 3072, timed alone: 64x96 tiles 18.5 us, eight wavefronts 17.6, with the loaders 15.8; INT8 output
        //  17.1 -> 14.4.  A short K gains nothing from it: S5 of Base 8.7 against 9.0.)
        if (tiles(128, 96) <= 256 && d.K >= 2048 && !gelu) return 21;
        if (tiles(128, 96) <= 256 && d.out_dtype != IBERT_I8 && !gelu) return 18;
        return tiles(128, 96) <= 256 && d.K >= 2048 ? 11 : 9;
    }
    // (eight wavefronts for INT8 outputs: S7+S8 of Large 34.7 -> 32.5 us; INT32 outputs lose 5 % with them)
    if (tiles(256, 128) >= 448) return (gelu || d.out_dtype == IBERT_I8) ? 14 : 10;
    if (tiles(128, 128) >= 128) {
        // (likewise 64x128 tiles for a short K: S5 of Large 14.4 -> 12.9 us; with K 4096 they lose, 25.9 -> 30 us)
        if (tiles(128, 128) <= 256 && d.K < 2048 && d.out_dtype != IBERT_I8 && !gelu) return 19;
        // (one tile per CU and a long K: eight wavefronts plus four loaders -- S9 of Large, [4096,1024] x K 4096: 27.0 -> 23.3 us)
        if (tiles(128, 128) <= 256 && d.K >= 2048 && !gelu) return 22;
        return tiles(128, 128) <= 256 && d.K >= 2048 ? 12 : 7;
    }
    const int64_t tiles128 = (((int64_t)d.M + 127) / 128) * (((int64_t)d.N + 127) / 128) * nb;
    if (tiles128 >= 384) return 2;
    // (a handful of sequences: 32x32 tiles put four times as many compute units on a long K than 64x64 do;
    //  [128,768] x K 3072: 10.5 -> 7.0 us, K 768: 5.6 -> 4.5 us)
    const int64_t tiles64 = (((int64_t)d.M + 63) / 64) * (((int64_t)d.N + 63) / 64) * nb;
    if (d.K >= 512) return tiles64 <= 96 ? 15 : 3;
    return 4;
}

// gelu != nullptr asks for the GELU epilogue (INT8 output, no residual; out_clamp must be gelu->q_max): only the
// direct-to-LDS tiles carry it, any other problem returns IBERT_ERR_NOT_IMPLEMENTED without launching.
int launch_gemm(const ibert_gemm_desc& d, const int8_t* A, const int8_t* W, const int32_t* bias,
                const int32_t* mult, const int32_t* shift, const int8_t* residual, void* C, hipStream_t stream,
                const ibert_gelu_params* gelu)
{
    const int64_t nb = (int64_t)d.batch_outer * d.batch_inner;
    if (nb == 0 || d.M == 0 || d.N == 0) return IBERT_OK;
    GemmArgs g;
    g.A = A; g.W = W; g.bias = bias; g.mult = mult; g.shift = shift; g.R = residual; g.C = C;
    g.M = d.M; g.N = d.N; g.K = d.K;
    g.batch_inner = d.batch_inner; g.nbatch = (int32_t)nb;
    g.tiles_m = g.tiles_n = 0;
    g.xcd_chunk = 0;
    g.xcd_xn = g.xcd_xs = g.xcd_bm = g.xcd_bn = 0;
    g.lda = d.lda; g.ldw = d.ldw; g.ldc = d.ldc; g.ldr = d.ldr;
    g.sA_o = d.strideA_outer; g.sA_i = d.strideA_inner;
    g.sW_o = d.strideW_outer; g.sW_i = d.strideW_inner;
    g.sC_o = d.strideC_outer; g.sC_i = d.strideC_inner;
    g.sR_o = d.strideR_outer; g.sR_i = d.strideR_inner;
    g.per_channel = d.per_channel ? 1 : 0;
    g.dy_m = d.requant.m; g.dy_s = d.requant.s;
    g.out_clamp = d.out_clamp;
    g.res_m = d.residual_dy.m; g.res_s = d.residual_dy.s;
    g.res_fast = (!residual || (d.residual_dy.s >= 8 && d.residual_dy.s <= 62)) ? 1 : 0;
    g.res_rnd = (residual && d.residual_dy.s >= 1 && d.residual_dy.s <= 62) ? ((int64_t)1 << (d.residual_dy.s - 1)) : 0;
    const bool i8 = d.out_dtype == IBERT_I8;
    g.c16 = d.out_dtype == IBERT_I16 ? 1 : 0;
    g.path_word = g_path_word;
    g.gelu_fast = 0;
    g.gelu = GeluConst{0, 0, 0, 0, 0, 0};
    g.gelu_lut_lo = g.gelu_lut_n = 0;
    if (gelu) {
        if (!i8 || residual || d.out_clamp != gelu->q_max) return IBERT_ERR_NOT_IMPLEMENTED;
        g.gelu = GeluConst{gelu->q_b, gelu->q_c, gelu->q_1, gelu->q_max, gelu->out.m, gelu->out.s};
        g.gelu_fast = gelu_fast_ok(*gelu) ? 1 : 0;
        gelu_table_range(*gelu, &g.gelu_lut_lo, &g.gelu_lut_n);
    }
    g.c_vec = aligned(C, i8 ? 4 : (g.c16 ? 8 : 16)) && d.ldc % 4 == 0 && d.strideC_outer % 4 == 0 && d.strideC_inner % 4 == 0;
    g.c_vec16 = i8 && aligned(C, 16) && d.ldc % 16 == 0 && d.strideC_outer % 16 == 0 && d.strideC_inner % 16 == 0;
    g.r_vec = residual && aligned(residual, 16) && d.ldr % 16 == 0 && d.strideR_outer % 16 == 0 && d.strideR_inner % 16 == 0;

    const bool fast = d.trans_w == 0 && d.K > 0 && aligned(A, 16) && aligned(W, 16) && d.lda % 16 == 0 && d.ldw % 16 == 0 &&
                      d.strideA_outer % 16 == 0 && d.strideA_inner % 16 == 0 && d.strideW_outer % 16 == 0 &&
                      d.strideW_inner % 16 == 0;
    if (gelu && !(fast && d.K % 16 == 0)) return IBERT_ERR_NOT_IMPLEMENTED;
    if (fast) {
        if (d.K % 16 != 0) return launch_tail(g, i8, stream);       // bytewise K tail
        const int cfg = choose_config(d, nb, gelu != nullptr);
        if (gelu) {
            switch (cfg) {
                case 3: return launch_mfma<64, 64, 128, 3, false, false, true>(g, i8, stream);
                case 15: return launch_mfma<32, 32, 128, 4, false, false, true>(g, i8, stream);
                case 6: if (dma_ok(d, 256, 192)) return launch_mfma<256, 192, 128, 2, false, true, true>(g, i8, stream); break;
                case 7: if (dma_ok(d, 128, 128)) return launch_mfma<128, 128, 128, 2, false, true, true>(g, i8, stream); break;
                case 9: if (dma_ok(d, 128, 96)) return launch_mfma<128, 96, 128, 2, false, true, true>(g, i8, stream); break;
                case 10: if (dma_ok(d, 256, 128)) return launch_mfma<256, 128, 128, 2, false, true, true>(g, i8, stream); break;
                case 13: if (dma_ok(d, 256, 192)) return launch_mfma<256, 192, 128, 2, false, true, true, 8>(g, i8, stream); break;
                case 14: if (dma_ok(d, 256, 128)) return launch_mfma<256, 128, 128, 2, false, true, true, 8>(g, i8, stream); break;
                default: break;
            }
            return IBERT_ERR_NOT_IMPLEMENTED;
        }
        switch (cfg) {
            case 0: return launch_mfma<256, 192, 128, 2>(g, i8, stream);
            case 1: return launch_mfma<128, 128, 128, 2>(g, i8, stream);
            case 2: return launch_mfma<128, 128, 64, 2>(g, i8, stream);
            case 3: return launch_mfma<64, 64, 128, 3>(g, i8, stream);
            case 4: return launch_mfma<64, 128, 64, 3>(g, i8, stream);
            case 5: return launch_mfma<128, 96, 128, 2>(g, i8, stream);
            case 6: if (dma_ok(d, 256, 192)) return launch_mfma<256, 192, 128, 2, false, true>(g, i8, stream); break;
            case 7: if (dma_ok(d, 128, 128)) return launch_mfma<128, 128, 128, 2, false, true>(g, i8, stream); break;
            case 8: if (dma_ok(d, 256, 256)) return launch_mfma<256, 256, 128, 2, false, true>(g, i8, stream); break;
            case 9: if (dma_ok(d, 128, 96)) return launch_mfma<128, 96, 128, 2, false, true>(g, i8, stream); break;
            case 10: if (dma_ok(d, 256, 128)) return launch_mfma<256, 128, 128, 2, false, true>(g, i8, stream); break;
            case 11: if (dma_ok(d, 128, 96)) return launch_mfma<128, 96, 128, 3, false, true>(g, i8, stream); break;
            case 12: if (dma_ok(d, 128, 128)) return launch_mfma<128, 128, 128, 3, false, true>(g, i8, stream); break;
            case 13: if (dma_ok(d, 256, 192)) return launch_mfma<256, 192, 128, 2, false, true, false, 8>(g, i8, stream); break;
            case 14: if (dma_ok(d, 256, 128)) return launch_mfma<256, 128, 128, 2, false, true, false, 8>(g, i8, stream); break;
            case 15: return launch_mfma<32, 32, 128, 4>(g, i8, stream);
            case 16: if (dma_ok(d, 256, 256)) return launch_mfma<256, 256, 128, 2, false, true, false, 8>(g, i8, stream); break;
            case 17: if (dma_ok(d, 64, 96)) return launch_mfma<64, 96, 128, 3, false, true>(g, i8, stream); break;
            case 18: if (dma_ok(d, 64, 96)) return launch_mfma<64, 96, 128, 2, false, true>(g, i8, stream); break;
            case 19: if (dma_ok(d, 64, 128)) return launch_mfma<64, 128, 128, 2, false, true>(g, i8, stream); break;
            case 20: if (dma_ok(d, 128, 96)) return launch_mfma<128, 96, 128, 3, false, true, false, 8>(g, i8, stream); break;
            case 21: if (dma_ok(d, 128, 96)) return launch_mfma<128, 96, 128, 3, false, true, false, 8, 4>(g, i8, stream); break;
            case 22: if (dma_ok(d, 128, 128)) return launch_mfma<128, 128, 128, 3, false, true, false, 8, 4>(g, i8, stream); break;
            default: break;
        }
        return launch_mfma<128, 128, 64, 2>(g, i8, stream);
    }
    const bool fast_tw = d.trans_w == 1 && d.K > 0 && d.K % 16 == 0 && d.N >= 4 && d.N % 4 == 0 && aligned(A, 16) &&
                         aligned(W, 4) && d.lda % 16 == 0 && d.ldw % 4 == 0 && d.strideA_outer % 16 == 0 &&
                         d.strideA_inner % 16 == 0 && d.strideW_outer % 4 == 0 && d.strideW_inner % 4 == 0;
    if (fast_tw) {
        if (d.N <= 64) return launch_mfma<128, 64, 64, 2, true>(g, i8, stream);
        return launch_mfma<128, 128, 64, 2, true>(g, i8, stream);
    }
    const int64_t total = (int64_t)d.M * d.N * nb;
    const int64_t blocks = (total + GEMM_THREADS - 1) / GEMM_THREADS;
    if (blocks > 0x7fffffffLL) return IBERT_ERR_SHAPE;
    if (d.trans_w) {
        if (i8) hipLaunchKernelGGL((gemm_generic_kernel<true, true>), dim3((unsigned)blocks), dim3(GEMM_THREADS), 0, stream, g);
        else hipLaunchKernelGGL((gemm_generic_kernel<true, false>), dim3((unsigned)blocks), dim3(GEMM_THREADS), 0, stream, g);
    } else {
        if (i8) hipLaunchKernelGGL((gemm_generic_kernel<false, true>), dim3((unsigned)blocks), dim3(GEMM_THREADS), 0, stream, g);
        else hipLaunchKernelGGL((gemm_generic_kernel<false, false>), dim3((unsigned)blocks), dim3(GEMM_THREADS), 0, stream, g);
    }
    IBERT_LAUNCH_CHECK("gemm_generic_kernel");
    g_last_kernel = "gemm_generic_kernel";
    return IBERT_OK;
}

// MatMul + GELU.  One kernel when a direct-to-LDS tile fits the problem; otherwise the MatMul writes its INT32
// result (clamped to +-q_max) to `scratch` and the element-wise GELU kernel follows, which needs dense outputs.
int launch_gemm_gelu(const ibert_gemm_desc& d0, const int8_t* A, const int8_t* W, const int32_t* bias,
                     const int32_t* mult, const int32_t* shift, const ibert_gelu_params& gelu, int8_t* C,
                     int32_t* scratch, hipStream_t stream)
{
    ibert_gemm_desc d = d0;
    d.out_dtype = IBERT_I8;
    d.out_clamp = gelu.q_max;
    int rc = launch_gemm(d, A, W, bias, mult, shift, nullptr, C, stream, &gelu);
    if (rc != IBERT_ERR_NOT_IMPLEMENTED) return rc;
    const int64_t nb = (int64_t)d.batch_outer * d.batch_inner;
    const bool dense = d.ldc == d.N && (d.batch_inner == 1 || d.strideC_inner == (int64_t)d.M * d.N) &&
                       (d.batch_outer == 1 || d.strideC_outer == (int64_t)d.batch_inner * d.M * d.N);
    if (!dense) return IBERT_ERR_NOT_IMPLEMENTED;
    if (!scratch) return IBERT_ERR_WORKSPACE;
    d.out_dtype = IBERT_I32;
    rc = launch_gemm(d, A, W, bias, mult, shift, nullptr, scratch, stream);
    if (rc) return rc;
    return launch_gelu(scratch, C, nb * d.M * d.N, gelu, stream);
}

}  // namespace ibert


extern "C" int ibert_gemm_config_override(int32_t config)
{
    ibert::g_config_override = config;
    return ibert::kNumConfigs;
}


extern "C" void ibert_gemm_xcd_blocks(int32_t on) { ibert::g_xcd_blocks = on != 0; }

extern "C" void ibert_gemm_epilogue_record(uint32_t* device_word) { ibert::g_path_word = device_word; }

extern "C" int ibert_gemm_i8_requant(const ibert_gemm_desc* desc, const int8_t* A, const int8_t* W,
                                     const int32_t* bias, const int32_t* mult, const int32_t* shift,
                                     const int8_t* residual, void* C, void* stream)
{
    if (!desc) return IBERT_ERR_NULL;
    const int rc = ibert::check_gemm(*desc, A, W, mult, shift, residual, C);
    if (rc) return rc;
    return ibert::launch_gemm(*desc, A, W, bias, mult, shift, residual, C, (hipStream_t)stream);
}

extern "C" int ibert_gemm_i8_gelu(const ibert_gemm_desc* desc, const int8_t* A, const int8_t* W, const int32_t* bias,
                                  const int32_t* mult, const int32_t* shift, const ibert_gelu_params* gelu,
                                  int8_t* C, int32_t* scratch, void* stream)
{
    if (!desc || !gelu) return IBERT_ERR_NULL;
    int rc = ibert::check_gelu(*gelu);
    if (rc) return rc;
    ibert_gemm_desc d = *desc;
    d.out_dtype = IBERT_I32;                       // range checks of the MatMul part: an INT32 result clamped to q_max
    d.out_clamp = gelu->q_max;
    rc = ibert::check_gemm(d, A, W, mult, shift, nullptr, C);
    if (rc) return rc;
    return ibert::launch_gemm_gelu(*desc, A, W, bias, mult, shift, *gelu, C, scratch, (hipStream_t)stream);
}
