// INT8 x INT8 -> INT32 MatMul (Sec. 1 third contribution, App. C.1) with bias, dyadic requantization,
// optional residual and clamp fused into the epilogue.
//
// Fast path (W is [N,K], rows 16-byte aligned): LDS-staged tiles feeding v_mfma_i32_16x16x64_i8.
//   * The weight rows are fed as the MFMA "A" operand and the activation rows as the "B" operand, so
//     that each lane ends up with four consecutive output channels n of one token m: the epilogue
//     packs them into one dword (INT8 out) or one 16-byte store (INT32 out).
//   * Both operands are K-contiguous in memory; a lane's MFMA operand is 16 consecutive K bytes, one
//     ds_read_b128.  LDS rows are 64 bytes with the 16-byte chunk index XOR-swizzled by the row so that
//     the 16 rows a quarter-wave reads in one instruction fall into distinct banks.
//   * Integer accumulation is exact, so any consistent K order gives the oracle's bits.
// Generic path (W is [K,N], or unaligned operands): one output element per lane, byte loads.
#include "common.h"

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
    int32_t c_vec;     // INT32 output rows allow 16-byte stores / INT8 rows allow dword stores
    int32_t r_vec;     // residual rows allow dword loads
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
// ---------------------------------------------------------------------------------------------
constexpr int GEMM_THREADS = 256;
constexpr int BK = 64;

__device__ __forceinline__ int swz(int row) { return ((row >> 1) & 3) ^ ((row >> 3) & 1); }

// 16 bytes of row `p` starting at column k; bytes at or beyond K read as zero.
__device__ __forceinline__ v4i load_chunk(const int8_t* p, int k, int K, bool row_ok)
{
    v4i r = {0, 0, 0, 0};
    if (!row_ok || k >= K) return r;
    if (k + 16 <= K) return *reinterpret_cast<const v4i*>(p + k);
    union { v4i v; int8_t b[16]; } u;
    u.v = r;
    for (int i = 0; i < 16; ++i)
        if (k + i < K) u.b[i] = p[k + i];
    return u.v;
}

template <int BM, int BN, int WAVES_M, int WAVES_N, bool OUT_I8>
__global__ __launch_bounds__(GEMM_THREADS) void gemm_nt_mfma_kernel(GemmArgs g)
{
    static_assert(WAVES_M * WAVES_N == GEMM_THREADS / 64, "four waves");
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    constexpr int FM = WM / 16, FN = WN / 16;
    constexpr int LA = BM / 64, LW = BN / 64;          // 16-byte chunks per lane per K step
    static_assert(BM % 64 == 0 && BN % 64 == 0 && WM % 16 == 0 && WN % 16 == 0, "tile shape");

    __shared__ __attribute__((aligned(16))) int8_t lds_a[2][BM * BK];
    __shared__ __attribute__((aligned(16))) int8_t lds_w[2][BN * BK];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave % WAVES_M) * WM, wn0 = (wave / WAVES_M) * WN;

    // tile coordinates: consecutive workgroups walk along N inside one M panel
    int bid = blockIdx.x;
    const int tiles = g.tiles_m * g.tiles_n;
    const int z = bid / tiles;
    bid -= z * tiles;
    const int tm = bid / g.tiles_n, tn = bid - tm * g.tiles_n;
    const int m0 = tm * BM, n0 = tn * BN;
    const int zo = z / g.batch_inner, zi = z - zo * g.batch_inner;

    const int8_t* A = g.A + zo * g.sA_o + zi * g.sA_i;
    const int8_t* W = g.W + zo * g.sW_o + zi * g.sW_i;

    const int lrow = tid >> 2, lch = tid & 3;          // this lane's (row, chunk) inside a 64-row slab
    v4i ra[LA], rw[LW];

    auto load_global = [&](int kt) {
        const int k = kt * BK + lch * 16;
#pragma unroll
        for (int i = 0; i < LA; ++i) {
            const int row = m0 + i * 64 + lrow;
            ra[i] = load_chunk(A + (int64_t)row * g.lda, k, g.K, row < g.M);
        }
#pragma unroll
        for (int i = 0; i < LW; ++i) {
            const int row = n0 + i * 64 + lrow;
            rw[i] = load_chunk(W + (int64_t)row * g.ldw, k, g.K, row < g.N);
        }
    };
    auto store_lds = [&](int buf) {
#pragma unroll
        for (int i = 0; i < LA; ++i) {
            const int row = i * 64 + lrow;
            *reinterpret_cast<v4i*>(&lds_a[buf][row * BK + ((lch ^ swz(row)) << 4)]) = ra[i];
        }
#pragma unroll
        for (int i = 0; i < LW; ++i) {
            const int row = i * 64 + lrow;
            *reinterpret_cast<v4i*>(&lds_w[buf][row * BK + ((lch ^ swz(row)) << 4)]) = rw[i];
        }
    };

    v4i acc[FN][FM];
#pragma unroll
    for (int i = 0; i < FN; ++i)
#pragma unroll
        for (int j = 0; j < FM; ++j) acc[i][j] = v4i{0, 0, 0, 0};

    const int nk = (g.K + BK - 1) / BK;
    const int frow = lane & 15, fch = lane >> 4;       // MFMA operand: row within the 16-block, K chunk
    if (nk > 0) {
        load_global(0);
        store_lds(0);
    }
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < nk) load_global(kt + 1);
        v4i xa[FM], wb[FN];
#pragma unroll
        for (int j = 0; j < FM; ++j) {
            const int row = wm0 + j * 16 + frow;
            xa[j] = *reinterpret_cast<const v4i*>(&lds_a[buf][row * BK + ((fch ^ swz(row)) << 4)]);
        }
#pragma unroll
        for (int i = 0; i < FN; ++i) {
            const int row = wn0 + i * 16 + frow;
            wb[i] = *reinterpret_cast<const v4i*>(&lds_w[buf][row * BK + ((fch ^ swz(row)) << 4)]);
        }
#pragma unroll
        for (int i = 0; i < FN; ++i)
#pragma unroll
            for (int j = 0; j < FM; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wb[i], xa[j], acc[i][j], 0, 0, 0);
        if (kt + 1 < nk) store_lds(buf ^ 1);
        __syncthreads();
    }

    // Epilogue.  acc[i][j][r] = C[m0 + wm0 + 16 j + lane%16][n0 + wn0 + 16 i + 4 (lane/16) + r].
    const int64_t c_off = zo * g.sC_o + zi * g.sC_i;
    const int8_t* R = g.R ? g.R + zo * g.sR_o + zi * g.sR_i : nullptr;
#pragma unroll
    for (int i = 0; i < FN; ++i) {
        const int n = n0 + wn0 + i * 16 + fch * 4;
        if (n >= g.N) continue;
        int32_t bs[4], ml[4], sh[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int nn = n + r < g.N ? n + r : g.N - 1;
            bs[r] = g.bias ? g.bias[nn] : 0;
            ml[r] = g.per_channel ? g.mult[nn] : g.dy_m;
            sh[r] = g.per_channel ? g.shift[nn] : g.dy_s;
        }
        const bool full = n + 3 < g.N;
#pragma unroll
        for (int j = 0; j < FM; ++j) {
            const int m = m0 + wm0 + j * 16 + frow;
            if (m >= g.M) continue;
            int32_t res[4] = {0, 0, 0, 0};
            if (R) {
                const int8_t* rp = R + (int64_t)m * g.ldr + n;
                if (full && g.r_vec) {
                    const uint32_t pk = *reinterpret_cast<const uint32_t*>(rp);
                    res[0] = (int8_t)(pk & 0xff); res[1] = (int8_t)((pk >> 8) & 0xff);
                    res[2] = (int8_t)((pk >> 16) & 0xff); res[3] = (int8_t)(pk >> 24);
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (n + r < g.N) res[r] = rp[r];
                }
            }
            int32_t o[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) o[r] = finish(acc[i][j][r] + bs[r], ml[r], sh[r], R != nullptr, res[r], g);
            const int64_t off = c_off + (int64_t)m * g.ldc + n;
            if (OUT_I8) {
                int8_t* cp = reinterpret_cast<int8_t*>(g.C) + off;
                if (full && g.c_vec) {
                    *reinterpret_cast<uint32_t*>(cp) = pack4_i8(o[0], o[1], o[2], o[3]);
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (n + r < g.N) cp[r] = (int8_t)o[r];
                }
            } else {
                int32_t* cp = reinterpret_cast<int32_t*>(g.C) + off;
                if (full && g.c_vec) {
                    *reinterpret_cast<int4*>(cp) = make_int4(o[0], o[1], o[2], o[3]);
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (n + r < g.N) cp[r] = o[r];
                }
            }
        }
    }
}

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
    else reinterpret_cast<int32_t*>(g.C)[off] = o;
}

// ---------------------------------------------------------------------------------------------
int check_gemm(const ibert_gemm_desc& d, const void* A, const void* W, const void* mult, const void* shift,
               const void* residual, const void* C)
{
    (void)residual;
    if (d.M < 0 || d.N < 0 || d.K < 0 || d.batch_outer < 0 || d.batch_inner < 0) return IBERT_ERR_SHAPE;
    if (d.K > (1 << 17)) return IBERT_ERR_SHAPE;
    if (d.out_dtype != IBERT_I8 && d.out_dtype != IBERT_I32) return IBERT_ERR_PARAM_RANGE;
    if (d.out_clamp < 0 || (d.out_dtype == IBERT_I8 && d.out_clamp > 127)) return IBERT_ERR_PARAM_RANGE;
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

template <int BM, int BN, int WAVES_M, int WAVES_N>
static int launch_mfma(GemmArgs& g, bool i8, hipStream_t stream)
{
    g.tiles_m = (g.M + BM - 1) / BM;
    g.tiles_n = (g.N + BN - 1) / BN;
    const int64_t blocks = (int64_t)g.tiles_m * g.tiles_n * g.nbatch;
    if (blocks > 0x7fffffffLL) return IBERT_ERR_SHAPE;
    if (i8)
        hipLaunchKernelGGL((gemm_nt_mfma_kernel<BM, BN, WAVES_M, WAVES_N, true>), dim3((unsigned)blocks),
                           dim3(GEMM_THREADS), 0, stream, g);
    else
        hipLaunchKernelGGL((gemm_nt_mfma_kernel<BM, BN, WAVES_M, WAVES_N, false>), dim3((unsigned)blocks),
                           dim3(GEMM_THREADS), 0, stream, g);
    IBERT_LAUNCH_CHECK("gemm_nt_mfma_kernel");
    g_last_kernel = "gemm_nt_mfma_kernel";
    return IBERT_OK;
}

int launch_gemm(const ibert_gemm_desc& d, const int8_t* A, const int8_t* W, const int32_t* bias,
                const int32_t* mult, const int32_t* shift, const int8_t* residual, void* C, hipStream_t stream)
{
    const int64_t nb = (int64_t)d.batch_outer * d.batch_inner;
    if (nb == 0 || d.M == 0 || d.N == 0) return IBERT_OK;
    GemmArgs g;
    g.A = A; g.W = W; g.bias = bias; g.mult = mult; g.shift = shift; g.R = residual; g.C = C;
    g.M = d.M; g.N = d.N; g.K = d.K;
    g.batch_inner = d.batch_inner; g.nbatch = (int32_t)nb;
    g.tiles_m = g.tiles_n = 0;
    g.lda = d.lda; g.ldw = d.ldw; g.ldc = d.ldc; g.ldr = d.ldr;
    g.sA_o = d.strideA_outer; g.sA_i = d.strideA_inner;
    g.sW_o = d.strideW_outer; g.sW_i = d.strideW_inner;
    g.sC_o = d.strideC_outer; g.sC_i = d.strideC_inner;
    g.sR_o = d.strideR_outer; g.sR_i = d.strideR_inner;
    g.per_channel = d.per_channel ? 1 : 0;
    g.dy_m = d.requant.m; g.dy_s = d.requant.s;
    g.out_clamp = d.out_clamp;
    g.res_m = d.residual_dy.m; g.res_s = d.residual_dy.s;
    const bool i8 = d.out_dtype == IBERT_I8;
    const size_t calign = i8 ? 4 : 16;
    const int64_t cmod = i8 ? 4 : 4;                   // elements: 4 bytes (int8) or 16 bytes (int32)
    g.c_vec = aligned(C, calign) && d.ldc % cmod == 0 && d.strideC_outer % cmod == 0 && d.strideC_inner % cmod == 0;
    g.r_vec = residual && aligned(residual, 4) && d.ldr % 4 == 0 && d.strideR_outer % 4 == 0 && d.strideR_inner % 4 == 0;

    const bool fast = d.trans_w == 0 && aligned(A, 16) && aligned(W, 16) && d.lda % 16 == 0 && d.ldw % 16 == 0 &&
                      d.strideA_outer % 16 == 0 && d.strideA_inner % 16 == 0 && d.strideW_outer % 16 == 0 &&
                      d.strideW_inner % 16 == 0;
    if (fast) {
        if (d.N <= 64) return launch_mfma<128, 64, 4, 1>(g, i8, stream);
        return launch_mfma<128, 128, 2, 2>(g, i8, stream);
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

}  // namespace ibert

extern "C" int ibert_gemm_i8_requant(const ibert_gemm_desc* desc, const int8_t* A, const int8_t* W,
                                     const int32_t* bias, const int32_t* mult, const int32_t* shift,
                                     const int8_t* residual, void* C, void* stream)
{
    if (!desc) return IBERT_ERR_NULL;
    const int rc = ibert::check_gemm(*desc, A, W, mult, shift, residual, C);
    if (rc) return rc;
    return ibert::launch_gemm(*desc, A, W, bias, mult, shift, residual, C, (hipStream_t)stream);
}
