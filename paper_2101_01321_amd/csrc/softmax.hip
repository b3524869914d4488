// Integer-only Softmax (Alg. 3; Eq. 11-14).  HBM-bound: 4 bytes in, 1 (or 4) bytes out per element.
//
// Row kernel: a row is owned by LPR lanes (16, 32 or 64) of one wavefront and lives entirely in
// registers (NCH 16-byte chunks per lane), so HBM is read once and written once.  Row maximum and
// row sum are butterfly reductions inside the LPR-lane group.  Several rows share a wavefront when
// rows are short (cols <= 128 -> 4 rows per wave), which keeps all 64 lanes loading.
// Long rows (cols > 64*4*NCH_MAX) fall back to one workgroup per row with three passes.
#include "common.h"
#include "softmax_math.h"

namespace ibert {

struct SoftmaxArgs {
    const int32_t* x;
    void* y;
    int64_t rows;
    int32_t cols;
    int64_t ldx, ldy;
    SoftmaxConst c;
    const int32_t* key_lens;   // optional: row r keeps its first key_lens[r / rows_per_len] columns, the rest are masked
    int64_t rows_per_len;
};

// Number of columns of `row` that are real keys.  A masked column takes the logit INT32_MIN ("minus infinity"): its
// exponential is then zero unless the whole row sits at the bottom of the INT32 range.
__device__ __forceinline__ int32_t live_cols(const SoftmaxArgs& a, int64_t row)
{
    if (!a.key_lens) return a.cols;
    const int32_t n = a.key_lens[row / a.rows_per_len];
    return n < 1 ? 1 : (n > a.cols ? a.cols : n);
}

template <int LPR>
__device__ __forceinline__ int32_t group_max(int32_t v)
{
    return group_allreduce<LPR>(v, [](int32_t x, int32_t y) { return x > y ? x : y; });
}

template <int LPR>
__device__ __forceinline__ uint32_t group_sum(uint32_t v)
{
    return (uint32_t)group_allreduce<LPR>((int32_t)v, [](int32_t x, int32_t y) { return (int32_t)((uint32_t)x + (uint32_t)y); });
}

constexpr int SM_THREADS = 256;

// LPR lanes per row, NCH chunks of 4 elements per lane.  ALIGNED: rows start 16-byte aligned (x) and
// 4-byte aligned (int8 y) / 16-byte aligned (int32 y), so full chunks move as vectors.
template <int LPR, int NCH, bool ALIGNED, bool OUT_I8, bool FAST>
__global__ __launch_bounds__(SM_THREADS) void softmax_rows_kernel(SoftmaxArgs a)
{
    constexpr int ROWS_PER_BLOCK = SM_THREADS / LPR;
    const int lane = threadIdx.x % LPR;
    const int64_t row = (int64_t)blockIdx.x * ROWS_PER_BLOCK + threadIdx.x / LPR;
    const bool live = row < a.rows;
    const int32_t* xr = a.x + (live ? row : 0) * a.ldx;
    const int32_t nk = live_cols(a, live ? row : 0);

    int32_t q[NCH][4];
    int32_t mx = INT32_MIN;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int col = (c * LPR + lane) * 4;
        if (ALIGNED && live && col + 3 < a.cols) {
            const int4 v = *reinterpret_cast<const int4*>(xr + col);
            q[c][0] = col < nk ? v.x : INT32_MIN; q[c][1] = col + 1 < nk ? v.y : INT32_MIN;
            q[c][2] = col + 2 < nk ? v.z : INT32_MIN; q[c][3] = col + 3 < nk ? v.w : INT32_MIN;
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) q[c][e] = (live && col + e < nk) ? xr[col + e] : INT32_MIN;
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) mx = q[c][e] > mx ? q[c][e] : mx;
    }
    mx = group_max<LPR>(mx);

    // Padding lanes hold INT32_MIN: their difference is huge, so their e is zero unless the whole row is
    // INT32_MIN; they are masked explicitly to cover that case.
    uint32_t ex[NCH][4];
    uint32_t sum = 0;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int col = (c * LPR + lane) * 4;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t d = (uint32_t)mx - (uint32_t)q[c][e];
            const uint32_t v = FAST ? iexp_from_diff_fast(d, a.c) : iexp_from_diff(d, a.c);
            ex[c][e] = (col + e < a.cols) ? v : 0u;
            sum += ex[c][e];
        }
    }
    sum = group_sum<LPR>(sum);
    if (!live) return;
    const uint32_t Fz = 0x80000000u / sum;             // sum >= q_b^2 + q_c >= 1 (the maximum itself)

#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int col = (c * LPR + lane) * 4;
        uint32_t o[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            // FAST: e < 2^24 and Fz <= 2^23 (sum >= q_b^2 + q_c >= 2^8), so the 24-bit multiply is exact
            o[e] = FAST ? umad24(ex[c][e], Fz, 1u << (30 - a.c.k)) >> (31 - a.c.k) : normalise(ex[c][e], Fz, a.c.k);
            if (OUT_I8) o[e] = o[e] > 127u ? 127u : o[e];
        }
        if (OUT_I8) {
            int8_t* yr = reinterpret_cast<int8_t*>(a.y) + row * a.ldy;
            if (ALIGNED && col + 3 < a.cols) {
                *reinterpret_cast<uint32_t*>(yr + col) = o[0] | (o[1] << 8) | (o[2] << 16) | (o[3] << 24);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (col + e < a.cols) yr[col + e] = (int8_t)o[e];
            }
        } else {
            int32_t* yr = reinterpret_cast<int32_t*>(a.y) + row * a.ldy;
            if (ALIGNED && col + 3 < a.cols) {
                *reinterpret_cast<int4*>(yr + col) = make_int4((int)o[0], (int)o[1], (int)o[2], (int)o[3]);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (col + e < a.cols) yr[col + e] = (int32_t)o[e];
            }
        }
    }
}

// Long rows: one workgroup per row, three passes over the row (max, sum, output).
template <bool OUT_I8>
__global__ __launch_bounds__(SM_THREADS) void softmax_long_kernel(SoftmaxArgs a)
{
    __shared__ int32_t s_max[SM_THREADS / 64];
    __shared__ uint32_t s_sum[SM_THREADS / 64];
    const int64_t row = blockIdx.x;
    const int32_t* xr = a.x + row * a.ldx;
    const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
    const int32_t nk = live_cols(a, row);
    auto at = [&](int j) { return j < nk ? xr[j] : INT32_MIN; };

    int32_t mx = INT32_MIN;
    for (int j = threadIdx.x; j < nk; j += SM_THREADS) mx = xr[j] > mx ? xr[j] : mx;
    mx = group_max<64>(mx);
    if (lane == 0) s_max[wave] = mx;
    __syncthreads();
    mx = s_max[0];
#pragma unroll
    for (int w = 1; w < SM_THREADS / 64; ++w) mx = s_max[w] > mx ? s_max[w] : mx;

    uint32_t sum = 0;
    for (int j = threadIdx.x; j < a.cols; j += SM_THREADS) sum += iexp_from_diff((uint32_t)mx - (uint32_t)at(j), a.c);
    sum = group_sum<64>(sum);
    if (lane == 0) s_sum[wave] = sum;
    __syncthreads();
    sum = 0;
#pragma unroll
    for (int w = 0; w < SM_THREADS / 64; ++w) sum += s_sum[w];
    const uint32_t Fz = 0x80000000u / sum;

    for (int j = threadIdx.x; j < a.cols; j += SM_THREADS) {
        uint32_t o = normalise(iexp_from_diff((uint32_t)mx - (uint32_t)at(j), a.c), Fz, a.c.k);
        if (OUT_I8) {
            o = o > 127u ? 127u : o;
            (reinterpret_cast<int8_t*>(a.y) + row * a.ldy)[j] = (int8_t)o;
        } else {
            (reinterpret_cast<int32_t*>(a.y) + row * a.ldy)[j] = (int32_t)o;
        }
    }
}

int check_softmax(const ibert_softmax_params& p, int32_t cols)
{
    if (cols < 1) return IBERT_ERR_SHAPE;
    if (p.q_ln2 < 1 || p.q_b < 1 || p.q_c < 0 || p.out_frac_bits < 0) return IBERT_ERR_PARAM_RANGE;
    if (p.q_ln2 > p.q_b) return IBERT_ERR_PARAM_RANGE;   // ln2 < b: keeps q_b - r in (0, q_b]
    if (p.out_dtype == IBERT_I8) {
        if (p.out_frac_bits > 7) return IBERT_ERR_PARAM_RANGE;
    } else if (p.out_dtype == IBERT_I32) {
        if (p.out_frac_bits > 30) return IBERT_ERR_PARAM_RANGE;
    } else {
        return IBERT_ERR_PARAM_RANGE;
    }
    const __int128 top = (__int128)p.q_b * p.q_b + p.q_c;
    if (top * cols >= ((__int128)1 << 31)) return IBERT_ERR_PARAM_RANGE;
    return IBERT_OK;
}

template <int LPR, int NCH>
static void launch_rows(const SoftmaxArgs& a, bool al, bool i8, bool fast, hipStream_t stream)
{
    constexpr int rpb = SM_THREADS / LPR;
    const dim3 grid((unsigned)((a.rows + rpb - 1) / rpb)), block(SM_THREADS);
    if (al && i8 && fast) {                 // the layer's case
        hipLaunchKernelGGL((softmax_rows_kernel<LPR, NCH, true, true, true>), grid, block, 0, stream, a);
    } else if (al && i8) {
        hipLaunchKernelGGL((softmax_rows_kernel<LPR, NCH, true, true, false>), grid, block, 0, stream, a);
    } else if (al) {
        hipLaunchKernelGGL((softmax_rows_kernel<LPR, NCH, true, false, false>), grid, block, 0, stream, a);
    } else if (i8) {
        hipLaunchKernelGGL((softmax_rows_kernel<LPR, NCH, false, true, false>), grid, block, 0, stream, a);
    } else {
        hipLaunchKernelGGL((softmax_rows_kernel<LPR, NCH, false, false, false>), grid, block, 0, stream, a);
    }
}

int launch_softmax(const int32_t* x, void* y, int64_t rows, int32_t cols, int64_t ldx, int64_t ldy,
                   const ibert_softmax_params& p, hipStream_t stream, const int32_t* key_lens, int64_t rows_per_len)
{
    if (rows == 0) return IBERT_OK;
    SoftmaxArgs a;
    a.x = x; a.y = y; a.rows = rows; a.cols = cols; a.ldx = ldx; a.ldy = ldy;
    a.key_lens = key_lens; a.rows_per_len = rows_per_len > 0 ? rows_per_len : 1;
    a.c = softmax_const(p);
    const bool i8 = p.out_dtype == IBERT_I8;
    const bool fast = softmax_fast_ok(p);
    const bool al = aligned(x, 16) && ldx % 4 == 0 && (i8 ? (aligned(y, 4) && ldy % 4 == 0) : (aligned(y, 16) && ldy % 4 == 0));
    if (rows > 0x7fffffffLL) return IBERT_ERR_SHAPE;

    if (cols <= 16 * 4) launch_rows<16, 1>(a, al, i8, fast, stream);
    else if (cols <= 16 * 8) launch_rows<16, 2>(a, al, i8, fast, stream);
    else if (cols <= 32 * 8) launch_rows<32, 2>(a, al, i8, fast, stream);
    else if (cols <= 64 * 8) launch_rows<64, 2>(a, al, i8, fast, stream);
    else if (cols <= 64 * 16) launch_rows<64, 4>(a, al, i8, fast, stream);
    else if (cols <= 64 * 32) launch_rows<64, 8>(a, al, i8, fast, stream);
    else {
        if (i8) hipLaunchKernelGGL(softmax_long_kernel<true>, dim3((unsigned)rows), dim3(SM_THREADS), 0, stream, a);
        else hipLaunchKernelGGL(softmax_long_kernel<false>, dim3((unsigned)rows), dim3(SM_THREADS), 0, stream, a);
    }
    IBERT_LAUNCH_CHECK("softmax kernel");
    g_last_kernel = cols <= 64 * 32 ? "softmax_rows_kernel" : "softmax_long_kernel";
    return IBERT_OK;
}

}  // namespace ibert

extern "C" int ibert_softmax_i(const int32_t* x, void* y, int64_t rows, int32_t cols, int64_t ldx, int64_t ldy,
                               const ibert_softmax_params* params, void* stream)
{
    if (!params) return IBERT_ERR_NULL;
    if (rows < 0 || cols < 1 || ldx < cols || ldy < cols) return IBERT_ERR_SHAPE;
    const int rc = ibert::check_softmax(*params, cols);
    if (rc) return rc;
    if (rows == 0) return IBERT_OK;
    if (!x || !y) return IBERT_ERR_NULL;
    return ibert::launch_softmax(x, y, rows, cols, ldx, ldy, *params, (hipStream_t)stream);
}

extern "C" int ibert_softmax_masked_i(const int32_t* x, void* y, int64_t rows, int32_t cols, int64_t ldx, int64_t ldy,
                                      const ibert_softmax_params* params, const int32_t* key_lens, int64_t rows_per_len,
                                      void* stream)
{
    if (!params) return IBERT_ERR_NULL;
    if (rows < 0 || cols < 1 || ldx < cols || ldy < cols || rows_per_len < 1) return IBERT_ERR_SHAPE;
    const int rc = ibert::check_softmax(*params, cols);
    if (rc) return rc;
    if (rows == 0) return IBERT_OK;
    if (!x || !y || !key_lens) return IBERT_ERR_NULL;
    return ibert::launch_softmax(x, y, rows, cols, ldx, ldy, *params, (hipStream_t)stream, key_lens, rows_per_len);
}
