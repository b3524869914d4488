// ibert_encoder_layer_i / ibert_encoder_i: the ten-step post-LN encoder layer as a sequence of
// kernel launches on one stream (Fig. 1 right; Sec. 4.1; App. C.1).  Host code only: validation,
// workspace carving, enqueueing.  No allocation, no synchronisation.
#include <cstring>
#include <mutex>

#include "common.h"

namespace ibert {

// Workspace of the layer call that takes none from its caller: one array in the library's own device image, so that
// nothing is allocated at run time.  Every GPU the library runs on holds its own copy (at its own address) until the
// process ends.  Host code must not use the array's name as an address: it asks the runtime for the copy's address
// once per device (static_scratch_address) and uses that pointer from then on.
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];          // per device: address of that device's copy of `scratch`
static std::mutex g_scratch_mutex;

// Address of the current device's copy of `scratch`; looked up on the first call on each device.
static int static_scratch_address(void** out)
{
    int dev = -1;
    IBERT_HIP_CHECK(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return IBERT_ERR_NOT_IMPLEMENTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        IBERT_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p || !aligned(p, 256)) return IBERT_ERR_WORKSPACE;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return IBERT_OK;
}

static size_t align_up(size_t v) { return (v + 255) & ~(size_t)255; }

// ---- optional per-step event profile ----------------------------------------------------------
struct StepMeta {
    int32_t step;
    double ops, bytes;
    const char* kernel;
};
static struct {
    bool open = false;
    int32_t capacity = 0, count = 0;
    hipEvent_t* ev = nullptr;      // 2 * capacity events: [2i] before, [2i+1] after step record i
    StepMeta* meta = nullptr;
} g_prof;

static void prof_before(hipStream_t s)
{
    if (g_prof.open && g_prof.count < g_prof.capacity) (void)hipEventRecord(g_prof.ev[2 * g_prof.count], s);
}
static void prof_after(hipStream_t s, int32_t step, double ops, double bytes)
{
    if (g_prof.open && g_prof.count < g_prof.capacity) {
        (void)hipEventRecord(g_prof.ev[2 * g_prof.count + 1], s);
        g_prof.meta[g_prof.count] = StepMeta{step, ops, bytes, g_last_kernel};
        g_prof.count += 1;
    }
}

// Algorithmic bytes of a MatMul step: each operand read once, the output written once, 12 bytes of
// per-channel constants per output column.
static double gemm_bytes(double M, double N, double K, double batch, double out_size, bool residual, bool w_shared)
{
    return batch * (M * K + (w_shared ? 0.0 : N * K) + M * N * out_size + (residual ? M * N : 0.0)) +
           (w_shared ? N * K : 0.0) + 12.0 * N;
}

static int layout(int32_t batch, int32_t seq, int32_t hidden, int32_t heads, int32_t ffn,
                  ibert_layer_workspace_layout* o)
{
    if (batch < 1 || seq < 1 || hidden < 1 || heads < 1 || ffn < 1 || hidden % heads) return IBERT_ERR_SHAPE;
    const size_t T = (size_t)batch * seq, H = hidden, F = ffn, BH = (size_t)batch * heads, L = seq;
    size_t p = 0;
    o->qkv = p;    p += align_up(T * 3 * H);
    o->scores = p; p += align_up(BH * L * L * 4);
    o->probs = p;  p += align_up(BH * L * L);
    o->ctx = p;    p += align_up(T * H);
    o->r1 = p;     p += align_up(T * H * 4);
    o->h1 = p;     p += align_up(T * H);
    o->f1 = p;     p += align_up(T * F * 4);
    o->g = p;      p += align_up(T * F);
    o->r2 = p;     p += align_up(T * H * 4);
    o->total = p;
    return IBERT_OK;
}

// Steps 2-4 (scores, Softmax, context) as three kernels through the INT32 scores and INT8 probabilities buffers.
static int run_attention_unfused(const int8_t* qkv, int32_t* scores, int8_t* probs, int8_t* ctx, int64_t B, int64_t L,
                                 int64_t H, int64_t nh, const ibert_dyadic& scores_dy, const ibert_softmax_params& softmax,
                                 const ibert_dyadic& ctx_dy, const int32_t* key_lens, hipStream_t stream)
{
    const int64_t dh = H / nh;
    ibert_gemm_desc d;
    int rc;
#define RUN_GEMM(A_, W_, b_, m_, s_, R_, C_)                                             \
    do {                                                                                 \
        rc = check_gemm(d, A_, W_, m_, s_, R_, C_);                                      \
        if (rc) return rc;                                                               \
        rc = launch_gemm(d, A_, W_, b_, m_, s_, R_, C_, stream);                         \
        if (rc) return rc;                                                               \
    } while (0)
    // 2: attention scores Q_h K_h^T per (batch, head); 1/sqrt(d) is inside scores_dy
    std::memset(&d, 0, sizeof d);
    d.M = (int32_t)L; d.N = (int32_t)L; d.K = (int32_t)dh; d.batch_outer = (int32_t)B; d.batch_inner = (int32_t)nh;
    d.lda = 3 * H; d.ldw = 3 * H; d.ldc = L;
    d.strideA_outer = L * 3 * H; d.strideA_inner = dh;
    d.strideW_outer = L * 3 * H; d.strideW_inner = dh;
    d.strideC_outer = nh * L * L; d.strideC_inner = L * L;
    d.per_channel = 0; d.requant = scores_dy; d.out_dtype = IBERT_I32; d.out_clamp = 2147483647;
    prof_before(stream);
    RUN_GEMM(qkv, qkv + H, nullptr, nullptr, nullptr, nullptr, scores);
    prof_after(stream, 2, 2.0 * B * nh * L * L * dh, gemm_bytes(L, L, dh, B * nh, 4, false, false));

    // 3: softmax over the key axis (the nh*L rows of sequence b keep key_lens[b] keys)
    prof_before(stream);
    rc = launch_softmax(scores, probs, B * nh * L, (int32_t)L, L, L, softmax, stream, key_lens, nh * L);
    if (rc) return rc;
    prof_after(stream, 3, 0.0, 5.0 * B * nh * L * L);

    // 4: context P V_h, scattered back into [T, H]
    std::memset(&d, 0, sizeof d);
    d.M = (int32_t)L; d.N = (int32_t)dh; d.K = (int32_t)L; d.batch_outer = (int32_t)B; d.batch_inner = (int32_t)nh;
    d.lda = L; d.ldw = 3 * H; d.ldc = H; d.trans_w = 1;
    d.strideA_outer = nh * L * L; d.strideA_inner = L * L;
    d.strideW_outer = L * 3 * H; d.strideW_inner = dh;
    d.strideC_outer = L * H; d.strideC_inner = dh;
    d.per_channel = 0; d.requant = ctx_dy; d.out_dtype = IBERT_I8; d.out_clamp = 127;
    prof_before(stream);
    RUN_GEMM(probs, qkv + 2 * H, nullptr, nullptr, nullptr, nullptr, ctx);
    prof_after(stream, 4, 2.0 * B * nh * L * dh * L, gemm_bytes(L, dh, L, B * nh, 1, false, false));

    return IBERT_OK;
#undef RUN_GEMM
}

// Steps 2-4: one kernel where the shape allows it (and `fused` asks for it), else the three-kernel route.
static int run_attention(const int8_t* qkv, int32_t* scores, int8_t* probs, int8_t* ctx, int64_t B, int64_t L, int64_t H,
                         int64_t nh, const ibert_dyadic& scores_dy, const ibert_softmax_params& softmax,
                         const ibert_dyadic& ctx_dy, const int32_t* key_lens, bool fused, hipStream_t stream)
{
    if (fused && attention_fused_ok(qkv, ctx, (int32_t)L, (int32_t)H, (int32_t)nh)) {
        prof_before(stream);
        const int rc = launch_attention(qkv, ctx, (int32_t)B, (int32_t)L, (int32_t)H, (int32_t)nh, scores_dy, softmax,
                                        ctx_dy, stream, key_lens);
        if (rc) return rc;
        // both MatMuls; bytes: Q, K, V read once, the context written once
        prof_after(stream, 2, 4.0 * B * nh * L * L * (H / nh), 4.0 * B * L * H);
        return IBERT_OK;
    }
    if (!scores || !probs) return IBERT_ERR_WORKSPACE;
    return run_attention_unfused(qkv, scores, probs, ctx, B, L, H, nh, scores_dy, softmax, ctx_dy, key_lens, stream);
}

static int run_layer(const ibert_layer_weights& w, const ibert_layer_quant& q, const int8_t* x, int8_t* y,
                     int32_t batch, int32_t seq, int32_t hidden, int32_t heads, int32_t ffn, const int32_t* key_lens,
                     char* ws, const ibert_layer_workspace_layout& lo, hipStream_t stream)
{
    const int64_t B = batch, L = seq, H = hidden, nh = heads, F = ffn, T = B * L, dh = H / nh;
    int8_t* qkv = reinterpret_cast<int8_t*>(ws + lo.qkv);
    int32_t* scores = reinterpret_cast<int32_t*>(ws + lo.scores);
    int8_t* probs = reinterpret_cast<int8_t*>(ws + lo.probs);
    int8_t* ctx = reinterpret_cast<int8_t*>(ws + lo.ctx);
    int32_t* r1 = reinterpret_cast<int32_t*>(ws + lo.r1);
    int8_t* h1 = reinterpret_cast<int8_t*>(ws + lo.h1);
    int32_t* f1 = reinterpret_cast<int32_t*>(ws + lo.f1);
    int8_t* g = reinterpret_cast<int8_t*>(ws + lo.g);
    int32_t* r2 = reinterpret_cast<int32_t*>(ws + lo.r2);

    const bool fuse_gelu = !(q.route & IBERT_ROUTE_SEPARATE_GELU);
    const bool fuse_attention = !(q.route & IBERT_ROUTE_SEPARATE_ATTENTION);
    const bool half = !(q.route & IBERT_ROUTE_I32_LN_INPUT);       // r1 / r2 as int16: half the bytes both ways

    ibert_gemm_desc d;
    int rc;
#define RUN_GEMM(A_, W_, b_, m_, s_, R_, C_)                                             \
    do {                                                                                 \
        rc = check_gemm(d, A_, W_, m_, s_, R_, C_);                                      \
        if (rc) return rc;                                                               \
        rc = launch_gemm(d, A_, W_, b_, m_, s_, R_, C_, stream);                         \
        if (rc) return rc;                                                               \
    } while (0)
    // A projection with residual (INT32 at the LayerNorm input scale, stored in 16 or 32 bits) and its LayerNorm.
#define RUN_GEMM_LN(STEP_, A_, W_, b_, m_, s_, R_, R32_, GQ_, BQ_, SH_, OUT_, OPS_, K_)                        \
    do {                                                                                                     \
        if (half) d.out_dtype = IBERT_I16;                                                                   \
        prof_before(stream);                                                                                 \
        RUN_GEMM(A_, W_, b_, m_, s_, R_, R32_);                                                              \
        prof_after(stream, STEP_, OPS_, gemm_bytes(T, H, K_, 1, half ? 2 : 4, true, true));                  \
        prof_before(stream);                                                                                 \
        if (half)                                                                                            \
            rc = launch_layernorm16(reinterpret_cast<const int16_t*>(R32_), OUT_, T, (int32_t)H, H, H,       \
                                    GQ_, BQ_, SH_, stream);                                                  \
        else                                                                                                 \
            rc = launch_layernorm(R32_, OUT_, T, (int32_t)H, H, H, GQ_, BQ_, SH_, stream);                   \
        if (rc) return rc;                                                                                   \
        prof_after(stream, (STEP_) + 1, 0.0, (half ? 3.0 : 5.0) * T * H);                                    \
    } while (0)

    // 1: QKV projection, one GEMM with N = 3H
    std::memset(&d, 0, sizeof d);
    d.M = (int32_t)T; d.N = (int32_t)(3 * H); d.K = (int32_t)H; d.batch_outer = d.batch_inner = 1;
    d.lda = H; d.ldw = H; d.ldc = 3 * H; d.per_channel = 1; d.out_dtype = IBERT_I8; d.out_clamp = 127;
    prof_before(stream);
    RUN_GEMM(x, w.w_qkv, w.b_qkv, w.m_qkv, w.s_qkv, nullptr, qkv);
    prof_after(stream, 1, 2.0 * T * 3 * H * H, gemm_bytes(T, 3 * H, H, 1, 1, false, true));

    // 2-4: attention scores, Softmax, context
    rc = run_attention(qkv, scores, probs, ctx, B, L, H, nh, q.scores_dy, q.softmax, q.ctx_dy, key_lens,
                       fuse_attention, stream);
    if (rc) return rc;

    // 5: output projection + residual x, INT32 at the LayerNorm input scale
    std::memset(&d, 0, sizeof d);
    d.M = (int32_t)T; d.N = (int32_t)H; d.K = (int32_t)H; d.batch_outer = d.batch_inner = 1;
    d.lda = H; d.ldw = H; d.ldc = H; d.ldr = H; d.per_channel = 1; d.out_dtype = IBERT_I32; d.out_clamp = 32767;
    d.residual_dy = q.res1_dy;
    // (+ 6: LayerNorm)
    RUN_GEMM_LN(5, ctx, w.w_o, w.b_o, w.m_o, w.s_o, x, r1, w.ln1_gamma_q, w.ln1_beta_q, q.ln1_shift, h1, 2.0 * T * H * H, H);

    // 7: FFN up-projection, INT32 at the GELU input scale
    std::memset(&d, 0, sizeof d);
    d.M = (int32_t)T; d.N = (int32_t)F; d.K = (int32_t)H; d.batch_outer = d.batch_inner = 1;
    d.lda = H; d.ldw = H; d.ldc = F; d.per_channel = 1; d.out_dtype = IBERT_I32; d.out_clamp = q.gelu.q_max;
    bool fused78 = false;
    if (fuse_gelu) {
        // 7+8 in one kernel when a tile fits: f1 is then never written
        rc = check_gemm(d, h1, w.w_1, w.m_1, w.s_1, nullptr, g);
        if (rc) return rc;
        prof_before(stream);
        ibert_gemm_desc df = d;
        df.out_dtype = IBERT_I8;                                   // what the kernel stores; the clamp stays q_max
        rc = launch_gemm(df, h1, w.w_1, w.b_1, w.m_1, w.s_1, nullptr, g, stream, &q.gelu);
        if (rc == IBERT_OK) {
            fused78 = true;
            prof_after(stream, 7, 2.0 * T * F * H, gemm_bytes(T, F, H, 1, 1, false, true));
        } else if (rc != IBERT_ERR_NOT_IMPLEMENTED) {
            return rc;
        }
    }
    if (!fused78) {
        prof_before(stream);
        RUN_GEMM(h1, w.w_1, w.b_1, w.m_1, w.s_1, nullptr, f1);
        prof_after(stream, 7, 2.0 * T * F * H, gemm_bytes(T, F, H, 1, 4, false, true));

        // 8: GELU
        prof_before(stream);
        rc = launch_gelu(f1, g, T * F, q.gelu, stream);
        if (rc) return rc;
        prof_after(stream, 8, 0.0, 5.0 * T * F);
    }

    // 9: FFN down-projection + residual h1
    std::memset(&d, 0, sizeof d);
    d.M = (int32_t)T; d.N = (int32_t)H; d.K = (int32_t)F; d.batch_outer = d.batch_inner = 1;
    d.lda = F; d.ldw = F; d.ldc = H; d.ldr = H; d.per_channel = 1; d.out_dtype = IBERT_I32; d.out_clamp = 32767;
    d.residual_dy = q.res2_dy;
    // (+ 10: LayerNorm)
    RUN_GEMM_LN(9, g, w.w_2, w.b_2, w.m_2, w.s_2, h1, r2, w.ln2_gamma_q, w.ln2_beta_q, q.ln2_shift, y, 2.0 * T * H * F, F);
    return IBERT_OK;
#undef RUN_GEMM
#undef RUN_GEMM_LN
}

static int check_layer(const ibert_layer_weights& w, const ibert_layer_quant& q, int32_t seq, int32_t hidden)
{
    const void* ptrs[] = {w.w_qkv, w.b_qkv, w.m_qkv, w.s_qkv, w.w_o, w.b_o, w.m_o, w.s_o, w.ln1_gamma_q,
                          w.ln1_beta_q, w.w_1, w.b_1, w.m_1, w.s_1, w.w_2, w.b_2, w.m_2, w.s_2, w.ln2_gamma_q,
                          w.ln2_beta_q};
    for (const void* p : ptrs)
        if (!p) return IBERT_ERR_NULL;
    if (!dyadic_ok(q.scores_dy) || !dyadic_ok(q.ctx_dy) || !dyadic_ok(q.res1_dy) || !dyadic_ok(q.res2_dy))
        return IBERT_ERR_PARAM_RANGE;
    if (q.softmax.out_dtype != IBERT_I8) return IBERT_ERR_PARAM_RANGE;
    int rc = check_softmax(q.softmax, seq);
    if (rc) return rc;
    rc = check_gelu(q.gelu);
    if (rc) return rc;
    rc = check_layernorm(hidden, q.ln1_shift);
    if (rc) return rc;
    return check_layernorm(hidden, q.ln2_shift);
}

}  // namespace ibert

extern "C" {

size_t ibert_attention_scratch_bytes(int32_t batch, int32_t seq, int32_t heads)
{
    if (batch < 0 || seq < 0 || heads < 0) return 0;
    const size_t n = (size_t)batch * heads * seq * seq;
    return ibert::align_up(n * 4) + ibert::align_up(n);
}

int ibert_attention_i(const int8_t* qkv, int8_t* ctx, int32_t batch, int32_t seq, int32_t hidden, int32_t heads,
                      const ibert_dyadic* scores_dy, const ibert_softmax_params* softmax, const ibert_dyadic* ctx_dy,
                      void* scratch, size_t scratch_bytes, void* stream)
{
    return ibert_attention_masked_i(qkv, ctx, batch, seq, hidden, heads, scores_dy, softmax, ctx_dy, nullptr, scratch,
                                    scratch_bytes, stream);
}

int ibert_attention_masked_i(const int8_t* qkv, int8_t* ctx, int32_t batch, int32_t seq, int32_t hidden, int32_t heads,
                             const ibert_dyadic* scores_dy, const ibert_softmax_params* softmax,
                             const ibert_dyadic* ctx_dy, const int32_t* key_lens, void* scratch, size_t scratch_bytes,
                             void* stream)
{
    using namespace ibert;
    if (!scores_dy || !softmax || !ctx_dy) return IBERT_ERR_NULL;
    if (batch < 0 || seq < 1 || hidden < 1 || heads < 1 || hidden % heads) return IBERT_ERR_SHAPE;
    if (!dyadic_ok(*scores_dy) || !dyadic_ok(*ctx_dy) || softmax->out_dtype != IBERT_I8) return IBERT_ERR_PARAM_RANGE;
    const int rc = check_softmax(*softmax, seq);
    if (rc) return rc;
    if (batch == 0) return IBERT_OK;
    if (!qkv || !ctx) return IBERT_ERR_NULL;
    int32_t* scores = nullptr;
    int8_t* probs = nullptr;
    if (scratch) {
        if (scratch_bytes < ibert_attention_scratch_bytes(batch, seq, heads) || ((uintptr_t)scratch & 255)) return IBERT_ERR_WORKSPACE;
        const size_t n = (size_t)batch * heads * seq * seq;
        scores = static_cast<int32_t*>(scratch);
        probs = static_cast<int8_t*>(scratch) + align_up(n * 4);
    }
    return run_attention(qkv, scores, probs, ctx, batch, seq, hidden, heads, *scores_dy, *softmax, *ctx_dy, key_lens,
                         true, (hipStream_t)stream);
}

int ibert_profile_begin(int32_t capacity)
{
    using ibert::g_prof;
    if (g_prof.open) return IBERT_ERR_PARAM_RANGE;
    if (capacity < 1 || capacity > (1 << 20)) return IBERT_ERR_SHAPE;
    g_prof.ev = new hipEvent_t[2 * (size_t)capacity];
    g_prof.meta = new ibert::StepMeta[(size_t)capacity];
    for (int32_t i = 0; i < 2 * capacity; ++i) {
        const hipError_t e = hipEventCreate(&g_prof.ev[i]);
        if (e != hipSuccess) {
            for (int32_t j = 0; j < i; ++j) (void)hipEventDestroy(g_prof.ev[j]);
            delete[] g_prof.ev;
            delete[] g_prof.meta;
            g_prof.ev = nullptr;
            g_prof.meta = nullptr;
            return ibert::hip_failed(e, "hipEventCreate");
        }
    }
    g_prof.capacity = capacity;
    g_prof.count = 0;
    g_prof.open = true;
    return IBERT_OK;
}

int ibert_profile_end(ibert_profile_record* out, int32_t capacity, int32_t* count)
{
    using ibert::g_prof;
    if (!g_prof.open) return IBERT_ERR_PARAM_RANGE;
    int rc = IBERT_OK;
    const int32_t n = g_prof.count < capacity ? g_prof.count : capacity;
    if (!out || !count) rc = IBERT_ERR_NULL;
    for (int32_t i = 0; rc == IBERT_OK && i < n; ++i) {
        hipError_t e = hipEventSynchronize(g_prof.ev[2 * i + 1]);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, g_prof.ev[2 * i], g_prof.ev[2 * i + 1]);
        if (e != hipSuccess) {
            rc = ibert::hip_failed(e, "profile event");
            break;
        }
        out[i].step = g_prof.meta[i].step;
        out[i].ms = ms;
        out[i].ops = g_prof.meta[i].ops;
        out[i].bytes = g_prof.meta[i].bytes;
        std::strncpy(out[i].kernel, g_prof.meta[i].kernel, sizeof out[i].kernel - 1);
        out[i].kernel[sizeof out[i].kernel - 1] = 0;
    }
    if (count) *count = rc == IBERT_OK ? n : 0;
    for (int32_t i = 0; i < 2 * g_prof.capacity; ++i) (void)hipEventDestroy(g_prof.ev[i]);
    delete[] g_prof.ev;
    delete[] g_prof.meta;
    g_prof.ev = nullptr;
    g_prof.meta = nullptr;
    g_prof.open = false;
    g_prof.capacity = g_prof.count = 0;
    return rc;
}

int ibert_encoder_layer_workspace_layout(int32_t batch, int32_t seq, int32_t hidden, int32_t heads, int32_t ffn,
                                         ibert_layer_workspace_layout* out)
{
    if (!out) return IBERT_ERR_NULL;
    return ibert::layout(batch, seq, hidden, heads, ffn, out);
}

size_t ibert_encoder_layer_workspace_bytes(int32_t batch, int32_t seq, int32_t hidden, int32_t heads, int32_t ffn)
{
    ibert_layer_workspace_layout lo;
    if (ibert::layout(batch, seq, hidden, heads, ffn, &lo)) return 0;
    return lo.total;
}

size_t ibert_encoder_workspace_bytes(int32_t batch, int32_t seq, int32_t hidden, int32_t heads, int32_t ffn)
{
    ibert_layer_workspace_layout lo;
    if (ibert::layout(batch, seq, hidden, heads, ffn, &lo)) return 0;
    return lo.total + 2 * ibert::align_up((size_t)batch * seq * hidden);
}

int ibert_encoder_layer_i(const ibert_layer_weights* weights, const ibert_layer_quant* quant, const int8_t* x,
                          int8_t* y, int32_t batch, int32_t seq, int32_t hidden, int32_t heads, int32_t ffn,
                          void* workspace, size_t workspace_bytes, void* stream)
{
    return ibert_encoder_layer_masked_i(weights, quant, x, y, batch, seq, hidden, heads, ffn, nullptr, workspace,
                                        workspace_bytes, stream);
}

int ibert_encoder_layer_masked_i(const ibert_layer_weights* weights, const ibert_layer_quant* quant, const int8_t* x,
                                 int8_t* y, int32_t batch, int32_t seq, int32_t hidden, int32_t heads, int32_t ffn,
                                 const int32_t* key_lens, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!weights || !quant || !x || !y || !workspace) return IBERT_ERR_NULL;
    ibert_layer_workspace_layout lo;
    int rc = ibert::layout(batch, seq, hidden, heads, ffn, &lo);
    if (rc) return rc;
    if (x == y) return IBERT_ERR_SHAPE;
    if (workspace_bytes < lo.total || !ibert::aligned(workspace, 256)) return IBERT_ERR_WORKSPACE;
    rc = ibert::check_layer(*weights, *quant, seq, hidden);
    if (rc) return rc;
    return ibert::run_layer(*weights, *quant, x, y, batch, seq, hidden, heads, ffn, key_lens, (char*)workspace, lo,
                            (hipStream_t)stream);
}

size_t ibert_static_scratch_bytes(void) { return ibert::kStaticScratchBytes; }

int ibert_static_scratch_init(void)
{
    void* p = nullptr;
    return ibert::static_scratch_address(&p);
}

int ibert_encoder_layer_static_i(const ibert_layer_weights* weights, const ibert_layer_quant* quant, const int8_t* x,
                                 int8_t* y, int32_t batch, int32_t seq, int32_t hidden, int32_t heads, int32_t ffn,
                                 const int32_t* key_lens, void* stream)
{
    if (!weights || !quant || !x || !y) return IBERT_ERR_NULL;
    ibert_layer_workspace_layout lo;
    int rc = ibert::layout(batch, seq, hidden, heads, ffn, &lo);
    if (rc) return rc;
    if (x == y) return IBERT_ERR_SHAPE;
    if (lo.total > ibert::kStaticScratchBytes) return IBERT_ERR_WORKSPACE;     // the problem needs more than the array holds
    rc = ibert::check_layer(*weights, *quant, seq, hidden);
    if (rc) return rc;
    void* ws = nullptr;
    rc = ibert::static_scratch_address(&ws);
    if (rc) return rc;
    // every region of the workspace is written by the step that produces it before any step reads it, so nothing of
    // the previous call's contents has to be cleared
    return ibert::run_layer(*weights, *quant, x, y, batch, seq, hidden, heads, ffn, key_lens, (char*)ws, lo,
                            (hipStream_t)stream);
}

int ibert_encoder_i(const ibert_layer_weights* weights, const ibert_layer_quant* quant, int32_t n_layers,
                    const int8_t* x, int8_t* y, int32_t batch, int32_t seq, int32_t hidden, int32_t heads,
                    int32_t ffn, void* workspace, size_t workspace_bytes, void* stream)
{
    return ibert_encoder_masked_i(weights, quant, n_layers, x, y, batch, seq, hidden, heads, ffn, nullptr, workspace,
                                  workspace_bytes, stream);
}

int ibert_encoder_masked_i(const ibert_layer_weights* weights, const ibert_layer_quant* quant, int32_t n_layers,
                           const int8_t* x, int8_t* y, int32_t batch, int32_t seq, int32_t hidden, int32_t heads,
                           int32_t ffn, const int32_t* key_lens, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!weights || !quant || !x || !y || !workspace) return IBERT_ERR_NULL;
    if (n_layers < 1) return IBERT_ERR_SHAPE;
    ibert_layer_workspace_layout lo;
    int rc = ibert::layout(batch, seq, hidden, heads, ffn, &lo);
    if (rc) return rc;
    if (x == y) return IBERT_ERR_SHAPE;
    const size_t act = ibert::align_up((size_t)batch * seq * hidden);
    if (workspace_bytes < lo.total + 2 * act || !ibert::aligned(workspace, 256)) return IBERT_ERR_WORKSPACE;
    for (int32_t l = 0; l < n_layers; ++l) {
        rc = ibert::check_layer(weights[l], quant[l], seq, hidden);
        if (rc) return rc;
    }
    char* ws = (char*)workspace;
    int8_t* pp[2] = {reinterpret_cast<int8_t*>(ws + lo.total), reinterpret_cast<int8_t*>(ws + lo.total + act)};
    const int8_t* in = x;
    for (int32_t l = 0; l < n_layers; ++l) {
        int8_t* out = (l == n_layers - 1) ? y : pp[l & 1];
        rc = ibert::run_layer(weights[l], quant[l], in, out, batch, seq, hidden, heads, ffn, key_lens, ws, lo,
                              (hipStream_t)stream);
        if (rc) return rc;
        in = out;
    }
    return IBERT_OK;
}

}  // extern "C"
