// Host side of libibert: status strings, HIP error record, and the helpers that turn real-valued
// static scales into the integer constants the kernels consume (static quantization, Sec. 3.1 and
// App. A; footnote of Alg. 1: the constants are pre-computed, never evaluated during inference).
#include <cmath>
#include <cstdio>
#include <cstring>

#include "common.h"

namespace ibert {

static thread_local char g_hip_error[256] = "";

int hip_failed(hipError_t e, const char* what)
{
    std::snprintf(g_hip_error, sizeof g_hip_error, "%s: %s", what, hipGetErrorString(e));
    return IBERT_ERR_HIP;
}

const char* g_last_kernel = "";

static const double kLn2 = 0.6931471805599453;   // ln 2 rounded to binary64

}  // namespace ibert

extern "C" {

const char* ibert_status_string(int status)
{
    switch (status) {
        case IBERT_OK: return "ok";
        case IBERT_ERR_NULL: return "a required pointer is NULL";
        case IBERT_ERR_SHAPE: return "invalid shape or stride";
        case IBERT_ERR_PARAM_RANGE: return "an integer constant violates a documented precondition";
        case IBERT_ERR_ALIGN: return "misaligned pointer or stride";
        case IBERT_ERR_WORKSPACE: return "workspace too small or misaligned";
        case IBERT_ERR_HIP: return "HIP runtime error";
        case IBERT_ERR_NOT_IMPLEMENTED: return "not implemented";
        default: return "unknown status";
    }
}

const char* ibert_last_hip_error(void) { return ibert::g_hip_error; }

int ibert_version(void) { return 100; }

int ibert_dyadic_from_double(double M, ibert_dyadic* out)
{
    if (!out) return IBERT_ERR_NULL;
    if (!std::isfinite(M)) return IBERT_ERR_PARAM_RANGE;
    out->m = 0;
    out->s = 0;
    if (M == 0.0) return IBERT_OK;
    int e = 0;
    const double f = std::frexp(std::fabs(M), &e);          // |M| = f * 2^e, f in [0.5, 1)
    long long m = (long long)std::nearbyint(f * 2147483648.0);   // exact product; round half to even
    if (m == 2147483648LL) {
        m = 1073741824LL;
        e += 1;
    }
    const int s = 31 - e;
    if (s > 62) return IBERT_OK;                              // |M| < 2^-32: the multiplier vanishes
    if (s < 0) return IBERT_ERR_PARAM_RANGE;
    out->m = (int32_t)(M < 0 ? -m : m);
    out->s = s;
    return IBERT_OK;
}

int ibert_channel_dyadics_from_scales(double S_in, const double* S_w, int32_t N, double S_out, int32_t* mult,
                                      int32_t* shift)
{
    if (N < 0) return IBERT_ERR_SHAPE;
    if (N > 0 && (!S_w || !mult || !shift)) return IBERT_ERR_NULL;
    for (int32_t n = 0; n < N; ++n) {
        ibert_dyadic d;
        const int rc = ibert_dyadic_from_double(S_in * S_w[n] / S_out, &d);
        if (rc) return rc;
        mult[n] = d.m;
        shift[n] = d.s;
    }
    return IBERT_OK;
}

int ibert_softmax_params_from_scale(double S, int32_t cols, int32_t out_frac_bits, int32_t out_dtype,
                                    ibert_softmax_params* out)
{
    if (!out) return IBERT_ERR_NULL;
    if (!(S > 0.0) || !std::isfinite(S)) return IBERT_ERR_PARAM_RANGE;
    const double a = 0.3585, b = 1.353, c = 0.344;            // Eq. 13
    const double q_ln2 = std::floor(ibert::kLn2 / S);
    const double q_b = std::floor(b / S);
    const double q_c = std::floor(c / (a * S * S));
    if (q_ln2 > 2147483647.0 || q_b > 2147483647.0 || q_c > 2147483647.0) return IBERT_ERR_PARAM_RANGE;
    out->q_ln2 = (int32_t)q_ln2;
    out->q_b = (int32_t)q_b;
    out->q_c = (int32_t)q_c;
    out->out_frac_bits = out_frac_bits;
    out->out_dtype = out_dtype;
    return ibert::check_softmax(*out, cols);
}

int ibert_gelu_params_from_scale(double S_in, double S_out, ibert_gelu_params* out)
{
    if (!out) return IBERT_ERR_NULL;
    if (!(S_in > 0.0) || !(S_out > 0.0) || !std::isfinite(S_in) || !std::isfinite(S_out)) return IBERT_ERR_PARAM_RANGE;
    const double a = -0.2888, b = -1.769;                     // Eq. 8
    const double Sp = S_in / std::sqrt(2.0);                  // I-Erf works on x/sqrt(2) (Alg. 2)
    const double S_erf = a * Sp * Sp;
    const double q_b = std::floor(b / Sp);
    const double q_c = std::floor(1.0 / S_erf);
    if (q_b < -2147483647.0 || q_c < -2147483647.0) return IBERT_ERR_PARAM_RANGE;
    out->q_b = (int32_t)q_b;
    out->q_c = (int32_t)q_c;
    out->q_1 = (int32_t)q_c;                                  // q_1 = floor(1/S_erf), the same number
    const long long top = (long long)out->q_b * out->q_b + out->q_c;
    const long long a1 = top < 0 ? -top : top;
    const long long a2 = -(long long)out->q_c;
    const long long bound = (a1 > a2 ? a1 : a2) + (out->q_1 < 0 ? -(long long)out->q_1 : out->q_1);
    if (bound <= 0) return IBERT_ERR_PARAM_RANGE;
    out->q_max = (int32_t)(2147483647LL / bound);
    const double S_t = S_in * S_erf / 2.0;
    const int rc = ibert_dyadic_from_double(S_t / S_out, &out->out);
    if (rc) return rc;
    return ibert::check_gelu(*out);
}

int ibert_hgelu_params_from_scale(double S_in, double S_out, ibert_hgelu_params* out)
{
    if (!out) return IBERT_ERR_NULL;
    if (!(S_in > 0.0) || !(S_out > 0.0) || !std::isfinite(S_in) || !std::isfinite(S_out)) return IBERT_ERR_PARAM_RANGE;
    int rc = ibert_dyadic_from_double(1.702, &out->slope);                    // Eq. 6
    if (rc) return rc;
    const double q_3 = std::floor(3.0 / S_in), q_6 = std::floor(6.0 / S_in);
    if (q_6 > 2147483647.0) return IBERT_ERR_PARAM_RANGE;
    out->q_3 = (int32_t)q_3;
    out->q_6 = (int32_t)q_6;
    out->q_max = (int32_t)(2147483647LL / (out->q_6 > 1 ? out->q_6 : 1));
    rc = ibert_dyadic_from_double(S_in * S_in / (6.0 * S_out), &out->out);
    if (rc) return rc;
    return ibert::check_hgelu(*out);
}

int ibert_layernorm_params_from_float(const double* gamma, const double* beta, int32_t C, double S_out,
                                      int32_t* gamma_q, int32_t* beta_q, int32_t* shift)
{
    if (!gamma || !beta || !gamma_q || !beta_q || !shift) return IBERT_ERR_NULL;
    if (C < 1 || C > 1024) return IBERT_ERR_PARAM_RANGE;
    if (!(S_out > 0.0) || !std::isfinite(S_out)) return IBERT_ERR_PARAM_RANGE;
    for (int s = 30; s >= 1; --s) {
        const double pg = std::ldexp(1.0, s - 10), pb = std::ldexp(1.0, s);
        bool ok = true;
        for (int i = 0; i < C && ok; ++i) {
            const double gq = std::nearbyint(gamma[i] / S_out * pg);
            const double bq = std::nearbyint(beta[i] / S_out * pb);
            ok = std::fabs(gq) < 16384.0 && std::fabs(bq) < 536870912.0;
        }
        if (!ok) continue;
        for (int i = 0; i < C; ++i) {
            gamma_q[i] = (int32_t)std::nearbyint(gamma[i] / S_out * pg);
            beta_q[i] = (int32_t)std::nearbyint(beta[i] / S_out * pb);
        }
        *shift = s;
        return IBERT_OK;
    }
    return IBERT_ERR_PARAM_RANGE;
}

int ibert_layer_quant_from_scales(const ibert_layer_scales* sc, int32_t seq, int32_t head_dim, ibert_layer_quant* out)
{
    if (!sc || !out) return IBERT_ERR_NULL;
    if (seq < 1 || head_dim < 1 || sc->softmax_k < 0 || sc->softmax_k > 7) return IBERT_ERR_PARAM_RANGE;
    std::memset(out, 0, sizeof *out);
    int rc;
    rc = ibert_dyadic_from_double(sc->S_q * sc->S_k / (std::sqrt((double)head_dim) * sc->S_s), &out->scores_dy);
    if (rc) return rc;
    rc = ibert_softmax_params_from_scale(sc->S_s, seq, sc->softmax_k, IBERT_I8, &out->softmax);
    if (rc) return rc;
    rc = ibert_dyadic_from_double(std::ldexp(1.0, -sc->softmax_k) * sc->S_v / sc->S_ctx, &out->ctx_dy);
    if (rc) return rc;
    rc = ibert_dyadic_from_double(sc->S_x / sc->S_r1, &out->res1_dy);
    if (rc) return rc;
    rc = ibert_gelu_params_from_scale(sc->S_g_in, sc->S_g_out, &out->gelu);
    if (rc) return rc;
    rc = ibert_dyadic_from_double(sc->S_h1 / sc->S_r2, &out->res2_dy);
    if (rc) return rc;
    out->ln1_shift = 0;
    out->ln2_shift = 0;
    return IBERT_OK;
}

}  // extern "C"
