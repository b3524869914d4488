/*
 * ibert_oracle.c -- CPU oracle for the integer-only encoder layer of I-BERT.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, exact
 * re-statement of the paper's integer algorithms, used only by the tests, the
 * smoke check and the cpu_baseline leg of the benchmark.  It shares no code,
 * header or table with the HIP library; it never runs on a GPU.
 *
 * Conventions
 *   - All arithmetic is done in int64_t (128-bit where a product could leave
 *     63 bits).  Every intermediate that a 32-bit machine is allowed to hold in
 *     32 bits is range-checked; a violation returns a negative ORC_E_* code.
 *   - floor() is the mathematical floor (toward minus infinity), as the
 *     footnote of Alg. 1 states; ">>" below always means floor division by a
 *     power of two.
 *   - Integer constants (q_b, q_c, q_ln2, dyadic multipliers ...) are inputs:
 *     they are pre-computed from the static scales outside of inference
 *     (footnote of Alg. 1; App. A, static quantization).
 *
 * Functions and the passages they follow
 *   orc_dyadic           Requantization INT32 -> INT8 (App. C.1); the paper
 *                        gives no formula, the reading is round-half-up of
 *                        x*m/2^s.
 *   orc_gemm_requant     INT8 MatMul with INT32 accumulation (Sec. 1
 *                        contribution 3, App. C.1) + bias + requantization.
 *   orc_ipoly            Alg. 1.
 *   orc_iexp             Alg. 3, I-Exp, Eq. 12-14.
 *   orc_softmax          Alg. 3, I-Softmax, Eq. 10-11.
 *   orc_ierf / orc_igelu_t / orc_gelu   Alg. 2, Eq. 8-9.
 *   orc_hgelu_t / orc_hgelu  h-GELU, Eq. 6 (the alternative the paper measures
 *                        i-GELU against; given there as a real-valued formula,
 *                        the integer form below is a reading).
 *   orc_isqrt            Alg. 4.
 *   orc_layernorm        Sec. 3.6, Eq. 15 + Alg. 4.
 *   orc_encoder_layer    Fig. 1 (right) attention block + the rest of a
 *                        post-LN encoder layer (Sec. 4.1: RoBERTa).
 *   orc_mask_scores      padded keys of a batch of sequences (the paper does
 *                        not mention padding; reading: a masked key has the
 *                        logit "minus infinity", i.e. INT32_MIN, so its
 *                        integer exponential is exactly zero).
 *   orc_embedding        INT8 embedding (Sec. 1 contribution 3, App. C.1 say
 *                        only that the embedding tables are INT8; how the
 *                        looked-up rows are added and normalized is not
 *                        spelled out; reading below).
 *
 * Parity pins live in tests/test_oracle_*.py.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef __int128 i128;

enum {
    ORC_OK = 0,
    ORC_E_ARG = -1,        /* bad pointer / shape */
    ORC_E_PARAM = -2,      /* an integer constant violates a precondition */
    ORC_E_RANGE = -3,      /* an intermediate left the range a 32-bit lane may hold */
    ORC_E_NOMEM = -4
};

#define ORC_I8 0
#define ORC_I32 1

static const int64_t I32_MAX = 2147483647LL;
static const int64_t I32_MIN = -2147483647LL - 1;

/* floor(v / 2^s), s in [0, 126] */
static i128 floor_shr(i128 v, int s)
{
    if (s == 0) return v;
    i128 d = (i128)1 << s;
    i128 q = v / d;          /* C division truncates toward zero */
    i128 r = v % d;
    if (r < 0) q -= 1;       /* make it a floor */
    return q;
}

/* floor(a / b), b > 0 */
static int64_t floor_div(int64_t a, int64_t b)
{
    int64_t q = a / b;
    int64_t r = a % b;
    if (r < 0) q -= 1;
    return q;
}

static int64_t clamp64(int64_t v, int64_t lo, int64_t hi)
{
    return v < lo ? lo : (v > hi ? hi : v);
}

/* ------------------------------------------------------------------------- */
/* Requantization (App. C.1): x * (m / 2^s), rounded half up.                */
/*   DY(x; m, s) = floor((x*m + 2^(s-1)) / 2^s)  for s >= 1,  x*m for s == 0 */
/* ------------------------------------------------------------------------- */
int64_t orc_dyadic(int64_t x, int32_t m, int32_t s)
{
    i128 p = (i128)x * (i128)m;
    if (s <= 0) return (int64_t)p;
    p += (i128)1 << (s - 1);
    return (int64_t)floor_shr(p, s);
}

static int dyadic_ok(int32_t s) { return s >= 0 && s <= 62; }

/* ------------------------------------------------------------------------- */
/* INT8 MatMul, INT32 accumulate, bias, requantization, optional residual.   */
/* ------------------------------------------------------------------------- */
typedef struct {
    int32_t M, N, K;
    int32_t batch_outer, batch_inner;   /* batch index z = zo*batch_inner + zi */
    int64_t lda, ldw, ldc, ldr;         /* row strides in elements */
    int64_t sA_o, sA_i, sW_o, sW_i, sC_o, sC_i, sR_o, sR_i; /* batch strides */
    int32_t trans_w;       /* 0: W is [N,K], element (n,k) at n*ldw+k ; 1: W is [K,N], (n,k) at k*ldw+n */
    int32_t per_channel;   /* 1: mult[n], shift[n] ; 0: dy_m, dy_s for every n */
    int32_t dy_m, dy_s;
    int32_t out_dtype;     /* ORC_I8 / ORC_I32 */
    int32_t out_clamp;     /* symmetric clamp, >= 0 */
    int32_t res_m, res_s;  /* residual requantization (used iff residual != NULL) */
} orc_gemm_t;

int orc_gemm_requant(const orc_gemm_t* d, const int8_t* A, const int8_t* W,
                     const int32_t* bias, const int32_t* mult, const int32_t* shift,
                     const int8_t* residual, void* C)
{
    if (!d || !C) return ORC_E_ARG;
    if (d->M < 0 || d->N < 0 || d->K < 0 || d->batch_outer < 0 || d->batch_inner < 0) return ORC_E_ARG;
    if (d->out_clamp < 0) return ORC_E_PARAM;
    if (d->out_dtype == ORC_I8 && d->out_clamp > 127) return ORC_E_PARAM;
    if (d->per_channel && (!mult || !shift)) return ORC_E_ARG;
    if (!d->per_channel && !dyadic_ok(d->dy_s)) return ORC_E_PARAM;
    if (residual && !dyadic_ok(d->res_s)) return ORC_E_PARAM;
    int64_t nb = (int64_t)d->batch_outer * d->batch_inner;
    if (nb == 0 || d->M == 0 || d->N == 0) return ORC_OK;
    if (d->K > 0 && (!A || !W)) return ORC_E_ARG;
    if (d->per_channel)
        for (int n = 0; n < d->N; ++n)
            if (!dyadic_ok(shift[n])) return ORC_E_PARAM;

    int status = ORC_OK;
    int64_t rows = nb * d->M;
#pragma omp parallel for schedule(static)
    for (int64_t zr = 0; zr < rows; ++zr) {
        int64_t z = zr / d->M, i = zr % d->M;
        int64_t zo = z / d->batch_inner, zi = z % d->batch_inner;
        const int8_t* a = A + zo * d->sA_o + zi * d->sA_i + i * d->lda;
        const int8_t* w = W + zo * d->sW_o + zi * d->sW_i;
        int64_t coff = zo * d->sC_o + zi * d->sC_i + i * d->ldc;
        const int8_t* r = residual ? residual + zo * d->sR_o + zi * d->sR_i + i * d->ldr : NULL;
        for (int n = 0; n < d->N; ++n) {
            int64_t acc = 0;
            if (d->trans_w == 0) {
                const int8_t* wr = w + (int64_t)n * d->ldw;
                for (int k = 0; k < d->K; ++k) acc += (int64_t)a[k] * (int64_t)wr[k];
            } else {
                for (int k = 0; k < d->K; ++k) acc += (int64_t)a[k] * (int64_t)w[(int64_t)k * d->ldw + n];
            }
            if (bias) acc += bias[n];
            if (acc > I32_MAX || acc < I32_MIN) {   /* INT32 accumulation must not wrap */
#pragma omp atomic write
                status = ORC_E_RANGE;
            }
            int32_t m = d->per_channel ? mult[n] : d->dy_m;
            int32_t s = d->per_channel ? shift[n] : d->dy_s;
            int64_t v = orc_dyadic(acc, m, s);
            if (r) v += orc_dyadic(r[n], d->res_m, d->res_s);
            v = clamp64(v, -(int64_t)d->out_clamp, d->out_clamp);
            if (d->out_dtype == ORC_I8) ((int8_t*)C)[coff + n] = (int8_t)v;
            else ((int32_t*)C)[coff + n] = (int32_t)v;
        }
    }
    return status;
}

/* ------------------------------------------------------------------------- */
/* Alg. 1: second-order polynomial a(x+b)^2+c on integers: (q+q_b)^2 + q_c.   */
/* ------------------------------------------------------------------------- */
int64_t orc_ipoly(int64_t q, int64_t q_b, int64_t q_c)
{
    int64_t t = q + q_b;
    return t * t + q_c;
}

/* ------------------------------------------------------------------------- */
/* Alg. 3, I-Exp.  q <= 0.  z = floor(-q/q_ln2); q_p = q + z*q_ln2;           */
/* result = I-Poly(q_p) >> z.  For z >= 63 the floor is 0 (I-Poly(q_p) < 2^63).*/
/* *z_out receives z (may be NULL).                                          */
/* ------------------------------------------------------------------------- */
int64_t orc_iexp(int64_t q, int64_t q_ln2, int64_t q_b, int64_t q_c, int64_t* z_out)
{
    int64_t z = floor_div(-q, q_ln2);
    int64_t q_p = q + z * q_ln2;
    int64_t q_L = orc_ipoly(q_p, q_b, q_c);
    if (z_out) *z_out = z;
    if (z >= 63) return 0;
    return (int64_t)floor_shr(q_L, (int)z);
}

/* ------------------------------------------------------------------------- */
/* Alg. 3, I-Softmax.  The paper leaves the final division open; reading:     */
/*   Fz = floor(2^31 / sum);  out_j = min(cap, (e_j*Fz + 2^(30-k)) >> (31-k)) */
/* with output scale 2^-k.  I8: k<=7, cap 127.  I32: k<=30, no cap.           */
/* ------------------------------------------------------------------------- */
typedef struct {
    int32_t q_ln2, q_b, q_c;
    int32_t out_frac_bits;   /* k */
    int32_t out_dtype;       /* ORC_I8 / ORC_I32 */
} orc_softmax_t;

int orc_softmax_check(const orc_softmax_t* p, int cols)
{
    if (!p || cols < 1) return ORC_E_ARG;
    if (p->q_ln2 < 1 || p->q_b < 1 || p->q_c < 0) return ORC_E_PARAM;
    if (p->q_ln2 > p->q_b) return ORC_E_PARAM;   /* ln2 < b (Eq. 13): q_b + q_p stays in (0, q_b] */
    if (p->out_frac_bits < 0) return ORC_E_PARAM;
    if (p->out_dtype == ORC_I8 && p->out_frac_bits > 7) return ORC_E_PARAM;
    if (p->out_dtype == ORC_I32 && p->out_frac_bits > 30) return ORC_E_PARAM;
    if (p->out_dtype != ORC_I8 && p->out_dtype != ORC_I32) return ORC_E_PARAM;
    /* every I-Poly value and every row sum must stay below 2^31 */
    i128 top = (i128)p->q_b * p->q_b + p->q_c;
    if (top * cols >= ((i128)1 << 31)) return ORC_E_PARAM;
    return ORC_OK;
}

int orc_softmax(const int32_t* x, void* y, int64_t rows, int cols, int64_t ldx, int64_t ldy,
                const orc_softmax_t* p)
{
    int rc = orc_softmax_check(p, cols);
    if (rc) return rc;
    if (rows < 0) return ORC_E_ARG;
    if (rows == 0) return ORC_OK;
    if (!x || !y) return ORC_E_ARG;
    const int k = p->out_frac_bits;
    int status = ORC_OK;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        const int32_t* xr = x + r * ldx;
        int64_t* e = (int64_t*)malloc(sizeof(int64_t) * (size_t)cols);
        if (!e) {
#pragma omp atomic write
            status = ORC_E_NOMEM;
            continue;
        }
        int64_t mx = xr[0];
        for (int j = 1; j < cols; ++j) if (xr[j] > mx) mx = xr[j];
        int64_t sum = 0;
        for (int j = 0; j < cols; ++j) {
            int64_t qt = (int64_t)xr[j] - mx;               /* q~ = q - max(q) <= 0 */
            e[j] = orc_iexp(qt, p->q_ln2, p->q_b, p->q_c, NULL);
            sum += e[j];
        }
        if (sum < 1 || sum >= (1LL << 31)) {
#pragma omp atomic write
            status = ORC_E_RANGE;
        }
        int64_t Fz = (1LL << 31) / sum;                      /* one division per row */
        for (int j = 0; j < cols; ++j) {
            int64_t P = e[j] * Fz;                           /* <= 2^31 */
            int64_t o = (P + (1LL << (30 - k))) >> (31 - k);
            if (p->out_dtype == ORC_I8) {
                if (o > 127) o = 127;
                ((int8_t*)y)[r * ldy + j] = (int8_t)o;
            } else {
                ((int32_t*)y)[r * ldy + j] = (int32_t)o;
            }
        }
        free(e);
    }
    return status;
}

/* ------------------------------------------------------------------------- */
/* Alg. 2.  I-Erf on the integer q whose scale is S/sqrt(2):                   */
/*   sgn(q) * I-Poly(min(|q|, -q_b)),  a=-0.2888, b=-1.769, c=1 (Eq. 8).      */
/* The clip limit -b/S is taken as the integer -q_b.                          */
/* ------------------------------------------------------------------------- */
typedef struct {
    int32_t q_b, q_c, q_1, q_max;
    int32_t out_m, out_s;
} orc_gelu_t;

int64_t orc_ierf(int64_t q, int64_t q_b, int64_t q_c)
{
    int64_t sg = (q > 0) - (q < 0);
    int64_t u = q < 0 ? -q : q;
    if (u > -q_b) u = -q_b;
    return sg * orc_ipoly(u, q_b, q_c);
}

/* I-GELU before requantization: t = q * (q_erf + q_1), scale S*S_erf/2 (Eq. 9). */
int64_t orc_igelu_t(int64_t q, const orc_gelu_t* p)
{
    q = clamp64(q, -(int64_t)p->q_max, p->q_max);
    return q * (orc_ierf(q, p->q_b, p->q_c) + p->q_1);
}

int orc_gelu_check(const orc_gelu_t* p)
{
    if (!p) return ORC_E_ARG;
    if (p->q_b > 0 || p->q_max < 0 || !dyadic_ok(p->out_s)) return ORC_E_PARAM;
    int64_t top = (int64_t)p->q_b * p->q_b + p->q_c;       /* I-Poly at u = 0 */
    int64_t a1 = top < 0 ? -top : top;
    int64_t a2 = p->q_c < 0 ? -(int64_t)p->q_c : p->q_c;   /* I-Poly at u = -q_b */
    int64_t a = a1 > a2 ? a1 : a2;
    if (a > I32_MAX) return ORC_E_PARAM;
    int64_t q1 = p->q_1 < 0 ? -(int64_t)p->q_1 : p->q_1;
    if ((i128)p->q_max * (a + q1) > I32_MAX) return ORC_E_PARAM;  /* |t| < 2^31 */
    return ORC_OK;
}

int orc_gelu(const int32_t* x, int8_t* y, int64_t n, const orc_gelu_t* p)
{
    int rc = orc_gelu_check(p);
    if (rc) return rc;
    if (n < 0) return ORC_E_ARG;
    if (n == 0) return ORC_OK;
    if (!x || !y) return ORC_E_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        int64_t t = orc_igelu_t(x[i], p);
        int64_t o = orc_dyadic(t, p->out_m, p->out_s);
        y[i] = (int8_t)clamp64(o, -127, 127);
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* Eq. 6, h-GELU(x) = x ReLU6(1.702 x + 3) / 6, on the integer q of scale S:   */
/*   q <- clamp(q, -q_max, q_max)                                             */
/*   u  = clamp(DY(q; slope) + q_3, 0, q_6)   slope ~ 1.702, q_3 = floor(3/S), */
/*                                            q_6 = floor(6/S); scale S        */
/*   t  = q u                                 scale S^2 (the 1/6 goes into the */
/*                                            output multiplier)               */
/*   y  = clamp(DY(t; out), -127, 127)        out ~ S^2 / (6 S_out)            */
/* ------------------------------------------------------------------------- */
typedef struct {
    int32_t slope_m, slope_s;
    int32_t q_3, q_6, q_max;
    int32_t out_m, out_s;
} orc_hgelu_par_t;

int orc_hgelu_check(const orc_hgelu_par_t* p)
{
    if (!p) return ORC_E_ARG;
    if (!dyadic_ok(p->slope_s) || !dyadic_ok(p->out_s)) return ORC_E_PARAM;
    if (p->q_3 < 0 || p->q_6 < p->q_3 || p->q_max < 0) return ORC_E_PARAM;
    if ((i128)p->q_max * p->q_6 > I32_MAX) return ORC_E_PARAM;       /* |t| < 2^31 */
    return ORC_OK;
}

int64_t orc_hgelu_t(int64_t q, const orc_hgelu_par_t* p)
{
    q = clamp64(q, -(int64_t)p->q_max, p->q_max);
    int64_t u = orc_dyadic(q, p->slope_m, p->slope_s) + p->q_3;
    u = u < 0 ? 0 : (u > p->q_6 ? p->q_6 : u);
    return q * u;
}

int orc_hgelu(const int32_t* x, int8_t* y, int64_t n, const orc_hgelu_par_t* p)
{
    int rc = orc_hgelu_check(p);
    if (rc) return rc;
    if (n < 0) return ORC_E_ARG;
    if (n == 0) return ORC_OK;
    if (!x || !y) return ORC_E_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        int64_t o = orc_dyadic(orc_hgelu_t(x[i], p), p->out_m, p->out_s);
        y[i] = (int8_t)clamp64(o, -127, 127);
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* Alg. 4, I-Sqrt: Newton iteration on integers, x0 = 2^ceil(Bits(n)/2).      */
/* *iters receives the number of passes through the loop body (may be NULL).  */
/* ------------------------------------------------------------------------- */
uint64_t orc_isqrt(uint64_t n, int* iters)
{
    if (iters) *iters = 0;
    if (n == 0) return 0;
    int bits = 0;
    for (uint64_t t = n; t; t >>= 1) ++bits;
    uint64_t x = (uint64_t)1 << ((bits + 1) / 2);
    int it = 0;
    for (;;) {
        ++it;
        uint64_t y = (x + n / x) / 2;
        if (y >= x) break;
        x = y;
    }
    if (iters) *iters = it;
    return x;
}

void orc_isqrt_array(const uint64_t* n, uint64_t* out, int32_t* iters, int64_t count)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; ++i) {
        int it;
        out[i] = orc_isqrt(n[i], &it);
        if (iters) iters[i] = it;
    }
}

/* ------------------------------------------------------------------------- */
/* Integer LayerNorm (Sec. 3.6, Eq. 15).  Only sqrt is spelled out in the     */
/* paper; the fixed-point format is the reading below.                        */
/*   x_i  <- clamp(x_i, +-(2^15-1))                                           */
/*   mu    = floor((sum x_i + floor(C/2)) / C)                                */
/*   d_i   = x_i - mu ; var = floor(sum d_i^2 / C) ; sigma = max(1, I-Sqrt)   */
/*   f     = floor(2^24 / sigma) ; y_i = floor(d_i*f / 2^14)   (10 frac bits) */
/*   out_i = clamp(floor((y_i*gamma_q[i] + beta_q[i] + 2^(s-1)) / 2^s), 127)  */
/* ------------------------------------------------------------------------- */
int orc_layernorm_check(int C, const int32_t* gamma_q, const int32_t* beta_q, int shift)
{
    if (C < 1 || C > 1024) return ORC_E_PARAM;
    if (shift < 1 || shift > 30) return ORC_E_PARAM;
    if (!gamma_q || !beta_q) return ORC_E_ARG;
    for (int i = 0; i < C; ++i) {
        int64_t g = gamma_q[i], b = beta_q[i];
        if (g <= -(1 << 14) || g >= (1 << 14)) return ORC_E_PARAM;
        if (b <= -(1 << 29) || b >= (1 << 29)) return ORC_E_PARAM;
    }
    return ORC_OK;
}

int orc_layernorm(const int32_t* x, int8_t* y, int64_t rows, int C, int64_t ldx, int64_t ldy,
                  const int32_t* gamma_q, const int32_t* beta_q, int shift)
{
    int rc = orc_layernorm_check(C, gamma_q, beta_q, shift);
    if (rc) return rc;
    if (rows < 0) return ORC_E_ARG;
    if (rows == 0) return ORC_OK;
    if (!x || !y) return ORC_E_ARG;
    int status = ORC_OK;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        const int32_t* xr = x + r * ldx;
        int64_t sum = 0;
        for (int i = 0; i < C; ++i) sum += clamp64(xr[i], -32767, 32767);
        int64_t mu = floor_div(sum + C / 2, C);
        int64_t ss = 0;
        for (int i = 0; i < C; ++i) {
            int64_t d = clamp64(xr[i], -32767, 32767) - mu;
            ss += d * d;
        }
        int64_t var = ss / C;
        if (var >= (1LL << 32)) {
#pragma omp atomic write
            status = ORC_E_RANGE;
        }
        int64_t sigma = (int64_t)orc_isqrt((uint64_t)var, NULL);
        if (sigma < 1) sigma = 1;
        int64_t f = (1LL << 24) / sigma;
        for (int i = 0; i < C; ++i) {
            int64_t d = clamp64(xr[i], -32767, 32767) - mu;
            int64_t df = d * f;
            int64_t yv = (int64_t)floor_shr(df, 14);
            int64_t g = yv * gamma_q[i];
            int64_t acc = g + beta_q[i] + (1LL << (shift - 1));
            if (df >= (1LL << 30) || df <= -(1LL << 30) || g >= (1LL << 30) || g <= -(1LL << 30) ||
                acc > I32_MAX || acc < I32_MIN) {
#pragma omp atomic write
                status = ORC_E_RANGE;
            }
            int64_t o = (int64_t)floor_shr(acc, shift);
            y[r * ldy + i] = (int8_t)clamp64(o, -127, 127);
        }
    }
    return status;
}

/* ------------------------------------------------------------------------- */
/* One post-LN encoder layer (Fig. 1 right for the attention block; RoBERTa    */
/* layer order, Sec. 4.1).  Steps:                                            */
/*  1 qkv   = RQ(x Wqkv^T + b)                  i8 [T,3H]   per-channel       */
/*  2 s     = RQ(Q_h K_h^T)                     i32 [B*h,L,L] per-tensor      */
/*            (the 1/sqrt(d) factor lives in the multiplier)                  */
/*  3 p     = I-Softmax(s)                      i8 [B*h,L,L], scale 2^-7      */
/*  4 ctx   = RQ(p V_h)                         i8 [T,H]                      */
/*  5 r1    = RQ(ctx Wo^T + b) + RQ(x)          i32 [T,H], clamp 2^15-1       */
/*  6 h1    = I-LayerNorm(r1)                   i8 [T,H]                      */
/*  7 f1    = RQ(h1 W1^T + b)                   i32 [T,F], clamp q_max        */
/*  8 g     = I-GELU(f1)                        i8 [T,F]                      */
/*  9 r2    = RQ(g W2^T + b) + RQ(h1)           i32 [T,H], clamp 2^15-1       */
/* 10 y     = I-LayerNorm(r2)                   i8 [T,H]                      */
/* Head j owns columns [64j, 64j+64) of each of Q, K, V (d = H/heads).        */
/* ------------------------------------------------------------------------- */
typedef struct {
    const int8_t* w_qkv; const int32_t* b_qkv; const int32_t* m_qkv; const int32_t* s_qkv;
    const int8_t* w_o;   const int32_t* b_o;   const int32_t* m_o;   const int32_t* s_o;
    const int32_t* ln1_gamma_q; const int32_t* ln1_beta_q;
    const int8_t* w_1;   const int32_t* b_1;   const int32_t* m_1;   const int32_t* s_1;
    const int8_t* w_2;   const int32_t* b_2;   const int32_t* m_2;   const int32_t* s_2;
    const int32_t* ln2_gamma_q; const int32_t* ln2_beta_q;
} orc_layer_weights_t;

typedef struct {
    int32_t scores_m, scores_s;
    orc_softmax_t softmax;
    int32_t ctx_m, ctx_s;
    int32_t res1_m, res1_s;
    int32_t ln1_shift;
    orc_gelu_t gelu;
    int32_t res2_m, res2_s;
    int32_t ln2_shift;
} orc_layer_quant_t;

/* Optional copies of every intermediate (any pointer may be NULL). */
typedef struct {
    int8_t* qkv; int32_t* scores; int8_t* probs; int8_t* ctx; int32_t* r1; int8_t* h1;
    int32_t* f1; int8_t* g; int32_t* r2;
} orc_layer_dump_t;

/* Keys at positions >= key_lens[b] of sequence b are padding: their logits become INT32_MIN before the
 * Softmax (for every head and every query), so that d = max - q is at least 2^31 - 2^20 or so, z >= 31
 * and the integer exponential is exactly 0 (Alg. 3; the maximum is taken over the row after masking, and
 * 1 <= key_lens[b] <= L keeps a real key in it).  scores: [B*heads, L, L]. */
int orc_mask_scores(int32_t* scores, int batch, int heads, int seq, const int32_t* key_lens)
{
    if (!scores || !key_lens || batch < 0 || heads < 1 || seq < 1) return ORC_E_ARG;
    for (int b = 0; b < batch; ++b) {
        if (key_lens[b] < 1 || key_lens[b] > seq) return ORC_E_ARG;
        for (int h = 0; h < heads; ++h)
            for (int i = 0; i < seq; ++i) {
                int32_t* row = scores + (((int64_t)b * heads + h) * seq + i) * seq;
                for (int j = key_lens[b]; j < seq; ++j) row[j] = (int32_t)I32_MIN;
            }
    }
    return ORC_OK;
}

int orc_encoder_layer_masked(const orc_layer_weights_t* w, const orc_layer_quant_t* q,
                             const int8_t* x, int8_t* y, int batch, int seq, int hidden, int heads, int ffn,
                             const int32_t* key_lens, const orc_layer_dump_t* dump)
{
    if (!w || !q || !x || !y) return ORC_E_ARG;
    if (batch < 1 || seq < 1 || hidden < 1 || heads < 1 || ffn < 1 || hidden % heads) return ORC_E_ARG;
    const int64_t B = batch, L = seq, H = hidden, nh = heads, F = ffn, T = B * L, dh = H / nh;
    int rc = ORC_OK, st;

    int8_t* qkv = (int8_t*)malloc((size_t)(T * 3 * H));
    int32_t* sc = (int32_t*)malloc(sizeof(int32_t) * (size_t)(B * nh * L * L));
    int8_t* pr = (int8_t*)malloc((size_t)(B * nh * L * L));
    int8_t* ctx = (int8_t*)malloc((size_t)(T * H));
    int32_t* r1 = (int32_t*)malloc(sizeof(int32_t) * (size_t)(T * H));
    int8_t* h1 = (int8_t*)malloc((size_t)(T * H));
    int32_t* f1 = (int32_t*)malloc(sizeof(int32_t) * (size_t)(T * F));
    int8_t* g = (int8_t*)malloc((size_t)(T * F));
    int32_t* r2 = (int32_t*)malloc(sizeof(int32_t) * (size_t)(T * H));
    if (!qkv || !sc || !pr || !ctx || !r1 || !h1 || !f1 || !g || !r2) { rc = ORC_E_NOMEM; goto done; }

    orc_gemm_t d;
#define RUN(call) do { st = (call); if (st == ORC_E_RANGE) rc = st; else if (st) { rc = st; goto done; } } while (0)

    /* 1: QKV projection */
    memset(&d, 0, sizeof d);
    d.M = (int32_t)T; d.N = (int32_t)(3 * H); d.K = (int32_t)H; d.batch_outer = d.batch_inner = 1;
    d.lda = H; d.ldw = H; d.ldc = 3 * H; d.per_channel = 1; d.out_dtype = ORC_I8; d.out_clamp = 127;
    RUN(orc_gemm_requant(&d, x, w->w_qkv, w->b_qkv, w->m_qkv, w->s_qkv, NULL, qkv));

    /* 2: scores per (b, head): Q_h K_h^T */
    memset(&d, 0, sizeof d);
    d.M = (int32_t)L; d.N = (int32_t)L; d.K = (int32_t)dh; d.batch_outer = (int32_t)B; d.batch_inner = (int32_t)nh;
    d.lda = 3 * H; d.ldw = 3 * H; d.ldc = L;
    d.sA_o = L * 3 * H; d.sA_i = dh; d.sW_o = L * 3 * H; d.sW_i = dh; d.sC_o = nh * L * L; d.sC_i = L * L;
    d.per_channel = 0; d.dy_m = q->scores_m; d.dy_s = q->scores_s; d.out_dtype = ORC_I32; d.out_clamp = 2147483647;
    RUN(orc_gemm_requant(&d, qkv, qkv + H, NULL, NULL, NULL, NULL, sc));

    /* (padded keys, if any) */
    if (key_lens) RUN(orc_mask_scores(sc, batch, heads, seq, key_lens));

    /* 3: softmax over the last axis */
    RUN(orc_softmax(sc, pr, B * nh * L, (int)L, L, L, &q->softmax));

    /* 4: context per (b, head): P V_h, written into [T,H] */
    memset(&d, 0, sizeof d);
    d.M = (int32_t)L; d.N = (int32_t)dh; d.K = (int32_t)L; d.batch_outer = (int32_t)B; d.batch_inner = (int32_t)nh;
    d.lda = L; d.ldw = 3 * H; d.ldc = H; d.trans_w = 1;
    d.sA_o = nh * L * L; d.sA_i = L * L; d.sW_o = L * 3 * H; d.sW_i = dh; d.sC_o = L * H; d.sC_i = dh;
    d.per_channel = 0; d.dy_m = q->ctx_m; d.dy_s = q->ctx_s; d.out_dtype = ORC_I8; d.out_clamp = 127;
    RUN(orc_gemm_requant(&d, pr, qkv + 2 * H, NULL, NULL, NULL, NULL, ctx));

    /* 5: output projection + residual(x) */
    memset(&d, 0, sizeof d);
    d.M = (int32_t)T; d.N = (int32_t)H; d.K = (int32_t)H; d.batch_outer = d.batch_inner = 1;
    d.lda = H; d.ldw = H; d.ldc = H; d.ldr = H; d.per_channel = 1; d.out_dtype = ORC_I32; d.out_clamp = 32767;
    d.res_m = q->res1_m; d.res_s = q->res1_s;
    RUN(orc_gemm_requant(&d, ctx, w->w_o, w->b_o, w->m_o, w->s_o, x, r1));

    /* 6: LayerNorm */
    RUN(orc_layernorm(r1, h1, T, (int)H, H, H, w->ln1_gamma_q, w->ln1_beta_q, q->ln1_shift));

    /* 7: FFN up-projection, output at the GELU input scale */
    memset(&d, 0, sizeof d);
    d.M = (int32_t)T; d.N = (int32_t)F; d.K = (int32_t)H; d.batch_outer = d.batch_inner = 1;
    d.lda = H; d.ldw = H; d.ldc = F; d.per_channel = 1; d.out_dtype = ORC_I32; d.out_clamp = q->gelu.q_max;
    RUN(orc_gemm_requant(&d, h1, w->w_1, w->b_1, w->m_1, w->s_1, NULL, f1));

    /* 8: GELU */
    RUN(orc_gelu(f1, g, T * F, &q->gelu));

    /* 9: FFN down-projection + residual(h1) */
    memset(&d, 0, sizeof d);
    d.M = (int32_t)T; d.N = (int32_t)H; d.K = (int32_t)F; d.batch_outer = d.batch_inner = 1;
    d.lda = F; d.ldw = F; d.ldc = H; d.ldr = H; d.per_channel = 1; d.out_dtype = ORC_I32; d.out_clamp = 32767;
    d.res_m = q->res2_m; d.res_s = q->res2_s;
    RUN(orc_gemm_requant(&d, g, w->w_2, w->b_2, w->m_2, w->s_2, h1, r2));

    /* 10: LayerNorm */
    RUN(orc_layernorm(r2, y, T, (int)H, H, H, w->ln2_gamma_q, w->ln2_beta_q, q->ln2_shift));
#undef RUN

    if (dump) {
        if (dump->qkv) memcpy(dump->qkv, qkv, (size_t)(T * 3 * H));
        if (dump->scores) memcpy(dump->scores, sc, sizeof(int32_t) * (size_t)(B * nh * L * L));
        if (dump->probs) memcpy(dump->probs, pr, (size_t)(B * nh * L * L));
        if (dump->ctx) memcpy(dump->ctx, ctx, (size_t)(T * H));
        if (dump->r1) memcpy(dump->r1, r1, sizeof(int32_t) * (size_t)(T * H));
        if (dump->h1) memcpy(dump->h1, h1, (size_t)(T * H));
        if (dump->f1) memcpy(dump->f1, f1, sizeof(int32_t) * (size_t)(T * F));
        if (dump->g) memcpy(dump->g, g, (size_t)(T * F));
        if (dump->r2) memcpy(dump->r2, r2, sizeof(int32_t) * (size_t)(T * H));
    }
done:
    free(qkv); free(sc); free(pr); free(ctx); free(r1); free(h1); free(f1); free(g); free(r2);
    return rc;
}

int orc_encoder_layer(const orc_layer_weights_t* w, const orc_layer_quant_t* q,
                      const int8_t* x, int8_t* y, int batch, int seq, int hidden, int heads, int ffn,
                      const orc_layer_dump_t* dump)
{
    return orc_encoder_layer_masked(w, q, x, y, batch, seq, hidden, heads, ffn, NULL, dump);
}

/* ------------------------------------------------------------------------- */
/* INT8 embedding.  Reading (the paper only says the layer is kept at INT8):   */
/*   r[t][c] = clamp( DY(tok[id_t][c]; tok_dy) + DY(pos[t mod seq][c]; pos_dy), +-(2^15 - 1) )       */
/*   y[t]    = integer LayerNorm of r[t] (Sec. 3.6), INT8                                           */
/* i.e. both INT8 tables are brought to one INT32 scale, the input scale of the LayerNorm, exactly as   */
/* a residual is added in the layer; token ids outside [0, vocab) are clamped into it (data never     */
/* faults).  The position of token t is t mod seq (every sequence starts at position 0).              */
/* r_out (optional) receives r.                                                                       */
/* ------------------------------------------------------------------------- */
int orc_embedding(const int32_t* ids, int64_t tokens, int seq, int hidden, int vocab, int max_pos,
                  const int8_t* tok, const int8_t* pos, int32_t tok_m, int32_t tok_s, int32_t pos_m, int32_t pos_s,
                  const int32_t* gamma_q, const int32_t* beta_q, int ln_shift, int32_t* r_out, int8_t* y)
{
    if (!ids || !tok || !pos || !gamma_q || !beta_q || !y) return ORC_E_ARG;
    if (tokens < 0 || seq < 1 || hidden < 1 || vocab < 1 || max_pos < seq) return ORC_E_ARG;
    if (!dyadic_ok(tok_s) || !dyadic_ok(pos_s)) return ORC_E_PARAM;
    int32_t* r = (int32_t*)malloc(sizeof(int32_t) * (size_t)(tokens * hidden + 1));
    if (!r) return ORC_E_NOMEM;
    for (int64_t t = 0; t < tokens; ++t) {
        int64_t id = ids[t];
        id = id < 0 ? 0 : (id >= vocab ? vocab - 1 : id);
        const int64_t p = t % seq;
        for (int c = 0; c < hidden; ++c) {
            const int64_t v = orc_dyadic(tok[id * hidden + c], tok_m, tok_s) + orc_dyadic(pos[p * hidden + c], pos_m, pos_s);
            r[t * hidden + c] = (int32_t)clamp64(v, -32767, 32767);
        }
    }
    if (r_out) memcpy(r_out, r, sizeof(int32_t) * (size_t)(tokens * hidden));
    const int rc = orc_layernorm(r, y, tokens, hidden, hidden, hidden, gamma_q, beta_q, ln_shift);
    free(r);
    return rc;
}

int orc_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}
