/*
 * libibert -- integer-only Transformer encoder layer (I-BERT) for AMD MI355X (gfx950).
 *
 * C ABI.  Every compute entry point enqueues hand-written HIP kernels on the caller's stream and
 * returns without synchronising.  It never allocates or frees device memory.
 *
 * Conventions
 *   - Return value: IBERT_OK (0) or a negative IBERT_ERR_* code.  Nothing throws or aborts.
 *   - "device" pointers are GPU global-memory addresses owned by the caller and must stay valid
 *     until the stream has executed the call.  "host" pointers are read during the call only.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   - All tensors are dense row-major with explicit row strides (in elements).
 *   - Only integers reach the device: real scales appear solely in the host helpers at the end,
 *     which pre-compute the integer constants (static quantization, Sec. 3.1 and App. A; footnote
 *     of Alg. 1).  The device sources contain no floating-point type or operation (the integer square root of
 *     Alg. 4 included); the only place the compiler may use its reciprocal unit is its own expansion of the two
 *     per-row integer divisions with data-dependent divisors (2^31 / sum in Softmax, 2^24 / sigma in LayerNorm),
 *     each of which returns the exact integer quotient.
 *   - Out-of-range data never faults: it is clamped as documented (the functions are total on int32
 *     inputs); out-of-range *constants* are refused with IBERT_ERR_PARAM_RANGE.
 *   - floor(.) is the mathematical floor; ">>" on signed values is an arithmetic shift.
 */
#ifndef IBERT_H
#define IBERT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    IBERT_OK = 0,
    IBERT_ERR_NULL = -1,          /* a required pointer is NULL                                   */
    IBERT_ERR_SHAPE = -2,         /* negative / inconsistent sizes or strides                     */
    IBERT_ERR_PARAM_RANGE = -3,   /* an integer constant violates a documented precondition       */
    IBERT_ERR_ALIGN = -4,         /* a pointer or stride misses a documented alignment            */
    IBERT_ERR_WORKSPACE = -5,     /* workspace too small or misaligned                            */
    IBERT_ERR_HIP = -6,           /* a HIP call failed; see ibert_last_hip_error()                */
    IBERT_ERR_NOT_IMPLEMENTED = -7
};

enum { IBERT_I8 = 0, IBERT_I32 = 1, IBERT_I16 = 2 };

/* A real multiplier M represented as m / 2^s.  0 <= s <= 62, m signed. */
typedef struct { int32_t m; int32_t s; } ibert_dyadic;

/* ------------------------------------------------------------------------------------------------
 * Requantization (App. C.1: INT32 results are brought back to INT8 by the dyadic-number scheme the
 * paper cites; the paper prints no formula).  Reading used by every function below:
 *     DY(x; m, s) = floor((x*m + 2^(s-1)) / 2^s)   for s >= 1,      DY(x; m, 0) = x*m
 * evaluated exactly in 64 bits: round-half-up of x*m/2^s.
 * ---------------------------------------------------------------------------------------------- */

/* ------------------------------------------------------------------------------------------------
 * ibert_gemm_i8_requant -- INT8 x INT8 -> INT32 MatMul with INT32 accumulation (Sec. 1, third
 * contribution; Sec. 4.1; App. C.1), bias, requantization and optional residual, batched-strided.
 *
 *   acc[i,n] = sum_k A[i,k] * W(n,k) + bias[n]
 *   v        = DY(acc; mult[n], shift[n])            (per_channel = 1)
 *            = DY(acc; requant.m, requant.s)         (per_channel = 0)
 *   v       += DY(residual[i,n]; residual_dy)        (iff residual != NULL)
 *   C[i,n]   = clamp(v, -out_clamp, +out_clamp)      stored as int8 (IBERT_I8), int32 (IBERT_I32) or int16
 *                                                    (IBERT_I16: the same values as IBERT_I32 in half the bytes, for
 *                                                    results clamped to 16 bits such as the LayerNorm input)
 *
 * W(n,k) = W[n*ldw + k] when trans_w = 0 (W is [N,K], the layout of a linear layer's weight) and
 * W[k*ldw + n] when trans_w = 1 (W is [K,N], used for probabilities x values).
 * Batch element z in [0, batch_outer*batch_inner) splits as zo = z / batch_inner, zi = z % batch_inner
 * and offsets each operand by zo*stride_outer + zi*stride_inner (elements).  bias / mult / shift are
 * shared by all batch elements.
 *
 * Pointers: A, W, residual (int8), bias, mult, shift (int32), C: device.  desc: host.
 * bias may be NULL (no bias).  mult/shift are required iff per_channel = 1 and hold N entries,
 * every shift in [0, 62].
 * Preconditions: M, N, K >= 0 (an empty problem is a no-op); K <= 2^17 so that the INT32 accumulator
 * cannot wrap (K * 127^2 + 2^31-ish bias is the caller's responsibility: |bias| + K*16129 < 2^31);
 * out_clamp >= 0, and <= 127 for IBERT_I8, <= 32767 for IBERT_I16.  No alignment is required; 16-byte aligned A/W rows
 * (pointers and lda/ldw/batch strides multiples of 16) select the fast MFMA path.
 * Output rows of different (z, i) must not overlap.  C must not alias the inputs.
 * ---------------------------------------------------------------------------------------------- */
typedef struct {
    int32_t M, N, K;
    int32_t batch_outer, batch_inner;
    int64_t lda, ldw, ldc, ldr;
    int64_t strideA_outer, strideA_inner;
    int64_t strideW_outer, strideW_inner;
    int64_t strideC_outer, strideC_inner;
    int64_t strideR_outer, strideR_inner;
    int32_t trans_w;
    int32_t per_channel;
    ibert_dyadic requant;        /* used iff per_channel == 0 */
    int32_t out_dtype;           /* IBERT_I8 | IBERT_I32 | IBERT_I16 */
    int32_t out_clamp;
    ibert_dyadic residual_dy;    /* used iff residual != NULL */
} ibert_gemm_desc;

int ibert_gemm_i8_requant(const ibert_gemm_desc* desc, const int8_t* A, const int8_t* W,
                          const int32_t* bias, const int32_t* mult, const int32_t* shift,
                          const int8_t* residual, void* C, void* stream);

/* ------------------------------------------------------------------------------------------------
 * ibert_softmax_i -- integer-only Softmax over the last axis (Alg. 3; Eq. 11-14).
 *
 * Per row q[0..cols):   d_j = max(q) - q_j  (as an unsigned 32-bit number, so any int32 logits are legal)
 *   z_j = floor(d_j / q_ln2),  r_j = d_j - z_j*q_ln2          (x~ = -z ln2 + p, p = -r_j S in (-ln2, 0])
 *   e_j = ((q_b - r_j)^2 + q_c) >> z_j,  and 0 once z_j >= 31  (I-Poly of Alg. 1 with the constants of Eq. 13)
 *   sum = sum_j e_j
 * The paper's last line (q_exp / sum) leaves the fixed-point format open; reading:
 *   Fz = floor(2^31 / sum),   y_j = min(cap, (e_j*Fz + 2^(30-k)) >> (31-k)),  output scale 2^-k
 *   IBERT_I8 : k = out_frac_bits <= 7, cap = 127 (a probability of exactly one saturates)
 *   IBERT_I32: k = out_frac_bits <= 30, no cap.
 * Preconditions (else IBERT_ERR_PARAM_RANGE): 1 <= q_ln2 <= q_b (ln2 < b of Eq. 13), q_c >= 0,
 *   cols * (q_b^2 + q_c) < 2^31 (every e_j and every row sum fits 31 bits).  cols >= 1.
 * x: device int32 [rows, ldx]; y: device int8 or int32 [rows, ldy]; params: host.
 * Rows whose addresses are 16-byte (x) / 4-byte (y) aligned take the vector path; others still work.
 * ---------------------------------------------------------------------------------------------- */
typedef struct {
    int32_t q_ln2, q_b, q_c;
    int32_t out_frac_bits;
    int32_t out_dtype;
} ibert_softmax_params;

int ibert_softmax_i(const int32_t* x, void* y, int64_t rows, int32_t cols, int64_t ldx, int64_t ldy,
                    const ibert_softmax_params* params, void* stream);

/* The same over padded rows: row r has n = key_lens[r / rows_per_len] real columns (key_lens: device int32,
 * ceil(rows / rows_per_len) entries, read by the kernel; values outside [1, cols] are clamped into it, since the
 * host cannot see them).  The paper does not treat padding; reading: a masked logit is "minus infinity", here
 * INT32_MIN, set before the row maximum is taken, so e_j of a masked column is 0 (unless the real logits themselves
 * sit within 31*q_ln2 of INT32_MIN) and y_j = 0 is written for it.  rows_per_len >= 1 (IBERT_ERR_SHAPE). */
int ibert_softmax_masked_i(const int32_t* x, void* y, int64_t rows, int32_t cols, int64_t ldx, int64_t ldy,
                           const ibert_softmax_params* params, const int32_t* key_lens, int64_t rows_per_len,
                           void* stream);

/* ------------------------------------------------------------------------------------------------
 * ibert_gelu_i -- integer-only GELU (Alg. 2; Eq. 8-9), element-wise, followed by requantization.
 *
 *   q   <- clamp(q, -q_max, q_max)                      (makes |t| < 2^31 below; the paper only notes
 *                                                        that products need double width)
 *   u    = min(|q|, -q_b)                               (clip of Eq. 8, limit taken as the integer -q_b)
 *   erf  = sgn(q) * ((u + q_b)^2 + q_c)                 (I-Erf, on the scale S/sqrt(2))
 *   t    = q * (erf + q_1)                              (scale S*S_erf/2, which is negative)
 *   y    = clamp(DY(t; out), -127, 127)                 (out.m is negative for a positive output scale)
 * Preconditions: q_b <= 0, q_max >= 0, q_max * (max(|q_c|, |q_b^2+q_c|) + |q_1|) <= 2^31-1, 0 <= out.s <= 62.
 * x: device int32 [n]; y: device int8 [n]; params: host.
 * ---------------------------------------------------------------------------------------------- */
typedef struct {
    int32_t q_b, q_c, q_1, q_max;
    ibert_dyadic out;
} ibert_gelu_params;

int ibert_gelu_i(const int32_t* x, int8_t* y, int64_t n, const ibert_gelu_params* params, void* stream);

/* ------------------------------------------------------------------------------------------------
 * ibert_hgelu_i -- h-GELU, the integer-friendly alternative the paper compares i-GELU with (Eq. 6; Table 1):
 * x ReLU6(1.702 x + 3) / 6.  The paper gives only the real-valued formula; reading, on integers of scale S:
 *   q   <- clamp(q, -q_max, q_max)
 *   u    = clamp(DY(q; slope) + q_3, 0, q_6)            slope ~ 1.702, q_3 = floor(3/S), q_6 = floor(6/S)
 *   t    = q * u                                        (scale S^2; the division by 6 is part of `out`)
 *   y    = clamp(DY(t; out), -127, 127)                 out ~ S^2 / (6 S_out)
 * Preconditions (else IBERT_ERR_PARAM_RANGE): 0 <= q_3 <= q_6, q_max >= 0, q_max * q_6 <= 2^31-1, both shifts in
 * [0, 62].  x: device int32 [n]; y: device int8 [n]; params: host.  Not used by ibert_encoder_layer_i.
 * ---------------------------------------------------------------------------------------------- */
typedef struct {
    ibert_dyadic slope;
    int32_t q_3, q_6, q_max;
    ibert_dyadic out;
} ibert_hgelu_params;

int ibert_hgelu_i(const int32_t* x, int8_t* y, int64_t n, const ibert_hgelu_params* params, void* stream);

/* ------------------------------------------------------------------------------------------------
 * ibert_gemm_i8_gelu -- the FFN up-projection and its GELU in one call (Sec. 4.1: the MatMul result is
 * requantized to the GELU input scale; Alg. 2 follows), bit-identical to
 *     ibert_gemm_i8_requant(desc with out_dtype = IBERT_I32, out_clamp = gelu->q_max, no residual) -> f
 *     ibert_gelu_i(f) -> C
 * C: device int8, laid out by desc (ldc, batch strides); desc->out_dtype, out_clamp and residual_dy are ignored.
 * When the problem fits a whole-tile MFMA configuration (M, N multiples of the tile, K a multiple of 128,
 * 16-byte aligned A/W rows) GELU runs in the MatMul epilogue and the INT32 tensor f never exists.  Otherwise the
 * two kernels run back to back through `scratch` (device int32, M*N*batch entries): that needs dense
 * outputs (ldc = N, dense batch strides; else IBERT_ERR_NOT_IMPLEMENTED) and a non-NULL scratch
 * (else IBERT_ERR_WORKSPACE).  scratch may always be passed; it is untouched on the one-kernel path.
 * ---------------------------------------------------------------------------------------------- */
int ibert_gemm_i8_gelu(const ibert_gemm_desc* desc, const int8_t* A, const int8_t* W, const int32_t* bias,
                       const int32_t* mult, const int32_t* shift, const ibert_gelu_params* gelu, int8_t* C,
                       int32_t* scratch, void* stream);

/* ------------------------------------------------------------------------------------------------
 * ibert_layernorm_i -- integer-only LayerNorm over the last axis (Sec. 3.6, Eq. 15, Alg. 4).
 * The paper specifies the integer square root and leaves the rest "straightforward"; reading:
 *   x_i  <- clamp(x_i, -(2^15-1), 2^15-1)
 *   mu    = floor((sum_i x_i + floor(C/2)) / C)
 *   d_i   = x_i - mu;  var = floor(sum_i d_i^2 / C)     (population variance, Eq. 15)
 *   sigma = max(1, floor(sqrt(var)))                    (Alg. 4 returns exactly floor(sqrt); no epsilon)
 *   f     = floor(2^24 / sigma);  n_i = (d_i * f) >> 14 (normalised value with 10 fractional bits)
 *   y_i   = clamp((n_i*gamma_q[i] + beta_q[i] + 2^(shift-1)) >> shift, -127, 127)
 * Preconditions: 1 <= C <= 1024, 1 <= shift <= 30.  gamma_q, beta_q: device int32 [C] with
 * |gamma_q| < 2^14 and |beta_q| < 2^29 (the caller's responsibility; ibert_layernorm_params_from_float
 * guarantees it) so that every intermediate fits 32 bits.
 * x: device int32 [rows, ldx]; y: device int8 [rows, ldy].
 * ---------------------------------------------------------------------------------------------- */
int ibert_layernorm_i(const int32_t* x, int8_t* y, int64_t rows, int32_t C, int64_t ldx, int64_t ldy,
                      const int32_t* gamma_q, const int32_t* beta_q, int32_t shift, void* stream);
/* The same on x: device int16 [rows, ldx] (the first step's clamp makes 16 bits lossless; an IBERT_I16 MatMul output
 * is such a tensor).  Bit-identical to ibert_layernorm_i on the widened values. */
int ibert_layernorm_i16(const int16_t* x, int8_t* y, int64_t rows, int32_t C, int64_t ldx, int64_t ldy,
                        const int32_t* gamma_q, const int32_t* beta_q, int32_t shift, void* stream);

/* ------------------------------------------------------------------------------------------------
 * ibert_isqrt_i -- the integer square root of Alg. 4 (Sec. 3.6) as a call of its own: root[i] = floor(sqrt(n[i])) for
 * any 32-bit n[i], which is what the Newton iteration of Alg. 4 returns (it starts at 2^ceil(Bits(n)/2), at or above the
 * root, and its integer iterates decrease to exactly that value).  The library reaches the same integer without a chain
 * of divisions, by the two routines the LayerNorm kernels use, selected by `method`:
 *   0: one value per lane, sixteen shift-and-subtract steps;
 *   1, 2, 3: the 64, 32 or 16 lanes that share a row test one candidate each per round and count the ones whose square
 *      does not exceed n (three or four rounds) -- the form ibert_layernorm_i runs, once per row.
 * n, root: device uint32 [count].  Errors: IBERT_ERR_SHAPE (count < 0), IBERT_ERR_PARAM_RANGE (method), IBERT_ERR_NULL.
 * ---------------------------------------------------------------------------------------------- */
int ibert_isqrt_i(const uint32_t* n, uint32_t* root, int64_t count, int32_t method, void* stream);

/* ------------------------------------------------------------------------------------------------
 * ibert_embedding_i -- the INT8 embedding that feeds the first layer (Sec. 1, third contribution; App. C.1: the
 * embedding tables are INT8 like every other parameter).  The paper does not spell out how the looked-up rows are
 * added and normalized; reading, for token t (its position is t mod seq):
 *   r_c = clamp(DY(tok[id_t][c]; tok_dy) + DY(pos[t mod seq][c]; pos_dy), -(2^15-1), 2^15-1)
 *         both tables rescaled to one INT32 scale S_r (tok_dy ~ S_tok/S_r, pos_dy ~ S_pos/S_r), summed exactly
 *   y   = ibert_layernorm_i(r; gamma_q, beta_q, ln_shift)              one kernel, r never stored
 * ids: device int32 [tokens], clamped into [0, vocab) by the kernel; tok: device int8 [vocab, hidden]; pos: device
 * int8 [max_pos, hidden] with max_pos >= seq; y: device int8 [tokens, ldy]; the dyadics are host pointers.
 * Segment (token-type) embeddings are not part of RoBERTa and not provided.
 * Errors: IBERT_ERR_SHAPE (negative sizes, max_pos < seq, ldy < hidden), IBERT_ERR_PARAM_RANGE (shift of a dyadic
 * outside [0, 62], hidden > 1024, ln_shift outside [1, 30]), IBERT_ERR_NULL.
 * ---------------------------------------------------------------------------------------------- */
int ibert_embedding_i(const int32_t* ids, const int8_t* tok, const int8_t* pos, int64_t tokens, int32_t seq,
                      int32_t hidden, int32_t vocab, int32_t max_pos, const ibert_dyadic* tok_dy,
                      const ibert_dyadic* pos_dy, const int32_t* gamma_q, const int32_t* beta_q, int32_t ln_shift,
                      int8_t* y, int64_t ldy, void* stream);

/* ------------------------------------------------------------------------------------------------
 * ibert_encoder_layer_i -- one post-LN encoder layer, integer-only end to end (Fig. 1 right for the
 * attention block; the RoBERTa layer of Sec. 4.1; INT8 MatMuls, INT32 non-linearities, requantization
 * after each, App. C.1).  T = batch*seq tokens, d = hidden/heads; head j owns columns [j*d, (j+1)*d) of
 * each of Q, K, V.  No mask, no dropout.  The result is defined as the composition of the primitives:
 *    1 qkv    = gemm(x, w_qkv; per-channel, I8)                          [T, 3*hidden]
 *    2 scores = gemm(Q_h, K_h; scores_dy, I32)  per (batch, head)        [batch*heads, seq, seq]
 *               (scores_dy carries S_q*S_k / (sqrt(d)*S_scores))
 *    3 probs  = softmax(scores; softmax)  I8                             [batch*heads, seq, seq]
 *    4 ctx    = gemm(probs, V_h (trans_w); ctx_dy, I8) written to        [T, hidden]
 *    5 r1     = gemm(ctx, w_o; per-channel, I32, clamp 32767) + DY(x; res1_dy)
 *    6 h1     = layernorm(r1; ln1)  I8
 *    7 f1     = gemm(h1, w_1; per-channel, I32, clamp gelu.q_max)        [T, ffn]
 *    8 g      = gelu(f1; gelu)  I8
 *    9 r2     = gemm(g, w_2; per-channel, I32, clamp 32767) + DY(h1; res2_dy)
 *   10 y      = layernorm(r2; ln2)  I8                                   [T, hidden]
 * weights: host struct of device pointers.  quant: host.  x, y: device int8 [T, hidden] (y may not
 * alias x).  workspace: device, 256-byte aligned, at least ibert_encoder_layer_workspace_bytes(); after
 * the call it holds every intermediate at the offsets ibert_encoder_layer_workspace_layout() reports.
 * Preconditions: hidden % heads == 0, hidden <= 1024, every primitive's own preconditions.
 * ---------------------------------------------------------------------------------------------- */
typedef struct {
    const int8_t*  w_qkv;  const int32_t* b_qkv;  const int32_t* m_qkv;  const int32_t* s_qkv;  /* [3H,H], [3H] */
    const int8_t*  w_o;    const int32_t* b_o;    const int32_t* m_o;    const int32_t* s_o;    /* [H,H],  [H]  */
    const int32_t* ln1_gamma_q;  const int32_t* ln1_beta_q;                                       /* [H]          */
    const int8_t*  w_1;    const int32_t* b_1;    const int32_t* m_1;    const int32_t* s_1;    /* [F,H],  [F]  */
    const int8_t*  w_2;    const int32_t* b_2;    const int32_t* m_2;    const int32_t* s_2;    /* [H,F],  [H]  */
    const int32_t* ln2_gamma_q;  const int32_t* ln2_beta_q;                                       /* [H]          */
} ibert_layer_weights;

typedef struct {
    ibert_dyadic scores_dy;
    ibert_softmax_params softmax;
    ibert_dyadic ctx_dy;
    ibert_dyadic res1_dy;
    int32_t ln1_shift;
    ibert_gelu_params gelu;
    ibert_dyadic res2_dy;
    int32_t ln2_shift;
    int32_t route;               /* 0: every fusion below; else IBERT_ROUTE_* flags OR-ed together */
} ibert_layer_quant;

/* Which kernels a layer call runs.  The result never depends on it (each fused kernel is bit-identical to the
 * composition it replaces; the tests run every combination); the flags exist so that each step can be run and looked
 * at by itself.  Default (0):
 *   - steps 7 and 8 (FFN up-projection and GELU) as one kernel where ibert_gemm_i8_gelu can do so; the workspace
 *     region f1 is then left untouched;
 *   - steps 2, 3 and 4 as one kernel where ibert_attention_i can do so; the workspace regions scores and probs are then
 *     left untouched (profile records: one, numbered 2);
 *   - r1 / r2, which are clamped to 16 bits by definition, stored as int16 [T, hidden] (IBERT_I16) at the start of their
 *     workspace regions and read by ibert_layernorm_i16: the two kernels move half the bytes. */
enum {
    IBERT_ROUTE_SEPARATE_GELU = 1,        /* step 7 writes f1 (int32), step 8 is a kernel of its own        */
    IBERT_ROUTE_SEPARATE_ATTENTION = 2,   /* steps 2, 3, 4 as three kernels through scores and probs        */
    IBERT_ROUTE_I32_LN_INPUT = 4          /* r1 / r2 stored as int32, steps 6 / 10 run ibert_layernorm_i     */
};

/* Byte offsets of the intermediates inside the workspace (each 256-byte aligned).  Element types are those of the step
 * list above, except that r1 / r2 hold int16 [T, hidden] (at the start of regions sized for int32) unless
 * IBERT_ROUTE_I32_LN_INPUT is set, and that a region whose tensor a fused kernel never materialises is left untouched. */
typedef struct {
    size_t qkv, scores, probs, ctx, r1, h1, f1, g, r2;
    size_t total;
} ibert_layer_workspace_layout;

size_t ibert_encoder_layer_workspace_bytes(int32_t batch, int32_t seq, int32_t hidden, int32_t heads, int32_t ffn);
int ibert_encoder_layer_workspace_layout(int32_t batch, int32_t seq, int32_t hidden, int32_t heads, int32_t ffn,
                                         ibert_layer_workspace_layout* out);

int ibert_encoder_layer_i(const ibert_layer_weights* weights, const ibert_layer_quant* quant,
                          const int8_t* x, int8_t* y,
                          int32_t batch, int32_t seq, int32_t hidden, int32_t heads, int32_t ffn,
                          void* workspace, size_t workspace_bytes, void* stream);

/* The layer over padded sequences: sequence b attends to its first key_lens[b] keys only (key_lens: device int32
 * [batch], read by the kernels, clamped into [1, seq]; see ibert_softmax_masked_i for the reading).  Every token
 * row, padded ones included, is still computed; on the first key_lens[b] tokens of a sequence the result equals the
 * layer run on that sequence alone at its own length.  key_lens == NULL is ibert_encoder_layer_i. */
int ibert_encoder_layer_masked_i(const ibert_layer_weights* weights, const ibert_layer_quant* quant,
                                 const int8_t* x, int8_t* y,
                                 int32_t batch, int32_t seq, int32_t hidden, int32_t heads, int32_t ffn,
                                 const int32_t* key_lens, void* workspace, size_t workspace_bytes, void* stream);

/* ibert_encoder_layer_static_i -- ibert_encoder_layer_masked_i for callers that cannot allocate device memory and have
 * no workspace to hand over: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The
 * intermediates live in an array inside the library's own device image (ibert_static_scratch_bytes() = 32 MiB; each GPU
 * the library runs on holds its copy until the process ends) instead of a caller's workspace; the call allocates and frees
 * nothing and gives the same y as ibert_encoder_layer_masked_i, bit for bit.  key_lens may be NULL (no padding).
 * Limit: ibert_encoder_layer_workspace_bytes(batch, seq, hidden, heads, ffn) must not exceed
 * ibert_static_scratch_bytes() -- e.g. up to 7 sequences of 128 tokens at hidden 768 / ffn 3072 -- else
 * IBERT_ERR_WORKSPACE and nothing is launched.  All calls on one GPU share that GPU's array: calls that overlap in time on
 * one GPU (two streams, two threads) race on it; calls on one stream, or ordered by events, are fine.  The array keeps
 * the last call's intermediates; no step depends on them (each region is written before it is read).
 * The array's address is looked up once per device, on the first call there (a host-side query of the loaded image, no
 * allocation); ibert_static_scratch_init() does that lookup for the current device ahead of time, e.g. before a graph
 * capture starts.  Errors otherwise as ibert_encoder_layer_masked_i. */
size_t ibert_static_scratch_bytes(void);
int ibert_static_scratch_init(void);
int ibert_encoder_layer_static_i(const ibert_layer_weights* weights, const ibert_layer_quant* quant,
                                 const int8_t* x, int8_t* y,
                                 int32_t batch, int32_t seq, int32_t hidden, int32_t heads, int32_t ffn,
                                 const int32_t* key_lens, void* stream);

/* n_layers layers back to back (layer l+1 reads layer l's output); weights/quant: host arrays of
 * n_layers entries.  x is not modified; y receives the last layer's output.  The workspace needs
 * ibert_encoder_workspace_bytes() (one layer's workspace plus two ping-pong activation buffers). */
size_t ibert_encoder_workspace_bytes(int32_t batch, int32_t seq, int32_t hidden, int32_t heads, int32_t ffn);
int ibert_encoder_i(const ibert_layer_weights* weights, const ibert_layer_quant* quant, int32_t n_layers,
                    const int8_t* x, int8_t* y,
                    int32_t batch, int32_t seq, int32_t hidden, int32_t heads, int32_t ffn,
                    void* workspace, size_t workspace_bytes, void* stream);
int ibert_encoder_masked_i(const ibert_layer_weights* weights, const ibert_layer_quant* quant, int32_t n_layers,
                           const int8_t* x, int8_t* y,
                           int32_t batch, int32_t seq, int32_t hidden, int32_t heads, int32_t ffn,
                           const int32_t* key_lens, void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------------------------
 * Host-only helpers: the one place where a real number appears.  All arithmetic is IEEE binary64 in
 * the written order followed by floor (or round-half-even where "rint" is written).
 * ---------------------------------------------------------------------------------------------- */

/* M ~ m/2^s with |m| in [2^30, 2^31).  |M| < 2^-32 gives (0,0); |M| >= 2^31 or non-finite is refused. */
int ibert_dyadic_from_double(double M, ibert_dyadic* out);

/* mult[n], shift[n] <- dyadic(S_in * S_w[n] / S_out), n < N (host arrays). */
int ibert_channel_dyadics_from_scales(double S_in, const double* S_w, int32_t N, double S_out,
                                      int32_t* mult, int32_t* shift);

/* Alg. 3 + Alg. 1 with a,b,c = 0.3585, 1.353, 0.344:  q_ln2 = floor(ln2/S), q_b = floor(b/S),
 * q_c = floor(c/(a*S*S)).  Checks the preconditions of ibert_softmax_i for `cols`. */
int ibert_softmax_params_from_scale(double S, int32_t cols, int32_t out_frac_bits, int32_t out_dtype,
                                    ibert_softmax_params* out);

/* Alg. 2 with a,b,c = -0.2888, -1.769, 1:  S' = S_in/sqrt(2); q_b = floor(b/S'); S_erf = a*S'*S';
 * q_c = q_1 = floor(1/S_erf); q_max = floor((2^31-1) / (max(|q_c|,|q_b^2+q_c|) + |q_1|));
 * out = dyadic((S_in*S_erf/2) / S_out). */
int ibert_gelu_params_from_scale(double S_in, double S_out, ibert_gelu_params* out);
/* h-GELU: slope = dyadic(1.702), q_3 = floor(3/S_in), q_6 = floor(6/S_in), q_max = floor((2^31-1) / max(1, q_6)),
 * out = dyadic(S_in^2 / (6 S_out)).  S_in, S_out > 0 and finite, q_6 must fit 31 bits. */
int ibert_hgelu_params_from_scale(double S_in, double S_out, ibert_hgelu_params* out);

/* gamma_q[i] = rint(gamma[i]/S_out * 2^(shift-10)), beta_q[i] = rint(beta[i]/S_out * 2^shift) with the
 * largest shift in [1,30] such that max|gamma_q| < 2^14 and max|beta_q| < 2^29 (host arrays). */
int ibert_layernorm_params_from_float(const double* gamma, const double* beta, int32_t C, double S_out,
                                      int32_t* gamma_q, int32_t* beta_q, int32_t* shift);

/* Real-valued static scales of one layer's activation tensors -> ibert_layer_quant (per-tensor part).
 * scores_dy = dyadic(S_q*S_k / (sqrt(d)*S_s)); ctx_dy = dyadic(2^-k * S_v / S_ctx);
 * res1_dy = dyadic(S_x/S_r1); res2_dy = dyadic(S_h1/S_r2); softmax from (S_s, seq, k); gelu from
 * (S_g_in, S_g_out).  The LayerNorm shifts are filled by the caller from ibert_layernorm_params_from_float. */
typedef struct {
    double S_x, S_q, S_k, S_v, S_s, S_ctx, S_r1, S_h1, S_g_in, S_g_out, S_r2, S_y;
    int32_t softmax_k;
} ibert_layer_scales;

int ibert_layer_quant_from_scales(const ibert_layer_scales* scales, int32_t seq, int32_t head_dim,
                                  ibert_layer_quant* out);

/* ------------------------------------------------------------------------------------------------
 * ibert_attention_i -- the self-attention core of the layer (Fig. 1 right; Sec. 4.1; Alg. 3), steps 2-4 of
 * ibert_encoder_layer_i, bit-identical to
 *     scores = ibert_gemm_i8_requant(Q_h, K_h; scores_dy, INT32)          per (batch, head): [seq, seq]
 *     probs  = ibert_softmax_i(scores; softmax)                            INT8
 *     ctx    = ibert_gemm_i8_requant(probs, V_h as [K,N]; ctx_dy, INT8, clamp 127), written into [T, hidden]
 * qkv: device int8 [batch*seq, 3*hidden] (Q | K | V, the heads of each side by side); ctx: device int8
 * [batch*seq, hidden].  softmax->out_dtype must be IBERT_I8.
 * With seq in {128, 256, 384, 512} and hidden/heads = 64 (qkv 16-byte aligned, ctx 4-byte aligned) the three steps
 * run as one kernel and scores/probs are never stored.  Any other shape takes the
 * three-kernel route through `scratch` (device, 256-byte aligned, ibert_attention_scratch_bytes() bytes;
 * IBERT_ERR_WORKSPACE if it is NULL, small or misaligned).  scratch may always be passed.
 * ---------------------------------------------------------------------------------------------- */
size_t ibert_attention_scratch_bytes(int32_t batch, int32_t seq, int32_t heads);
int ibert_attention_i(const int8_t* qkv, int8_t* ctx, int32_t batch, int32_t seq, int32_t hidden, int32_t heads,
                      const ibert_dyadic* scores_dy, const ibert_softmax_params* softmax, const ibert_dyadic* ctx_dy,
                      void* scratch, size_t scratch_bytes, void* stream);
/* With padded sequences: key_lens as for ibert_encoder_layer_masked_i (NULL: no padding). */
int ibert_attention_masked_i(const int8_t* qkv, int8_t* ctx, int32_t batch, int32_t seq, int32_t hidden, int32_t heads,
                             const ibert_dyadic* scores_dy, const ibert_softmax_params* softmax,
                             const ibert_dyadic* ctx_dy, const int32_t* key_lens, void* scratch, size_t scratch_bytes,
                             void* stream);

/* ------------------------------------------------------------------------------------------------
 * Optional instrumentation for benchmarks (not part of the method): while a profile is open,
 * ibert_encoder_layer_i / ibert_encoder_i bracket each of the ten steps with HIP events on the caller's
 * stream.  ibert_profile_begin creates the events (host objects; no device memory) for up to `capacity`
 * steps; ibert_profile_end waits for the recorded events, fills `out` (host) with one record per executed
 * step, destroys the events and closes the profile.  Steps beyond the capacity are not recorded.
 * Not thread-safe; one profile at a time.
 * ---------------------------------------------------------------------------------------------- */
typedef struct {
    int32_t step;        /* 1..10, the step numbers of ibert_encoder_layer_i */
    float ms;            /* event-to-event time of the step's launch(es); includes what the two event records cost */
    double ops;          /* algorithmic integer ops: 2*M*N*K*batch for MatMul steps, 0 otherwise */
    double bytes;        /* algorithmic bytes: operands read once + outputs written once */
    char kernel[96];     /* name of the kernel the step launched, as a profiler shows it (without namespace) */
} ibert_profile_record;

int ibert_profile_begin(int32_t capacity);
int ibert_profile_end(ibert_profile_record* out, int32_t capacity, int32_t* count);

const char* ibert_status_string(int status);
const char* ibert_last_hip_error(void);
int ibert_version(void);

#ifdef __cplusplus
}
#endif
#endif /* IBERT_H */
