"""Pins for the tensor-level oracle functions (no GPU): GEMM+requant, I-Softmax, I-GELU, I-LayerNorm, layer.

Expected values come from library routines (numpy matmul), exact rationals, closed forms, invariants and the
float counterparts of each op applied to the dequantised inputs -- never from the HIP path.
"""
import math
from fractions import Fraction

import numpy as np
import pytest

import oracle
from oracle import params as P, GemmSpec, I8, I32
from paper_2101_01321_amd import synth
import fpref

RNG = np.random.default_rng(99)


def _round_half_up_rational(acc, m, s):
    return math.floor(Fraction(int(acc) * int(m), 2 ** int(s)) + Fraction(1, 2))


# ------------------------------------------------------------------ GEMM + requant
def test_gemm_matches_numpy_matmul_and_rational_rounding():
    M, N, K = 37, 29, 83                       # all different so a transposed operand cannot pass
    A = RNG.integers(-127, 128, size=(M, K), dtype=np.int8)
    W = RNG.integers(-127, 128, size=(N, K), dtype=np.int8)
    bias = RNG.integers(-2 ** 15, 2 ** 15 + 1, size=N, dtype=np.int32)
    mult = RNG.integers(2 ** 30, 2 ** 31, size=N).astype(np.int32) * RNG.choice([-1, 1], size=N).astype(np.int32)
    shift = RNG.integers(38, 46, size=N).astype(np.int32)
    acc = A.astype(np.int64) @ W.astype(np.int64).T + bias.astype(np.int64)
    got = oracle.gemm_requant(GemmSpec(M, N, K, out_dtype=I32, out_clamp=2 ** 31 - 1), A, W, bias, mult, shift)
    got = got.reshape(M, N)
    for i in range(M):
        for n in range(N):
            assert got[i, n] == _round_half_up_rational(acc[i, n], mult[n], shift[n])
    # int8 output: same numbers clamped to +-127
    got8 = oracle.gemm_requant(GemmSpec(M, N, K), A, W, bias, mult, shift).reshape(M, N)
    assert np.array_equal(got8, np.clip(got, -127, 127).astype(np.int8))
    assert np.abs(got).max() > 127             # the clamp was exercised


def test_gemm_identity_weights_reproduce_input():
    K = 48
    A = RNG.integers(-127, 128, size=(21, K), dtype=np.int8)
    W = np.eye(K, dtype=np.int8)
    one = np.full(K, 2 ** 30, dtype=np.int32), np.full(K, 30, dtype=np.int32)
    out = oracle.gemm_requant(GemmSpec(21, K, K), A, W, None, *one).reshape(21, K)
    assert np.array_equal(out, A)
    # 1x1x1
    out = oracle.gemm_requant(GemmSpec(1, 1, 1, per_channel=0, dy=(3, 1), out_dtype=I32, out_clamp=10 ** 6),
                              np.array([[-5]], np.int8), np.array([[7]], np.int8))
    assert out[0] == -52                        # -35*3/2 = -52.5 -> half up -> -52


def test_gemm_trans_w_and_batch_strides_and_residual():
    B, nh, L, d = 2, 3, 10, 8
    H = nh * d
    qkv = RNG.integers(-127, 128, size=(B * L, 3 * H), dtype=np.int8)
    # scores: batched Q_h K_h^T through strides on the packed [T,3H] buffer
    spec = GemmSpec(L, L, d, lda=3 * H, ldw=3 * H, ldc=L, batch_outer=B, batch_inner=nh,
                    sA=(L * 3 * H, d), sW=(L * 3 * H, d), sC=(nh * L * L, L * L),
                    per_channel=0, dy=(2 ** 30, 30), out_dtype=I32, out_clamp=2 ** 31 - 1)
    flat = qkv.reshape(-1)
    sc = oracle.gemm_requant(spec, flat, flat[H:], out_elems=B * nh * L * L).reshape(B, nh, L, L)
    q4 = qkv.reshape(B, L, 3, nh, d).astype(np.int64)
    want = np.einsum("blhd,bmhd->bhlm", q4[:, :, 0], q4[:, :, 1])
    assert np.array_equal(sc, want)
    # context: P V_h with W given as [K,N] (trans_w), output scattered back into [T,H]
    Pm = RNG.integers(0, 128, size=(B, nh, L, L), dtype=np.int8)
    spec = GemmSpec(L, d, L, lda=L, ldw=3 * H, ldc=H, batch_outer=B, batch_inner=nh, trans_w=1,
                    sA=(nh * L * L, L * L), sW=(L * 3 * H, d), sC=(L * H, d),
                    per_channel=0, dy=(2 ** 30, 30), out_dtype=I32, out_clamp=2 ** 31 - 1)
    ctx = oracle.gemm_requant(spec, Pm.reshape(-1), flat[2 * H:], out_elems=B * L * H).reshape(B, L, nh, d)
    want = np.einsum("bhlm,bmhd->blhd", Pm.astype(np.int64), q4[:, :, 2])
    assert np.array_equal(ctx, want)
    # residual: out = DY(acc) + DY(res), then clamp
    M, N, K = 9, 7, 16
    A = RNG.integers(-127, 128, size=(M, K), dtype=np.int8)
    W = RNG.integers(-127, 128, size=(N, K), dtype=np.int8)
    R = RNG.integers(-127, 128, size=(M, N), dtype=np.int8)
    spec = GemmSpec(M, N, K, per_channel=0, dy=(3 * 2 ** 29, 36), out_dtype=I32, out_clamp=300, res_dy=(5 * 2 ** 28, 27))
    out = oracle.gemm_requant(spec, A, W, residual=R).reshape(M, N)
    acc = A.astype(np.int64) @ W.astype(np.int64).T
    for i in range(M):
        for n in range(N):
            v = _round_half_up_rational(acc[i, n], 3 * 2 ** 29, 36) + _round_half_up_rational(R[i, n], 5 * 2 ** 28, 27)
            assert out[i, n] == max(-300, min(300, v))


def test_gemm_requant_tracks_float_linear():
    M, N, K = 64, 48, 96
    A, W, sw, b = synth.gemm_operands(M, N, K)
    S_in, S_out = 0.03, 0.5
    mult, shift = P.channel_dyadics(S_in, sw, S_out)
    out = oracle.gemm_requant(GemmSpec(M, N, K), A, W, b, mult, shift).reshape(M, N)
    real = fpref.linear(A.astype(np.float64) * S_in, W, sw, b, S_in)
    want = np.clip(real / S_out, -127, 127)
    assert np.max(np.abs(out - want)) <= 0.5 + 1e-6


def test_gemm_rejects_bad_parameters():
    A = np.zeros((2, 2), np.int8)
    with pytest.raises(oracle.OracleError):
        oracle.gemm_requant(GemmSpec(2, 2, 2, per_channel=0, dy=(1, 63)), A, A)
    with pytest.raises(oracle.OracleError):
        oracle.gemm_requant(GemmSpec(2, 2, 2, per_channel=0, dy=(1, 1), out_clamp=128), A, A)


# ------------------------------------------------------------------ I-Softmax
@pytest.mark.parametrize("cols", [128, 512, 77])
def test_softmax_vs_float_and_row_sum(cols):
    q, S = synth.softmax_logits(300, cols)
    sp = P.softmax_params(S)
    out = oracle.softmax(q, sp)
    assert out.min() >= 0 and out.max() <= 127
    ref = fpref.softmax(q.astype(np.float64) * S)
    assert np.max(np.abs(out / 128.0 - ref)) <= 0.02
    # every output is rounded to nearest (<= 1/2 each) and Fz = floor(2^31/sum) loses < sum/2^31 relative
    assert np.all(np.abs(out.sum(axis=1) - 128) <= cols / 2 + 2)


def test_softmax_i32_mode_sums_to_fixed_point_one():
    cols, k = 128, 24
    q, S = synth.softmax_logits(64, cols)
    sp = P.softmax_params(S, out_frac_bits=k, out_dtype=I32)
    out = oracle.softmax(q, sp).astype(np.int64)
    # sum_j round(e_j Fz / 2^(31-k)) with 2^31 - sum < Fz*sum <= 2^31  and sum < 2^31/..., |rounding| <= 1/2 each
    sums = out.sum(axis=1)
    top = (sp.q_b ** 2 + sp.q_c) * cols
    assert np.all(sums <= 2 ** k + cols / 2)
    assert np.all(sums >= 2 ** k - cols / 2 - top / 2 ** (31 - k) - 1)
    ref = fpref.softmax(q.astype(np.float64) * S)
    assert np.max(np.abs(out / 2.0 ** k - ref)) <= 0.012     # no int8 rounding in this mode


def test_softmax_invariants_and_special_rows():
    S = 2.0 ** -6
    sp = P.softmax_params(S)
    q, _ = synth.softmax_logits(16, 96)
    base = oracle.softmax(q, sp)
    # adding a constant to a row changes nothing (Eq. 11), also near the int32 limits
    assert np.array_equal(oracle.softmax(q + 12345, sp), base)
    big = q.astype(np.int64) - q.max() + (2 ** 31 - 1)
    assert np.array_equal(oracle.softmax(big.astype(np.int32), sp), base)
    # permuting a row permutes the output
    perm = RNG.permutation(96)
    assert np.array_equal(oracle.softmax(q[:, perm], sp), base[:, perm])
    # all-equal row: every output is the rounded 128/cols
    for cols in (2, 7, 64, 128):
        out = oracle.softmax(np.full((1, cols), -321, np.int32), sp)
        assert np.all(np.abs(out - 128.0 / cols) <= 0.5 + 1e-3 * 128)
        assert len(set(out[0].tolist())) == 1
    # one element far above the rest (>= 31 ln2 in integer units): a one-hot row, saturated at 127
    row = np.full((1, 50), -10 ** 6, np.int32)
    row[0, 17] = 5
    out = oracle.softmax(row, sp)
    assert out[0, 17] == 127 and out.sum() == 127
    # extreme spread
    row = np.array([[-2 ** 31, 2 ** 31 - 1, 0]], np.int32)
    assert oracle.softmax(row, sp).tolist() == [[0, 127, 0]]
    # two equal maxima, others negligible: 64 each
    row = np.full((1, 9), -10 ** 5, np.int32)
    row[0, 2] = row[0, 5] = 40
    out = oracle.softmax(row, sp)
    assert out[0, 2] == out[0, 5] == 64 and out.sum() == 128


def test_softmax_precondition():
    sp = P.softmax_params(2.0 ** -12)
    assert oracle.lib().orc_softmax_check(sp, 128) == oracle.E_PARAM   # 128 * (q_b^2+q_c) >= 2^31
    assert oracle.lib().orc_softmax_check(P.softmax_params(2.0 ** -6), 512) == 0


# ------------------------------------------------------------------ I-GELU (tensor)
@pytest.mark.parametrize("S_in,S_out", [(2.0 ** -7, 8.0 / 127), (2.0 ** -6, 0.41), (0.011, 0.05)])
def test_gelu_vs_float(S_in, S_out):
    q, _ = synth.gelu_inputs(64, 257, scale=S_in)
    gp = P.gelu_params(S_in, S_out)
    out = oracle.gelu(q, gp)
    x = np.clip(q, -gp.q_max, gp.q_max) * S_in
    want = np.clip(fpref.gelu(x) / S_out, -127, 127)
    # Table 1 gap + scale flooring (see the scalar pins) + half an output step
    assert np.max(np.abs(out - want)) <= (0.0182 + S_in + 1.5 * S_in ** 2) / S_out + 0.5 + 1e-6
    assert np.all(out[q < gp.q_b * 2] == 0)


# ------------------------------------------------------------------ I-LayerNorm
@pytest.mark.parametrize("C", [256, 768, 1024, 100])
def test_layernorm_vs_float(C):
    q, S, gamma, beta = synth.layernorm_inputs(200, C)
    S_out = 5.0 / 127
    gq, bq, s = P.layernorm_params(gamma, beta, S_out)
    assert oracle.lib().orc_layernorm_check(C, gq.ctypes.data, bq.ctypes.data, s) == 0
    out = oracle.layernorm(q, gq, bq, s)
    want = np.clip(fpref.layernorm(q * S, gamma, beta) / S_out, -127, 127)
    assert np.max(np.abs(out - want)) <= 1.0


def test_layernorm_special_rows():
    C = 64
    gamma = np.linspace(0.7, 1.3, C)
    beta = np.linspace(-0.4, 0.4, C)
    S_out = 0.02
    gq, bq, s = P.layernorm_params(gamma, beta, S_out)
    # constant row: variance 0, sigma clamps to 1, d = 0 -> out = round(beta/S_out)
    out = oracle.layernorm(np.full((1, C), 777, np.int32), gq, bq, s)
    assert np.max(np.abs(out[0] - beta / S_out)) <= 0.5 + 1e-3
    # +-a alternating (a power of two): mu = 0, sigma = a, normalised values are exactly +-1
    for a in (1, 64, 4096, 16384):
        x = (a * (-1) ** np.arange(C)).astype(np.int32)[None, :]
        out = oracle.layernorm(x, gq, bq, s)
        want = ((-1.0) ** np.arange(C) * gamma + beta) / S_out
        assert np.max(np.abs(out[0] - np.clip(want, -127, 127))) <= 0.5 + 2e-3 * 127
    # scale invariance in the exact case: doubling the +-a row changes nothing
    x = (64 * (-1) ** np.arange(C)).astype(np.int32)[None, :]
    assert np.array_equal(oracle.layernorm(x, gq, bq, s), oracle.layernorm(2 * x, gq, bq, s))
    # adversarial rows stay inside every 32-bit bound (the oracle would return E_RANGE otherwise)
    for row in (np.r_[32767, np.zeros(1023)], 32767 * (-1) ** np.arange(1024), np.r_[1, np.zeros(1023)],
                np.r_[-32767 * np.ones(512), 32767 * np.ones(512)], 10 ** 9 * np.ones(1024)):
        g1024, b1024, s1024 = P.layernorm_params(np.full(1024, 1.4), np.full(1024, 0.4), S_out)
        oracle.layernorm(row.astype(np.int32)[None, :], g1024, b1024, s1024)
    # inputs are clamped to +-(2^15-1) on load
    x = RNG.integers(-40000, 40000, size=(3, C)).astype(np.int32)
    assert np.array_equal(oracle.layernorm(x, gq, bq, s), oracle.layernorm(np.clip(x, -32767, 32767), gq, bq, s))


def test_layernorm_mean_rounding_and_population_variance():
    # gamma = 1, beta = 0, S_out = 2^-10/.. chosen so the output shows the normalised value itself
    C = 4
    gq, bq, s = P.layernorm_params(np.ones(C), np.zeros(C), 1.0 / 64)
    # row (0,0,0,8): mean 2, population variance (4+4+4+36)/4 = 12 (sample variance would be 16), sigma = 3
    out = oracle.layernorm(np.array([[0, 0, 0, 8]], np.int32), gq, bq, s)
    want = np.array([-2, -2, -2, 6]) / 3.0 * 64
    assert np.max(np.abs(out[0] - np.clip(want, -127, 127))) <= 1.0
    # row (1,2,2,2): sum 7, mean rounds half up to 2 -> d = (-1,0,0,0), sigma = max(1, 0)
    out = oracle.layernorm(np.array([[1, 2, 2, 2]], np.int32), gq, bq, s)
    assert out[0].tolist() == [-64, 0, 0, 0]


# ------------------------------------------------------------------ encoder layer, teacher-forced per op
@pytest.mark.parametrize("cfg", [synth.CONFIGS["tiny"],
                                 synth.EncoderConfig("ragged", 192, 3, 320, 40, 2, 1)])
def test_encoder_layer_each_step_tracks_its_float_counterpart(cfg):
    x_q, S_x, _ = synth.input_activations(cfg)
    sc = synth.static_scales(cfg, S_x)
    raw = synth.layer_raw(cfg, 0)
    w, q = P.layer_params(raw, sc, cfg.hidden, cfg.heads)
    y, d = oracle.encoder_layer(w, q, x_q, cfg.batch, cfg.seq, cfg.hidden, cfg.heads, cfg.ffn, dump=True)
    B, L, H, nh, F = cfg.batch, cfg.seq, cfg.hidden, cfg.heads, cfg.ffn
    dh = H // nh
    eps = 1e-5
    xr = x_q * S_x
    # 1 qkv
    S_qkv = np.r_[np.full(H, sc["S_q"]), np.full(H, sc["S_k"]), np.full(H, sc["S_v"])]
    want = np.clip(fpref.linear(xr, raw["w_qkv"], raw["sw_qkv"], raw["b_qkv"], S_x) / S_qkv, -127, 127)
    assert np.max(np.abs(d["qkv"] - want)) <= 0.5 + eps
    # 2 scores (float uses the integer qkv, dequantised)
    qkv = d["qkv"].reshape(B, L, 3, nh, dh).astype(np.float64)
    Q, K, V = qkv[:, :, 0] * sc["S_q"], qkv[:, :, 1] * sc["S_k"], qkv[:, :, 2] * sc["S_v"]
    s_real = np.einsum("blhd,bmhd->bhlm", Q, K) / math.sqrt(dh)
    want = (s_real / sc["S_s"]).reshape(B * nh, L, L)
    assert np.max(np.abs(d["scores"] - want)) <= 0.5 + np.max(np.abs(want)) * 2.0 ** -30
    # 3 softmax
    want = fpref.softmax(d["scores"] * sc["S_s"])
    assert np.max(np.abs(d["probs"] / 128.0 - want)) <= 0.02
    # 4 context
    Pm = d["probs"].reshape(B, nh, L, L) / 128.0
    want = np.clip(np.einsum("bhlm,bmhd->blhd", Pm, V).reshape(B * L, H) / sc["S_ctx"], -127, 127)
    assert np.max(np.abs(d["ctx"] - want)) <= 0.5 + eps
    # 5 out-proj + residual (two roundings)
    want = (fpref.linear(d["ctx"] * sc["S_ctx"], raw["w_o"], raw["sw_o"], raw["b_o"], sc["S_ctx"]) + xr) / sc["S_r1"]
    assert np.max(np.abs(d["r1"] - np.clip(want, -32767, 32767))) <= 1.0 + 1e-3
    # 6 LayerNorm
    want = np.clip(fpref.layernorm(d["r1"] * sc["S_r1"], raw["gamma1"], raw["beta1"]) / sc["S_h1"], -127, 127)
    assert np.max(np.abs(d["h1"] - want)) <= 1.0
    # 7 FFN1
    h1r = d["h1"] * sc["S_h1"]
    want = fpref.linear(h1r, raw["w_1"], raw["sw_1"], raw["b_1"], sc["S_h1"]) / sc["S_g_in"]
    assert np.max(np.abs(d["f1"] - np.clip(want, -q.gelu.q_max, q.gelu.q_max))) <= 0.5 + 1e-3
    # 8 GELU
    want = np.clip(fpref.gelu(d["f1"] * sc["S_g_in"]) / sc["S_g_out"], -127, 127)
    assert np.max(np.abs(d["g"] - want)) <= (0.0182 + sc["S_g_in"] + 1.5 * sc["S_g_in"] ** 2 +
                                             600 * 0.1445 * sc["S_g_in"] ** 2) / sc["S_g_out"] + 0.5
    # 9 FFN2 + residual
    want = (fpref.linear(d["g"] * sc["S_g_out"], raw["w_2"], raw["sw_2"], raw["b_2"], sc["S_g_out"]) + h1r) / sc["S_r2"]
    assert np.max(np.abs(d["r2"] - np.clip(want, -32767, 32767))) <= 1.0 + 1e-3
    # 10 LayerNorm
    want = np.clip(fpref.layernorm(d["r2"] * sc["S_r2"], raw["gamma2"], raw["beta2"]) / sc["S_y"], -127, 127)
    assert np.max(np.abs(y - want)) <= 1.0
    # the layer is the composition of the standalone ops
    assert np.array_equal(oracle.softmax(d["scores"], q.softmax), d["probs"])
    assert np.array_equal(oracle.gelu(d["f1"], q.gelu), d["g"])
    assert np.array_equal(oracle.layernorm(d["r2"], w["ln2_gamma_q"], w["ln2_beta_q"], q.ln2_shift), y)


# ------------------------------------------------------------------ padded keys
def _masked_case():
    cfg = synth.EncoderConfig("masked", 128, 2, 256, 48, 3, 1)
    x_q, S_x, _ = synth.input_activations(cfg)
    sc = synth.model_scales(cfg, S_x)
    w, q = P.layer_params(synth.layer_raw(cfg, 0), sc[0], cfg.hidden, cfg.heads)
    return cfg, x_q, w, q


def test_masked_keys_equal_a_shorter_sequence():
    # A sequence padded to L with its keys masked must give, on its valid tokens, exactly what the same tokens
    # give as a sequence of their own length: nothing but the attention looks across tokens.
    cfg, x_q, w, q = _masked_case()
    B, L, H = cfg.batch, cfg.seq, cfg.hidden
    lens = np.array([L, 29, 1], np.int32)
    y = oracle.encoder_layer(w, q, x_q, B, L, H, cfg.heads, cfg.ffn, key_lens=lens).reshape(B, L, H)
    for b, n in enumerate(lens):
        alone = oracle.encoder_layer(w, q, x_q.reshape(B, L, H)[b, :n], 1, int(n), H, cfg.heads, cfg.ffn)
        assert np.array_equal(y[b, :n], alone), "sequence %d" % b
    # and masking nothing is the unmasked layer
    full = np.full(B, L, np.int32)
    assert np.array_equal(oracle.encoder_layer(w, q, x_q, B, L, H, cfg.heads, cfg.ffn, key_lens=full),
                          oracle.encoder_layer(w, q, x_q, B, L, H, cfg.heads, cfg.ffn))


def test_masked_keys_get_probability_zero_and_rows_still_sum_to_one():
    cfg, x_q, w, q = _masked_case()
    B, L, H, nh = cfg.batch, cfg.seq, cfg.hidden, cfg.heads
    lens = np.array([L, 17, 40], np.int32)
    _, d = oracle.encoder_layer(w, q, x_q, B, L, H, nh, cfg.ffn, dump=True, key_lens=lens)
    probs = d["probs"].reshape(B, nh, L, L)
    for b, n in enumerate(lens):
        assert np.all(probs[b, :, :, n:] == 0)
        assert np.all(np.abs(probs[b, :, :, :n].astype(np.int64).sum(-1) - 128) <= n // 2 + 1)   # sum of n roundings of a unit mass
    assert np.all(d["scores"].reshape(B, nh, L, L)[1, :, :, 17:] == -2 ** 31)
    # the mask itself: only the padded columns change
    sc0 = RNG.integers(-50000, 50000, size=(B * nh, L, L)).astype(np.int32)
    m = oracle.mask_scores(sc0, B, nh, L, lens).reshape(B, nh, L, L)
    for b, n in enumerate(lens):
        assert np.array_equal(m[b, :, :, :n], sc0.reshape(B, nh, L, L)[b, :, :, :n]) and np.all(m[b, :, :, n:] == -2 ** 31)
    for bad in ([L, 0, 5], [L + 1, 3, 3]):
        with pytest.raises(oracle.OracleError):
            oracle.mask_scores(sc0, B, nh, L, np.array(bad, np.int32))


# ------------------------------------------------------------------ INT8 embedding
def test_embedding_vs_big_int_and_float():
    H, V, Pmax, seq, T = 96, 50, 40, 20, 60
    emb = synth.embedding_raw(H, V, Pmax)
    S_out = 5.0 / 127
    tok_dy, pos_dy, gq, bq, s = P.embedding_params(emb, S_out)
    ids = synth.token_ids(T, V)
    ids[:4] = [0, V - 1, -7, V + 100]                                  # the last two are clamped into the table
    y, r = oracle.embedding(ids, seq, emb["tok"], emb["pos"], tok_dy, pos_dy, gq, bq, s, return_sum=True)
    # the INT32 sum, element by element in Python integers
    cid = np.clip(ids, 0, V - 1)
    for t in (0, 1, 2, 3, 19, 20, 21, 59):
        for c in (0, 1, H - 1):
            a = (int(emb["tok"][cid[t], c]) * tok_dy[0] + (1 << (tok_dy[1] - 1))) >> tok_dy[1]
            b = (int(emb["pos"][t % seq, c]) * pos_dy[0] + (1 << (pos_dy[1] - 1))) >> pos_dy[1]
            assert r[t, c] == max(-32767, min(32767, a + b))
    # position = t mod seq: tokens t and t + seq with the same id get the same row
    ids2 = np.r_[np.arange(seq), np.arange(seq)].astype(np.int32) % V
    y2 = oracle.embedding(ids2, seq, emb["tok"], emb["pos"], tok_dy, pos_dy, gq, bq, s)
    assert np.array_equal(y2[:seq], y2[seq:])
    # it is the LayerNorm of that sum
    assert np.array_equal(y, oracle.layernorm(r, gq, bq, s))
    # and tracks the float embedding: LN(tok S_tok + pos S_pos) gamma + beta
    real = emb["tok"][cid].astype(np.float64) * emb["S_tok"] + emb["pos"][np.arange(T) % seq].astype(np.float64) * emb["S_pos"]
    assert np.max(np.abs(r * emb["S_r"] - real)) <= emb["S_r"] * 1.0 + 1e-9           # two roundings of half a step each
    want = np.clip(fpref.layernorm(real, emb["gamma"], emb["beta"]) / S_out, -127, 127)
    assert np.max(np.abs(y - want)) <= 1.5
