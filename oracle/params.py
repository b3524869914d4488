"""The oracle's own derivation of integer constants from real scales (test infrastructure).

Static quantization (Sec. 3.1, App. A): every scale is fixed before inference, so
q_b, q_c, q_ln2, q_1 and all requantization multipliers are pre-computed on the host
(footnote of Alg. 1).  Everything here is IEEE binary64 evaluated in the written order,
followed by a mathematical floor (or round-half-even where stated).
"""
from __future__ import annotations

import math

import numpy as np

from . import GeluT, HGeluT, LayerQuantT, SoftmaxT, I8, I32

LN2 = 0.6931471805599453  # ln 2 rounded to binary64


def dyadic_from_double(M: float):
    """M ~ m / 2^s with |m| in [2^30, 2^31) (31 significant bits), 0 <= s <= 62.

    Multipliers below 2^-32 (s would exceed 62) become (0, 0); multipliers of 2^31 or more are refused.
    """
    if M == 0.0 or not math.isfinite(M):
        if M == 0.0:
            return 0, 0
        raise ValueError("multiplier is not finite")
    f, e = math.frexp(abs(M))           # |M| = f * 2^e, f in [0.5, 1)
    m = int(round(f * 2147483648.0))    # exact product, round half to even
    if m == 2147483648:
        m, e = 1073741824, e + 1
    s = 31 - e
    if s > 62:
        return 0, 0
    if s < 0:
        raise ValueError("multiplier too large for a dyadic with s >= 0")
    return (-m if M < 0 else m), s


def channel_dyadics(S_in: float, S_w, S_out: float):
    """Per-output-channel requantization multipliers M[n] = S_in * S_w[n] / S_out (App. C.1)."""
    S_w = np.asarray(S_w, dtype=np.float64)
    mult = np.empty(S_w.shape, dtype=np.int32)
    shift = np.empty(S_w.shape, dtype=np.int32)
    for n, sw in enumerate(S_w.tolist()):
        m, s = dyadic_from_double(S_in * sw / S_out)
        mult[n], shift[n] = m, s
    return mult, shift


def softmax_params(S: float, out_frac_bits: int = 7, out_dtype: int = I8) -> SoftmaxT:
    """Alg. 3 with Alg. 1: q_ln2 = floor(ln2/S), q_b = floor(b/S), q_c = floor(c/(a S^2)); a,b,c of Eq. 13."""
    a, b, c = 0.3585, 1.353, 0.344
    p = SoftmaxT()
    p.q_ln2 = math.floor(LN2 / S)
    p.q_b = math.floor(b / S)
    p.q_c = math.floor(c / (a * S * S))
    p.out_frac_bits = out_frac_bits
    p.out_dtype = out_dtype
    return p


def softmax_exp_scale(S: float) -> float:
    """S_out of I-Exp = a S^2 (Alg. 1; the floor printed there would make it zero)."""
    return 0.3585 * S * S


def gelu_params(S_in: float, S_out: float) -> GeluT:
    """Alg. 2: I-Erf is called with S' = S/sqrt(2); a,b,c of Eq. 8; q_1 = floor(1/S_erf); S_t = S*S_erf/2."""
    a, b = -0.2888, -1.769
    Sp = S_in / math.sqrt(2.0)
    S_erf = a * Sp * Sp
    p = GeluT()
    p.q_b = math.floor(b / Sp)
    p.q_c = math.floor(1.0 / S_erf)
    p.q_1 = math.floor(1.0 / S_erf)
    bound = max(abs(p.q_c), abs(p.q_b * p.q_b + p.q_c)) + abs(p.q_1)
    p.q_max = (2 ** 31 - 1) // bound
    S_t = S_in * S_erf / 2.0
    p.out_m, p.out_s = dyadic_from_double(S_t / S_out)
    return p


def hgelu_params(S_in: float, S_out: float) -> HGeluT:
    """Eq. 6 on integers of scale S: slope = dyadic(1.702), q_3 = floor(3/S), q_6 = floor(6/S), q_max the largest
    input for which q*q_6 fits 31 bits, out = dyadic(S^2 / (6 S_out))."""
    p = HGeluT()
    p.slope_m, p.slope_s = dyadic_from_double(1.702)
    p.q_3 = math.floor(3.0 / S_in)
    p.q_6 = math.floor(6.0 / S_in)
    p.q_max = (2 ** 31 - 1) // max(1, p.q_6)
    p.out_m, p.out_s = dyadic_from_double(S_in * S_in / (6.0 * S_out))
    return p


def gelu_t_scale(S_in: float) -> float:
    Sp = S_in / math.sqrt(2.0)
    return S_in * (-0.2888 * Sp * Sp) / 2.0


def layernorm_params(gamma, beta, S_out: float):
    """gamma_q = rint(gamma/S_out * 2^(s-10)), beta_q = rint(beta/S_out * 2^s); s is the largest shift in
    [1, 30] with max|gamma_q| < 2^14 and max|beta_q| < 2^29 (normalised values carry 10 fractional bits)."""
    gamma = np.asarray(gamma, dtype=np.float64)
    beta = np.asarray(beta, dtype=np.float64)
    for s in range(30, 0, -1):
        gq = np.rint(gamma / S_out * (2.0 ** (s - 10)))
        bq = np.rint(beta / S_out * (2.0 ** s))
        if np.max(np.abs(gq)) < 2 ** 14 and np.max(np.abs(bq)) < 2 ** 29:
            return gq.astype(np.int32), bq.astype(np.int32), s
    raise ValueError("no LayerNorm shift satisfies the range preconditions")


def embedding_params(emb: dict, S_out: float):
    """Integer constants of the INT8 embedding: the two table scales are brought to the LayerNorm input scale S_r,
    tok_dy = dyadic(S_tok / S_r), pos_dy = dyadic(S_pos / S_r); LayerNorm constants as in layernorm_params.
    Returns (tok_dy, pos_dy, gamma_q, beta_q, shift)."""
    gq, bq, s = layernorm_params(emb["gamma"], emb["beta"], S_out)
    return dyadic_from_double(emb["S_tok"] / emb["S_r"]), dyadic_from_double(emb["S_pos"] / emb["S_r"]), gq, bq, s


def layer_params(raw: dict, sc: dict, hidden: int, heads: int):
    """Integer parameters of one encoder layer from raw synthetic weights and static scales.

    raw: w_qkv,sw_qkv,b_qkv, w_o,sw_o,b_o, gamma1,beta1, w_1,sw_1,b_1, w_2,sw_2,b_2, gamma2,beta2
    sc:  S_x,S_q,S_k,S_v,S_s,softmax_k,S_ctx,S_r1,S_h1,S_g_in,S_g_out,S_r2,S_y
    Returns (weights dict for oracle.encoder_layer, LayerQuantT).
    """
    H = hidden
    d = H // heads
    w = {}
    w["w_qkv"], w["b_qkv"] = raw["w_qkv"], raw["b_qkv"]
    mq, sq = channel_dyadics(sc["S_x"], raw["sw_qkv"][:H], sc["S_q"])
    mk, sk = channel_dyadics(sc["S_x"], raw["sw_qkv"][H:2 * H], sc["S_k"])
    mv, sv = channel_dyadics(sc["S_x"], raw["sw_qkv"][2 * H:], sc["S_v"])
    w["m_qkv"], w["s_qkv"] = np.concatenate([mq, mk, mv]), np.concatenate([sq, sk, sv])
    w["w_o"], w["b_o"] = raw["w_o"], raw["b_o"]
    w["m_o"], w["s_o"] = channel_dyadics(sc["S_ctx"], raw["sw_o"], sc["S_r1"])
    w["ln1_gamma_q"], w["ln1_beta_q"], ln1_shift = layernorm_params(raw["gamma1"], raw["beta1"], sc["S_h1"])
    w["w_1"], w["b_1"] = raw["w_1"], raw["b_1"]
    w["m_1"], w["s_1"] = channel_dyadics(sc["S_h1"], raw["sw_1"], sc["S_g_in"])
    w["w_2"], w["b_2"] = raw["w_2"], raw["b_2"]
    w["m_2"], w["s_2"] = channel_dyadics(sc["S_g_out"], raw["sw_2"], sc["S_r2"])
    w["ln2_gamma_q"], w["ln2_beta_q"], ln2_shift = layernorm_params(raw["gamma2"], raw["beta2"], sc["S_y"])

    q = LayerQuantT()
    k = int(sc["softmax_k"])
    q.scores_m, q.scores_s = dyadic_from_double(sc["S_q"] * sc["S_k"] / (math.sqrt(float(d)) * sc["S_s"]))
    q.softmax = softmax_params(sc["S_s"], k, I8)
    q.ctx_m, q.ctx_s = dyadic_from_double((2.0 ** -k) * sc["S_v"] / sc["S_ctx"])
    q.res1_m, q.res1_s = dyadic_from_double(sc["S_x"] / sc["S_r1"])
    q.ln1_shift = ln1_shift
    q.gelu = gelu_params(sc["S_g_in"], sc["S_g_out"])
    q.res2_m, q.res2_s = dyadic_from_double(sc["S_h1"] / sc["S_r2"])
    q.ln2_shift = ln2_shift
    return w, q
