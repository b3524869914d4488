"""Seeded synthetic inputs for the integer-only encoder layer.

This module serves both the HIP library's tests/benchmark and the CPU oracle.  It holds no
part of the method's arithmetic: it only draws random tensors and fixes the *real-valued*
static scales of every activation tensor.  Turning scales into integer constants is done
separately by each side with its own code.

Everything is reproducible from (config, seed, layer index): each tensor family has its own
numpy ``Generator(PCG64([seed, layer, tag]))`` so a layer can be generated without generating
the ones before it.

Distributions
  weights        int8 uniform integers in [-127, 127]
  weight scales  per output channel, exp(N(ln 0.01, 0.3))
  biases         int32 uniform integers in [-2^15, 2^15], at the accumulator scale S_in * S_w[n]
  LayerNorm      gamma ~ N(1, 0.1), beta ~ N(0, 0.1)          (second parameter = standard deviation)
  input          float32 N(0, 1) [T, H], symmetric int8 with S_x = max|x| / 127, round half to even
Static scales of the intermediate activations are closed-form predictions from these
distributions (static quantization fixes ranges ahead of inference from expected statistics,
App. A); they do not look at the data.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np

SEED = 20210101


@dataclass(frozen=True)
class EncoderConfig:
    name: str
    hidden: int
    heads: int
    ffn: int
    seq: int
    batch: int
    layers: int

    @property
    def tokens(self) -> int:
        return self.batch * self.seq

    def with_batch(self, batch: int) -> "EncoderConfig":
        return EncoderConfig(self.name, self.hidden, self.heads, self.ffn, self.seq, batch, self.layers)


CONFIGS = {
    "tiny": EncoderConfig("tiny", 256, 4, 1024, 128, 1, 1),
    "base_b1": EncoderConfig("base_b1", 768, 12, 3072, 128, 1, 12),
    "base_b32": EncoderConfig("base_b32", 768, 12, 3072, 128, 32, 12),
    "large_b32": EncoderConfig("large_b32", 1024, 16, 4096, 128, 32, 24),
    "large_b256": EncoderConfig("large_b256", 1024, 16, 4096, 128, 256, 24),
    "base512_b64": EncoderConfig("base512_b64", 768, 12, 3072, 512, 64, 12),
}

_TAGS = {"qkv": 1, "o": 2, "ln1": 3, "ffn1": 4, "ffn2": 5, "ln2": 6, "x": 7,
         "softmax": 8, "gelu": 9, "layernorm": 10, "gemm": 11}


def _rng(seed: int, layer: int, tag: str) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64([seed, layer, _TAGS[tag]]))


def _linear(rng: np.random.Generator, n_out: int, n_in: int):
    w = rng.integers(-127, 128, size=(n_out, n_in), dtype=np.int8)
    sw = np.exp(rng.normal(math.log(0.01), 0.3, size=n_out))
    b = rng.integers(-(1 << 15), (1 << 15) + 1, size=n_out, dtype=np.int32)
    return w, sw.astype(np.float64), b


def layer_raw(cfg: EncoderConfig, layer: int, seed: int = SEED) -> dict:
    """Raw (un-derived) parameters of encoder layer ``layer``."""
    H, F = cfg.hidden, cfg.ffn
    raw = {}
    raw["w_qkv"], raw["sw_qkv"], raw["b_qkv"] = _linear(_rng(seed, layer, "qkv"), 3 * H, H)
    raw["w_o"], raw["sw_o"], raw["b_o"] = _linear(_rng(seed, layer, "o"), H, H)
    r = _rng(seed, layer, "ln1")
    raw["gamma1"], raw["beta1"] = r.normal(1.0, 0.1, size=H), r.normal(0.0, 0.1, size=H)
    raw["w_1"], raw["sw_1"], raw["b_1"] = _linear(_rng(seed, layer, "ffn1"), F, H)
    raw["w_2"], raw["sw_2"], raw["b_2"] = _linear(_rng(seed, layer, "ffn2"), H, F)
    r = _rng(seed, layer, "ln2")
    raw["gamma2"], raw["beta2"] = r.normal(1.0, 0.1, size=H), r.normal(0.0, 0.1, size=H)
    return raw


def input_activations(cfg: EncoderConfig, seed: int = SEED):
    """Returns (x_q int8 [T,H], S_x, x float32 [T,H])."""
    x = _rng(seed, 0, "x").standard_normal(size=(cfg.tokens, cfg.hidden), dtype=np.float32)
    S_x = float(np.max(np.abs(x)).astype(np.float64)) / 127.0
    x_q = np.clip(np.rint(x.astype(np.float64) / S_x), -127, 127).astype(np.int8)
    return x_q, S_x, x


# --- closed-form statistics of the synthetic model ------------------------------------------
_W2 = 127.0 * 128.0 / 3.0                 # E[w^2], w uniform integer in [-127, 127]
_SW2 = math.exp(2.0 * math.log(0.01) + 2.0 * 0.3 ** 2)   # E[S_w^2], lognormal
SIGMA_W = math.sqrt(_W2 * _SW2)          # std of a real-valued weight, ~0.805
_B_RMS = math.sqrt(_SW2) * (2.0 ** 15) / math.sqrt(3.0)   # rms of S_w[n]*bias[n] (times S_in = real bias)
LN_OUT_ALPHA = 5.0                        # clip range of a LayerNorm output (gamma*N(0,1)+beta)
CLIP_SIGMAS = 4.0                         # int8 activations clip at 4 predicted standard deviations


def _pow2_at_least(v: float) -> float:
    return 2.0 ** math.ceil(math.log2(v))


def static_scales(cfg: EncoderConfig, S_x: float) -> dict:
    """Real-valued static scale of every activation tensor of one layer whose input has scale S_x.

    Layer input is assumed to have unit variance (true for the N(0,1) input and for LayerNorm outputs
    with gamma ~ 1).  INT8 tensors use alpha/127 with alpha = 4 predicted sigmas; the three INT32
    non-linearity inputs use power-of-two scales.
    """
    H, F = cfg.hidden, cfg.ffn
    S_h1 = LN_OUT_ALPHA / 127.0
    sig_qkv = math.hypot(SIGMA_W * math.sqrt(H), S_x * _B_RMS)         # std of a Q/K/V element
    S_qkv = CLIP_SIGMAS * sig_qkv / 127.0
    sig_attn = math.hypot(sig_qkv * SIGMA_W * math.sqrt(H), S_qkv * _B_RMS)   # context ~ one V row
    sig_f1 = math.hypot(SIGMA_W * math.sqrt(H), S_h1 * _B_RMS)         # FFN1 output
    S_g_out = CLIP_SIGMAS * sig_f1 / 127.0
    sig_g = sig_f1 * math.sqrt(0.5)                                    # rms of GELU(N(0, sig^2))
    sig_f2 = math.hypot(sig_g * SIGMA_W * math.sqrt(F), S_g_out * _B_RMS)
    sc = {"S_x": float(S_x)}
    sc["S_q"] = sc["S_k"] = sc["S_v"] = S_qkv
    sc["S_s"] = 2.0 ** -6
    sc["softmax_k"] = 7
    sc["S_ctx"] = sc["S_v"]
    sc["S_r1"] = _pow2_at_least(8.0 * sig_attn / 32767.0)
    sc["S_h1"] = S_h1
    sc["S_g_in"] = 2.0 ** -6
    sc["S_g_out"] = S_g_out
    sc["S_r2"] = _pow2_at_least(8.0 * sig_f2 / 32767.0)
    sc["S_y"] = LN_OUT_ALPHA / 127.0
    return sc


def model_scales(cfg: EncoderConfig, S_x: float) -> list:
    """Static scales of all layers: layer l+1 takes layer l's output scale as S_x."""
    out = []
    s = S_x
    for _ in range(cfg.layers):
        sc = static_scales(cfg, s)
        out.append(sc)
        s = sc["S_y"]
    return out


# --- standalone non-linearity inputs at RoBERTa-Base activation shapes ----------------------
def softmax_logits(rows: int, cols: int, seed: int = SEED, std: float = 4.0, scale: float = 2.0 ** -6):
    """int32 logits = rint(N(0, std) / scale); returns (q, scale)."""
    x = _rng(seed, 0, "softmax").normal(0.0, std, size=(rows, cols))
    return np.rint(x / scale).astype(np.int32), scale


def gelu_inputs(rows: int, cols: int, seed: int = SEED, std: float = 2.0, scale: float = 2.0 ** -7):
    x = _rng(seed, 0, "gelu").normal(0.0, std, size=(rows, cols))
    return np.rint(x / scale).astype(np.int32), scale


def layernorm_inputs(rows: int, cols: int, seed: int = SEED, std: float = 3.0, scale: float = 2.0 ** -8):
    """Returns (q int32, scale, gamma float64 [cols], beta float64 [cols])."""
    r = _rng(seed, 0, "layernorm")
    x = r.normal(0.0, std, size=(rows, cols))
    gamma = r.normal(1.0, 0.1, size=cols)
    beta = r.normal(0.0, 0.1, size=cols)
    return np.rint(x / scale).astype(np.int32), scale, gamma, beta


def gemm_operands(M: int, N: int, K: int, seed: int = SEED, layer: int = 0):
    """int8 A [M,K], W [N,K], per-channel scales, int32 bias, for standalone GEMM cases."""
    r = _rng(seed, layer, "gemm")
    A = r.integers(-127, 128, size=(M, K), dtype=np.int8)
    W, sw, b = _linear(r, N, K)
    return A, W, sw, b


def embedding_raw(hidden: int, vocab: int, max_pos: int, seed: int = SEED):
    """Synthetic embedding tables (stand-ins for trained ones): token table N(0, 0.05), position table N(0, 0.02),
    each symmetric INT8 with its own scale max|.|/127; LayerNorm gamma ~ N(1, 0.1), beta ~ N(0, 0.1); the INT32 sum is
    held at the power-of-two scale S_r = 2^-12 (|sum| stays far below 2^15 - 1 for these tables).
    Returns dict(tok, S_tok, pos, S_pos, gamma, beta, S_r)."""
    rng = np.random.default_rng(seed + 7919)
    tok_f = rng.normal(0.0, 0.05, size=(vocab, hidden))
    pos_f = rng.normal(0.0, 0.02, size=(max_pos, hidden))
    S_tok, S_pos = float(np.max(np.abs(tok_f)) / 127), float(np.max(np.abs(pos_f)) / 127)
    tok = np.clip(np.rint(tok_f / S_tok), -127, 127).astype(np.int8)
    pos = np.clip(np.rint(pos_f / S_pos), -127, 127).astype(np.int8)
    gamma = rng.normal(1.0, 0.1, size=hidden)
    beta = rng.normal(0.0, 0.1, size=hidden)
    return dict(tok=tok, S_tok=S_tok, pos=pos, S_pos=S_pos, gamma=gamma, beta=beta, S_r=2.0 ** -12)


def token_ids(tokens: int, vocab: int, seed: int = SEED) -> np.ndarray:
    """Token ids with a Zipf-like skew (frequent ids repeat, as in text), int32 [tokens]."""
    rng = np.random.default_rng(seed + 104729)
    z = rng.zipf(1.3, size=tokens)
    return ((z - 1) % vocab).astype(np.int32)


def key_lengths(batch: int, seq: int, seed: int = SEED) -> np.ndarray:
    """Valid lengths of a padded batch: uniform in [seq/4, seq], the longest sequence full; int32 [batch]."""
    rng = np.random.default_rng(seed + 15485863)
    lens = rng.integers(max(1, seq // 4), seq + 1, size=batch).astype(np.int32)
    lens[0] = seq
    return lens
