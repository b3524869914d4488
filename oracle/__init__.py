"""CPU oracle for the integer-only encoder layer (test infrastructure, not the product).

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It wraps ``ibert_oracle.c`` (plain C,
exact integers) with ctypes and holds the oracle's own derivation of the
integer constants from real scales (``oracle.params``).  It imports nothing from
the HIP package and the HIP package imports nothing from here.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ibert_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

I8, I32 = 0, 1
OK, E_ARG, E_PARAM, E_RANGE, E_NOMEM = 0, -1, -2, -3, -4


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (cheap; done on demand)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


class GemmT(C.Structure):
    _fields_ = [("M", C.c_int32), ("N", C.c_int32), ("K", C.c_int32),
                ("batch_outer", C.c_int32), ("batch_inner", C.c_int32),
                ("lda", C.c_int64), ("ldw", C.c_int64), ("ldc", C.c_int64), ("ldr", C.c_int64),
                ("sA_o", C.c_int64), ("sA_i", C.c_int64), ("sW_o", C.c_int64), ("sW_i", C.c_int64),
                ("sC_o", C.c_int64), ("sC_i", C.c_int64), ("sR_o", C.c_int64), ("sR_i", C.c_int64),
                ("trans_w", C.c_int32), ("per_channel", C.c_int32),
                ("dy_m", C.c_int32), ("dy_s", C.c_int32),
                ("out_dtype", C.c_int32), ("out_clamp", C.c_int32),
                ("res_m", C.c_int32), ("res_s", C.c_int32)]


class SoftmaxT(C.Structure):
    _fields_ = [("q_ln2", C.c_int32), ("q_b", C.c_int32), ("q_c", C.c_int32),
                ("out_frac_bits", C.c_int32), ("out_dtype", C.c_int32)]


class GeluT(C.Structure):
    _fields_ = [("q_b", C.c_int32), ("q_c", C.c_int32), ("q_1", C.c_int32), ("q_max", C.c_int32),
                ("out_m", C.c_int32), ("out_s", C.c_int32)]


class HGeluT(C.Structure):
    _fields_ = [("slope_m", C.c_int32), ("slope_s", C.c_int32), ("q_3", C.c_int32), ("q_6", C.c_int32),
                ("q_max", C.c_int32), ("out_m", C.c_int32), ("out_s", C.c_int32)]


_P = C.c_void_p


class LayerWeightsT(C.Structure):
    _fields_ = [(n, _P) for n in (
        "w_qkv", "b_qkv", "m_qkv", "s_qkv", "w_o", "b_o", "m_o", "s_o", "ln1_gamma_q", "ln1_beta_q",
        "w_1", "b_1", "m_1", "s_1", "w_2", "b_2", "m_2", "s_2", "ln2_gamma_q", "ln2_beta_q")]


class LayerQuantT(C.Structure):
    _fields_ = [("scores_m", C.c_int32), ("scores_s", C.c_int32), ("softmax", SoftmaxT),
                ("ctx_m", C.c_int32), ("ctx_s", C.c_int32),
                ("res1_m", C.c_int32), ("res1_s", C.c_int32), ("ln1_shift", C.c_int32),
                ("gelu", GeluT),
                ("res2_m", C.c_int32), ("res2_s", C.c_int32), ("ln2_shift", C.c_int32)]


class LayerDumpT(C.Structure):
    _fields_ = [(n, _P) for n in ("qkv", "scores", "probs", "ctx", "r1", "h1", "f1", "g", "r2")]


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        L.orc_dyadic.restype = C.c_int64
        L.orc_dyadic.argtypes = [C.c_int64, C.c_int32, C.c_int32]
        L.orc_ipoly.restype = C.c_int64
        L.orc_ipoly.argtypes = [C.c_int64] * 3
        L.orc_iexp.restype = C.c_int64
        L.orc_iexp.argtypes = [C.c_int64] * 4 + [C.POINTER(C.c_int64)]
        L.orc_ierf.restype = C.c_int64
        L.orc_ierf.argtypes = [C.c_int64] * 3
        L.orc_igelu_t.restype = C.c_int64
        L.orc_igelu_t.argtypes = [C.c_int64, C.POINTER(GeluT)]
        L.orc_isqrt.restype = C.c_uint64
        L.orc_isqrt.argtypes = [C.c_uint64, C.POINTER(C.c_int)]
        L.orc_isqrt_array.restype = None
        L.orc_isqrt_array.argtypes = [_P, _P, _P, C.c_int64]
        L.orc_gemm_requant.restype = C.c_int
        L.orc_gemm_requant.argtypes = [C.POINTER(GemmT)] + [_P] * 7
        L.orc_softmax_check.restype = C.c_int
        L.orc_softmax_check.argtypes = [C.POINTER(SoftmaxT), C.c_int]
        L.orc_softmax.restype = C.c_int
        L.orc_softmax.argtypes = [_P, _P, C.c_int64, C.c_int, C.c_int64, C.c_int64, C.POINTER(SoftmaxT)]
        L.orc_gelu_check.restype = C.c_int
        L.orc_gelu_check.argtypes = [C.POINTER(GeluT)]
        L.orc_gelu.restype = C.c_int
        L.orc_gelu.argtypes = [_P, _P, C.c_int64, C.POINTER(GeluT)]
        L.orc_hgelu_t.restype = C.c_int64
        L.orc_hgelu_t.argtypes = [C.c_int64, C.POINTER(HGeluT)]
        L.orc_hgelu_check.restype = C.c_int
        L.orc_hgelu_check.argtypes = [C.POINTER(HGeluT)]
        L.orc_hgelu.restype = C.c_int
        L.orc_hgelu.argtypes = [_P, _P, C.c_int64, C.POINTER(HGeluT)]
        L.orc_layernorm_check.restype = C.c_int
        L.orc_layernorm_check.argtypes = [C.c_int, _P, _P, C.c_int]
        L.orc_layernorm.restype = C.c_int
        L.orc_layernorm.argtypes = [_P, _P, C.c_int64, C.c_int, C.c_int64, C.c_int64, _P, _P, C.c_int]
        L.orc_encoder_layer.restype = C.c_int
        L.orc_encoder_layer.argtypes = [C.POINTER(LayerWeightsT), C.POINTER(LayerQuantT), _P, _P,
                                        C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.POINTER(LayerDumpT)]
        L.orc_encoder_layer_masked.restype = C.c_int
        L.orc_encoder_layer_masked.argtypes = [C.POINTER(LayerWeightsT), C.POINTER(LayerQuantT), _P, _P,
                                               C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, _P, C.POINTER(LayerDumpT)]
        L.orc_mask_scores.restype = C.c_int
        L.orc_mask_scores.argtypes = [_P, C.c_int, C.c_int, C.c_int, _P]
        L.orc_embedding.restype = C.c_int
        L.orc_embedding.argtypes = [_P, C.c_int64, C.c_int, C.c_int, C.c_int, C.c_int, _P, _P, C.c_int32, C.c_int32,
                                    C.c_int32, C.c_int32, _P, _P, C.c_int, _P, _P]
        L.orc_num_threads.restype = C.c_int
        _lib = L
    return _lib


class OracleError(RuntimeError):
    def __init__(self, code: int, where: str):
        names = {E_ARG: "E_ARG", E_PARAM: "E_PARAM", E_RANGE: "E_RANGE", E_NOMEM: "E_NOMEM"}
        super().__init__("%s: oracle returned %s" % (where, names.get(code, code)))
        self.code = code


def _chk(rc: int, where: str):
    if rc != OK:
        raise OracleError(rc, where)


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data


def _arr(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


# ----------------------------------------------------------------------------- scalars
def dyadic(x: int, m: int, s: int) -> int:
    return int(lib().orc_dyadic(int(x), int(m), int(s)))


def ipoly(q: int, q_b: int, q_c: int) -> int:
    return int(lib().orc_ipoly(int(q), int(q_b), int(q_c)))


def iexp(q: int, q_ln2: int, q_b: int, q_c: int):
    """Returns (q_exp, z)."""
    z = C.c_int64(0)
    v = lib().orc_iexp(int(q), int(q_ln2), int(q_b), int(q_c), C.byref(z))
    return int(v), int(z.value)


def ierf(q: int, q_b: int, q_c: int) -> int:
    return int(lib().orc_ierf(int(q), int(q_b), int(q_c)))


def igelu_t(q: int, gp: "GeluT") -> int:
    return int(lib().orc_igelu_t(int(q), C.byref(gp)))


def isqrt(n: int):
    """Returns (floor(sqrt(n)), loop passes)."""
    it = C.c_int(0)
    v = lib().orc_isqrt(int(n), C.byref(it))
    return int(v), int(it.value)


def isqrt_array(n: np.ndarray):
    n = _arr(n, np.uint64)
    out = np.empty_like(n)
    iters = np.empty(n.shape, dtype=np.int32)
    lib().orc_isqrt_array(n.ctypes.data, out.ctypes.data, iters.ctypes.data, n.size)
    return out, iters


# ----------------------------------------------------------------------------- tensors
@dataclass
class GemmSpec:
    """Mirror of orc_gemm_t with defaults for a plain 2-D problem."""
    M: int
    N: int
    K: int
    lda: int = 0
    ldw: int = 0
    ldc: int = 0
    ldr: int = 0
    batch_outer: int = 1
    batch_inner: int = 1
    sA: tuple = (0, 0)
    sW: tuple = (0, 0)
    sC: tuple = (0, 0)
    sR: tuple = (0, 0)
    trans_w: int = 0
    per_channel: int = 1
    dy: tuple = (1, 0)
    out_dtype: int = I8
    out_clamp: int = 127
    res_dy: tuple = (0, 0)

    def to_c(self) -> GemmT:
        g = GemmT()
        g.M, g.N, g.K = self.M, self.N, self.K
        g.batch_outer, g.batch_inner = self.batch_outer, self.batch_inner
        g.lda = self.lda or self.K
        g.ldw = self.ldw or (self.N if self.trans_w else self.K)
        g.ldc = self.ldc or self.N
        g.ldr = self.ldr or self.N
        g.sA_o, g.sA_i = self.sA
        g.sW_o, g.sW_i = self.sW
        g.sC_o, g.sC_i = self.sC
        g.sR_o, g.sR_i = self.sR
        g.trans_w, g.per_channel = self.trans_w, self.per_channel
        g.dy_m, g.dy_s = self.dy
        g.out_dtype, g.out_clamp = self.out_dtype, self.out_clamp
        g.res_m, g.res_s = self.res_dy
        return g


def gemm_requant(spec: GemmSpec, A, W, bias=None, mult=None, shift=None, residual=None,
                 out: Optional[np.ndarray] = None, out_elems: Optional[int] = None) -> np.ndarray:
    """Raw strided call: A, W, residual and out are flat buffers addressed by the spec's strides."""
    A = _arr(A, np.int8)
    W = _arr(W, np.int8)
    bias = None if bias is None else _arr(bias, np.int32)
    mult = None if mult is None else _arr(mult, np.int32)
    shift = None if shift is None else _arr(shift, np.int32)
    residual = None if residual is None else _arr(residual, np.int8)
    g = spec.to_c()
    if out is None:
        if out_elems is None:
            nb = spec.batch_outer * spec.batch_inner
            assert nb == 1 or (spec.sC != (0, 0)), "give out or out_elems for batched problems"
            out_elems = (max(spec.M - 1, 0) * g.ldc + spec.N
                         + (spec.batch_outer - 1) * g.sC_o + (spec.batch_inner - 1) * g.sC_i)
        out = np.zeros(out_elems, dtype=np.int8 if spec.out_dtype == I8 else np.int32)
    rc = lib().orc_gemm_requant(C.byref(g), _ptr(A), _ptr(W), _ptr(bias), _ptr(mult), _ptr(shift),
                                _ptr(residual), _ptr(out))
    _chk(rc, "gemm_requant")
    return out


def softmax(x: np.ndarray, sp: SoftmaxT, cols: Optional[int] = None) -> np.ndarray:
    x = _arr(x, np.int32)
    cols = x.shape[-1] if cols is None else cols
    rows = x.size // x.shape[-1] if x.size else 0
    ld = x.shape[-1]
    y = np.zeros(x.shape, dtype=np.int8 if sp.out_dtype == I8 else np.int32)
    rc = lib().orc_softmax(_ptr(x), _ptr(y), rows, cols, ld, ld, C.byref(sp))
    _chk(rc, "softmax")
    return y


def gelu(x: np.ndarray, gp: GeluT) -> np.ndarray:
    x = _arr(x, np.int32)
    y = np.zeros(x.shape, dtype=np.int8)
    _chk(lib().orc_gelu(_ptr(x), _ptr(y), x.size, C.byref(gp)), "gelu")
    return y


def hgelu_t(q: int, hp: HGeluT) -> int:
    return int(lib().orc_hgelu_t(int(q), C.byref(hp)))


def hgelu(x: np.ndarray, hp: HGeluT) -> np.ndarray:
    """h-GELU (Eq. 6) in integers, requantized to INT8."""
    x = _arr(x, np.int32)
    y = np.zeros(x.shape, dtype=np.int8)
    _chk(lib().orc_hgelu(_ptr(x), _ptr(y), x.size, C.byref(hp)), "hgelu")
    return y


def layernorm(x: np.ndarray, gamma_q, beta_q, shift: int) -> np.ndarray:
    x = _arr(x, np.int32)
    Cc = x.shape[-1]
    rows = x.size // Cc if x.size else 0
    gamma_q = _arr(gamma_q, np.int32)
    beta_q = _arr(beta_q, np.int32)
    y = np.zeros(x.shape, dtype=np.int8)
    rc = lib().orc_layernorm(_ptr(x), _ptr(y), rows, Cc, Cc, Cc, _ptr(gamma_q), _ptr(beta_q), int(shift))
    _chk(rc, "layernorm")
    return y


_W_FIELDS = [n for n, _ in LayerWeightsT._fields_]
_D_FIELDS = [n for n, _ in LayerDumpT._fields_]
_W_DTYPES = {"w_qkv": np.int8, "w_o": np.int8, "w_1": np.int8, "w_2": np.int8}


def encoder_layer(weights: dict, quant: LayerQuantT, x: np.ndarray, batch: int, seq: int, hidden: int,
                  heads: int, ffn: int, dump: bool = False, key_lens=None):
    """weights: dict field -> numpy array (see LayerWeightsT).  Returns y, or (y, dict of intermediates).
    key_lens: optional int32 [batch], keys at or past it are padding (orc_mask_scores)."""
    keep = {}
    w = LayerWeightsT()
    for f in _W_FIELDS:
        a = _arr(weights[f], _W_DTYPES.get(f, np.int32))
        keep[f] = a
        setattr(w, f, a.ctypes.data)
    x = _arr(x, np.int8)
    T, H, F, nh, L = batch * seq, hidden, ffn, heads, seq
    assert x.size == T * H
    y = np.zeros((T, H), dtype=np.int8)
    d = LayerDumpT()
    inter = {}
    if dump:
        shapes = {"qkv": ((T, 3 * H), np.int8), "scores": ((batch * nh, L, L), np.int32),
                  "probs": ((batch * nh, L, L), np.int8), "ctx": ((T, H), np.int8),
                  "r1": ((T, H), np.int32), "h1": ((T, H), np.int8), "f1": ((T, F), np.int32),
                  "g": ((T, F), np.int8), "r2": ((T, H), np.int32)}
        for f in _D_FIELDS:
            inter[f] = np.zeros(shapes[f][0], dtype=shapes[f][1])
            setattr(d, f, inter[f].ctypes.data)
    kl = None if key_lens is None else _arr(key_lens, np.int32)
    assert kl is None or kl.size == batch
    rc = lib().orc_encoder_layer_masked(C.byref(w), C.byref(quant), _ptr(x), _ptr(y), batch, seq, hidden, heads, ffn,
                                        None if kl is None else _ptr(kl), C.byref(d) if dump else None)
    _chk(rc, "encoder_layer")
    return (y, inter) if dump else y


def mask_scores(scores: np.ndarray, batch: int, heads: int, seq: int, key_lens) -> np.ndarray:
    """Copy of scores [batch*heads, seq, seq] with the padded keys set to the masked logit."""
    out = _arr(scores, np.int32).copy()
    kl = _arr(key_lens, np.int32)
    _chk(lib().orc_mask_scores(_ptr(out), batch, heads, seq, _ptr(kl)), "mask_scores")
    return out


def embedding(ids, seq: int, tok, pos, tok_dy, pos_dy, gamma_q, beta_q, ln_shift: int, return_sum: bool = False):
    """INT8 embedding + integer LayerNorm.  ids int32 [T]; tok int8 [V,H]; pos int8 [P,H]; *_dy = (m, s)."""
    ids = _arr(ids, np.int32)
    tok, pos = _arr(tok, np.int8), _arr(pos, np.int8)
    gq, bq = _arr(gamma_q, np.int32), _arr(beta_q, np.int32)
    T, H = ids.size, tok.shape[1]
    y = np.zeros((T, H), dtype=np.int8)
    r = np.zeros((T, H), dtype=np.int32)
    rc = lib().orc_embedding(_ptr(ids), T, seq, H, tok.shape[0], pos.shape[0], _ptr(tok), _ptr(pos), tok_dy[0], tok_dy[1],
                             pos_dy[0], pos_dy[1], _ptr(gq), _ptr(bq), ln_shift, _ptr(r), _ptr(y))
    _chk(rc, "embedding")
    return (y, r) if return_sum else y


def num_threads() -> int:
    return int(lib().orc_num_threads())
