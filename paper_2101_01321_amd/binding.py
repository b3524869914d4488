"""ctypes binding of libibert: argument marshalling only, same names as the C entry points.

Tensors are torch CUDA tensors (device memory and streams are PyTorch's; every computation runs in
the library's HIP kernels).  Loading fails loudly when the shared library has not been built: there
is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libibert.so")

I8, I32, I16 = 0, 1, 2
OK = 0
_P = C.c_void_p


class IbertError(RuntimeError):
    def __init__(self, code: int, where: str):
        L = lib()
        msg = L.ibert_status_string(code).decode()
        if code == -6:
            msg += " (" + L.ibert_last_hip_error().decode() + ")"
        super().__init__("%s: %s [%d]" % (where, msg, code))
        self.code = code


class Dyadic(C.Structure):
    _fields_ = [("m", C.c_int32), ("s", C.c_int32)]

    def tuple(self):
        return (self.m, self.s)


class GemmDesc(C.Structure):
    _fields_ = [("M", C.c_int32), ("N", C.c_int32), ("K", C.c_int32),
                ("batch_outer", C.c_int32), ("batch_inner", C.c_int32),
                ("lda", C.c_int64), ("ldw", C.c_int64), ("ldc", C.c_int64), ("ldr", C.c_int64),
                ("strideA_outer", C.c_int64), ("strideA_inner", C.c_int64),
                ("strideW_outer", C.c_int64), ("strideW_inner", C.c_int64),
                ("strideC_outer", C.c_int64), ("strideC_inner", C.c_int64),
                ("strideR_outer", C.c_int64), ("strideR_inner", C.c_int64),
                ("trans_w", C.c_int32), ("per_channel", C.c_int32), ("requant", Dyadic),
                ("out_dtype", C.c_int32), ("out_clamp", C.c_int32), ("residual_dy", Dyadic)]


class SoftmaxParams(C.Structure):
    _fields_ = [("q_ln2", C.c_int32), ("q_b", C.c_int32), ("q_c", C.c_int32),
                ("out_frac_bits", C.c_int32), ("out_dtype", C.c_int32)]


class GeluParams(C.Structure):
    _fields_ = [("q_b", C.c_int32), ("q_c", C.c_int32), ("q_1", C.c_int32), ("q_max", C.c_int32),
                ("out", Dyadic)]


class HGeluParams(C.Structure):
    _fields_ = [("slope", Dyadic), ("q_3", C.c_int32), ("q_6", C.c_int32), ("q_max", C.c_int32), ("out", Dyadic)]


class LayerWeights(C.Structure):
    _fields_ = [(n, _P) for n in (
        "w_qkv", "b_qkv", "m_qkv", "s_qkv", "w_o", "b_o", "m_o", "s_o", "ln1_gamma_q", "ln1_beta_q",
        "w_1", "b_1", "m_1", "s_1", "w_2", "b_2", "m_2", "s_2", "ln2_gamma_q", "ln2_beta_q")]


class LayerQuant(C.Structure):
    _fields_ = [("scores_dy", Dyadic), ("softmax", SoftmaxParams), ("ctx_dy", Dyadic), ("res1_dy", Dyadic),
                ("ln1_shift", C.c_int32), ("gelu", GeluParams), ("res2_dy", Dyadic), ("ln2_shift", C.c_int32),
                ("route", C.c_int32)]


# ibert_layer_quant.route flags
ROUTE_SEPARATE_GELU, ROUTE_SEPARATE_ATTENTION, ROUTE_I32_LN_INPUT = 1, 2, 4


class WorkspaceLayout(C.Structure):
    _fields_ = [(n, C.c_size_t) for n in ("qkv", "scores", "probs", "ctx", "r1", "h1", "f1", "g", "r2", "total")]


class LayerScales(C.Structure):
    _fields_ = [(n, C.c_double) for n in ("S_x", "S_q", "S_k", "S_v", "S_s", "S_ctx", "S_r1", "S_h1",
                                          "S_g_in", "S_g_out", "S_r2", "S_y")] + [("softmax_k", C.c_int32)]


class ProfileRecord(C.Structure):
    _fields_ = [("step", C.c_int32), ("ms", C.c_float), ("ops", C.c_double), ("bytes", C.c_double),
                ("kernel", C.c_char * 96)]


# Every symbol include/ibert.h and include/ibert_testing.h declare, with its ctypes signature.
SIGNATURES = {
    "ibert_gemm_i8_requant": (C.c_int, [C.POINTER(GemmDesc)] + [_P] * 8),
    "ibert_gemm_config_override": (C.c_int, [C.c_int32]),
    "ibert_gemm_epilogue_record": (None, [_P]),
    "ibert_gemm_xcd_blocks": (None, [C.c_int32]),
    "ibert_gemm_i8_gelu": (C.c_int, [C.POINTER(GemmDesc)] + [_P] * 5 + [C.POINTER(GeluParams)] + [_P] * 3),
    "ibert_isqrt_i": (C.c_int, [_P, _P, C.c_int64, C.c_int32, _P]),
    "ibert_attention_scratch_bytes": (C.c_size_t, [C.c_int32] * 3),
    "ibert_attention_i": (C.c_int, [_P, _P] + [C.c_int32] * 4 + [C.POINTER(Dyadic), C.POINTER(SoftmaxParams),
                                                                 C.POINTER(Dyadic), _P, C.c_size_t, _P]),
    "ibert_attention_masked_i": (C.c_int, [_P, _P] + [C.c_int32] * 4 + [C.POINTER(Dyadic), C.POINTER(SoftmaxParams),
                                                                        C.POINTER(Dyadic), _P, _P, C.c_size_t, _P]),
    "ibert_softmax_masked_i": (C.c_int, [_P, _P, C.c_int64, C.c_int32, C.c_int64, C.c_int64, C.POINTER(SoftmaxParams), _P,
                                         C.c_int64, _P]),
    "ibert_embedding_i": (C.c_int, [_P, _P, _P, C.c_int64] + [C.c_int32] * 4 + [C.POINTER(Dyadic), C.POINTER(Dyadic), _P, _P,
                                                                                 C.c_int32, _P, C.c_int64, _P]),
    "ibert_encoder_layer_masked_i": (C.c_int, [C.POINTER(LayerWeights), C.POINTER(LayerQuant), _P, _P] + [C.c_int32] * 5 +
                                     [_P, _P, C.c_size_t, _P]),
    "ibert_encoder_masked_i": (C.c_int, [C.POINTER(LayerWeights), C.POINTER(LayerQuant), C.c_int32, _P, _P] +
                               [C.c_int32] * 5 + [_P, _P, C.c_size_t, _P]),
    "ibert_softmax_i": (C.c_int, [_P, _P, C.c_int64, C.c_int32, C.c_int64, C.c_int64, C.POINTER(SoftmaxParams), _P]),
    "ibert_gelu_i": (C.c_int, [_P, _P, C.c_int64, C.POINTER(GeluParams), _P]),
    "ibert_hgelu_i": (C.c_int, [_P, _P, C.c_int64, C.POINTER(HGeluParams), _P]),
    "ibert_hgelu_params_from_scale": (C.c_int, [C.c_double, C.c_double, C.POINTER(HGeluParams)]),
    "ibert_layernorm_i": (C.c_int, [_P, _P, C.c_int64, C.c_int32, C.c_int64, C.c_int64, _P, _P, C.c_int32, _P]),
    "ibert_layernorm_i16": (C.c_int, [_P, _P, C.c_int64, C.c_int32, C.c_int64, C.c_int64, _P, _P, C.c_int32, _P]),
    "ibert_encoder_layer_workspace_bytes": (C.c_size_t, [C.c_int32] * 5),
    "ibert_encoder_layer_workspace_layout": (C.c_int, [C.c_int32] * 5 + [C.POINTER(WorkspaceLayout)]),
    "ibert_encoder_layer_i": (C.c_int, [C.POINTER(LayerWeights), C.POINTER(LayerQuant), _P, _P] + [C.c_int32] * 5 +
                              [_P, C.c_size_t, _P]),
    "ibert_static_scratch_bytes": (C.c_size_t, []),
    "ibert_static_scratch_init": (C.c_int, []),
    "ibert_encoder_layer_static_i": (C.c_int, [C.POINTER(LayerWeights), C.POINTER(LayerQuant), _P, _P] + [C.c_int32] * 5 +
                                     [_P, _P]),
    "ibert_encoder_workspace_bytes": (C.c_size_t, [C.c_int32] * 5),
    "ibert_encoder_i": (C.c_int, [C.POINTER(LayerWeights), C.POINTER(LayerQuant), C.c_int32, _P, _P] +
                        [C.c_int32] * 5 + [_P, C.c_size_t, _P]),
    "ibert_dyadic_from_double": (C.c_int, [C.c_double, C.POINTER(Dyadic)]),
    "ibert_channel_dyadics_from_scales": (C.c_int, [C.c_double, _P, C.c_int32, C.c_double, _P, _P]),
    "ibert_softmax_params_from_scale": (C.c_int, [C.c_double, C.c_int32, C.c_int32, C.c_int32, C.POINTER(SoftmaxParams)]),
    "ibert_gelu_params_from_scale": (C.c_int, [C.c_double, C.c_double, C.POINTER(GeluParams)]),
    "ibert_layernorm_params_from_float": (C.c_int, [_P, _P, C.c_int32, C.c_double, _P, _P, C.POINTER(C.c_int32)]),
    "ibert_layer_quant_from_scales": (C.c_int, [C.POINTER(LayerScales), C.c_int32, C.c_int32, C.POINTER(LayerQuant)]),
    "ibert_profile_begin": (C.c_int, [C.c_int32]),
    "ibert_profile_end": (C.c_int, [C.POINTER(ProfileRecord), C.c_int32, C.POINTER(C.c_int32)]),
    "ibert_status_string": (C.c_char_p, [C.c_int]),
    "ibert_last_hip_error": (C.c_char_p, []),
    "ibert_version": (C.c_int, []),
}

_lib = None


def lib():
    """The loaded shared library.  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libibert.so is missing: build it with `python -m paper_2101_01321_amd.build` "
                               "(or __graft_entry__.build()); there is no fallback path")
        L = C.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(L, name)
            fn.restype = res
            fn.argtypes = args
        _lib = L
    return _lib


def _chk(rc: int, where: str):
    if rc != OK:
        raise IbertError(rc, where)


def _dp(t) -> Optional[int]:
    """Device pointer of a torch tensor (None -> NULL)."""
    return None if t is None else t.data_ptr()


def _stream(stream=None) -> int:
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream


# ------------------------------------------------------------------------- host helpers
def ibert_dyadic_from_double(M: float) -> Dyadic:
    d = Dyadic()
    _chk(lib().ibert_dyadic_from_double(float(M), C.byref(d)), "ibert_dyadic_from_double")
    return d


def ibert_channel_dyadics_from_scales(S_in: float, S_w: np.ndarray, S_out: float):
    S_w = np.ascontiguousarray(S_w, dtype=np.float64)
    mult = np.empty(S_w.shape, np.int32)
    shift = np.empty(S_w.shape, np.int32)
    _chk(lib().ibert_channel_dyadics_from_scales(float(S_in), S_w.ctypes.data, S_w.size, float(S_out),
                                                 mult.ctypes.data, shift.ctypes.data),
         "ibert_channel_dyadics_from_scales")
    return mult, shift


def ibert_softmax_params_from_scale(S: float, cols: int, out_frac_bits: int = 7, out_dtype: int = I8) -> SoftmaxParams:
    p = SoftmaxParams()
    _chk(lib().ibert_softmax_params_from_scale(float(S), cols, out_frac_bits, out_dtype, C.byref(p)),
         "ibert_softmax_params_from_scale")
    return p


def ibert_gelu_params_from_scale(S_in: float, S_out: float) -> GeluParams:
    p = GeluParams()
    _chk(lib().ibert_gelu_params_from_scale(float(S_in), float(S_out), C.byref(p)), "ibert_gelu_params_from_scale")
    return p


def ibert_layernorm_params_from_float(gamma: np.ndarray, beta: np.ndarray, S_out: float):
    gamma = np.ascontiguousarray(gamma, dtype=np.float64)
    beta = np.ascontiguousarray(beta, dtype=np.float64)
    gq = np.empty(gamma.shape, np.int32)
    bq = np.empty(gamma.shape, np.int32)
    s = C.c_int32(0)
    _chk(lib().ibert_layernorm_params_from_float(gamma.ctypes.data, beta.ctypes.data, gamma.size, float(S_out),
                                                 gq.ctypes.data, bq.ctypes.data, C.byref(s)),
         "ibert_layernorm_params_from_float")
    return gq, bq, int(s.value)


def ibert_layer_quant_from_scales(sc: dict, seq: int, head_dim: int) -> LayerQuant:
    s = LayerScales()
    for name, _ in LayerScales._fields_:
        setattr(s, name, sc[name])
    q = LayerQuant()
    _chk(lib().ibert_layer_quant_from_scales(C.byref(s), seq, head_dim, C.byref(q)), "ibert_layer_quant_from_scales")
    return q


# ------------------------------------------------------------------------- compute entry points
def ibert_gemm_i8_requant(desc: GemmDesc, A, W, bias, mult, shift, residual, Cout, stream=None):
    _chk(lib().ibert_gemm_i8_requant(C.byref(desc), _dp(A), _dp(W), _dp(bias), _dp(mult), _dp(shift), _dp(residual),
                                     _dp(Cout), _stream(stream)), "ibert_gemm_i8_requant")


def ibert_gemm_i8_gelu(desc: GemmDesc, A, W, bias, mult, shift, gelu: GeluParams, Cout, scratch, stream=None):
    _chk(lib().ibert_gemm_i8_gelu(C.byref(desc), _dp(A), _dp(W), _dp(bias), _dp(mult), _dp(shift), C.byref(gelu),
                                  _dp(Cout), _dp(scratch), _stream(stream)), "ibert_gemm_i8_gelu")


def ibert_attention_scratch_bytes(batch: int, seq: int, heads: int) -> int:
    return int(lib().ibert_attention_scratch_bytes(batch, seq, heads))


def ibert_attention_i(qkv, ctx, batch, seq, hidden, heads, scores_dy: Dyadic, softmax: SoftmaxParams, ctx_dy: Dyadic,
                      scratch=None, stream=None):
    nbytes = 0 if scratch is None else scratch.numel() * scratch.element_size()
    _chk(lib().ibert_attention_i(_dp(qkv), _dp(ctx), batch, seq, hidden, heads, C.byref(scores_dy), C.byref(softmax),
                                 C.byref(ctx_dy), _dp(scratch), nbytes, _stream(stream)), "ibert_attention_i")


def ibert_attention_masked_i(qkv, ctx, batch, seq, hidden, heads, scores_dy: Dyadic, softmax: SoftmaxParams, ctx_dy: Dyadic,
                             key_lens, scratch=None, stream=None):
    nbytes = 0 if scratch is None else scratch.numel() * scratch.element_size()
    _chk(lib().ibert_attention_masked_i(_dp(qkv), _dp(ctx), batch, seq, hidden, heads, C.byref(scores_dy), C.byref(softmax),
                                        C.byref(ctx_dy), _dp(key_lens), _dp(scratch), nbytes, _stream(stream)),
         "ibert_attention_masked_i")


def ibert_softmax_masked_i(x, y, rows: int, cols: int, ldx: int, ldy: int, params: SoftmaxParams, key_lens,
                           rows_per_len: int, stream=None):
    _chk(lib().ibert_softmax_masked_i(_dp(x), _dp(y), rows, cols, ldx, ldy, C.byref(params), _dp(key_lens), rows_per_len,
                                      _stream(stream)), "ibert_softmax_masked_i")


def ibert_embedding_i(ids, tok, pos, tokens: int, seq: int, hidden: int, vocab: int, max_pos: int, tok_dy: Dyadic,
                      pos_dy: Dyadic, gamma_q, beta_q, ln_shift: int, y, ldy: int, stream=None):
    _chk(lib().ibert_embedding_i(_dp(ids), _dp(tok), _dp(pos), tokens, seq, hidden, vocab, max_pos, C.byref(tok_dy),
                                 C.byref(pos_dy), _dp(gamma_q), _dp(beta_q), ln_shift, _dp(y), ldy, _stream(stream)),
         "ibert_embedding_i")


EPILOGUE_STAGED, EPILOGUE_DIRECT, EPILOGUE_DIRECT_GELU_TABLE, EPILOGUE_EDGE = 1, 2, 3, 4


def ibert_gemm_epilogue_record(word):
    """word: a uint32/int32 device tensor of one element, or None to switch the record off."""
    lib().ibert_gemm_epilogue_record(_dp(word))


def ibert_isqrt_i(n, root, count: int, method: int, stream=None):
    _chk(lib().ibert_isqrt_i(_dp(n), _dp(root), count, method, _stream(stream)), "ibert_isqrt_i")


def ibert_softmax_i(x, y, rows: int, cols: int, ldx: int, ldy: int, params: SoftmaxParams, stream=None):
    _chk(lib().ibert_softmax_i(_dp(x), _dp(y), rows, cols, ldx, ldy, C.byref(params), _stream(stream)),
         "ibert_softmax_i")


def ibert_gelu_i(x, y, n: int, params: GeluParams, stream=None):
    _chk(lib().ibert_gelu_i(_dp(x), _dp(y), n, C.byref(params), _stream(stream)), "ibert_gelu_i")


def ibert_hgelu_params_from_scale(S_in: float, S_out: float) -> HGeluParams:
    p = HGeluParams()
    _chk(lib().ibert_hgelu_params_from_scale(float(S_in), float(S_out), C.byref(p)), "ibert_hgelu_params_from_scale")
    return p


def ibert_hgelu_i(x, y, n: int, params: HGeluParams, stream=None):
    _chk(lib().ibert_hgelu_i(_dp(x), _dp(y), n, C.byref(params), _stream(stream)), "ibert_hgelu_i")


def ibert_layernorm_i(x, y, rows: int, Cc: int, ldx: int, ldy: int, gamma_q, beta_q, shift: int, stream=None):
    _chk(lib().ibert_layernorm_i(_dp(x), _dp(y), rows, Cc, ldx, ldy, _dp(gamma_q), _dp(beta_q), shift,
                                 _stream(stream)), "ibert_layernorm_i")


def ibert_layernorm_i16(x, y, rows: int, Cc: int, ldx: int, ldy: int, gamma_q, beta_q, shift: int, stream=None):
    _chk(lib().ibert_layernorm_i16(_dp(x), _dp(y), rows, Cc, ldx, ldy, _dp(gamma_q), _dp(beta_q), shift,
                                   _stream(stream)), "ibert_layernorm_i16")


def ibert_encoder_layer_workspace_bytes(batch, seq, hidden, heads, ffn) -> int:
    return int(lib().ibert_encoder_layer_workspace_bytes(batch, seq, hidden, heads, ffn))


def ibert_encoder_workspace_bytes(batch, seq, hidden, heads, ffn) -> int:
    return int(lib().ibert_encoder_workspace_bytes(batch, seq, hidden, heads, ffn))


def ibert_encoder_layer_workspace_layout(batch, seq, hidden, heads, ffn) -> WorkspaceLayout:
    lo = WorkspaceLayout()
    _chk(lib().ibert_encoder_layer_workspace_layout(batch, seq, hidden, heads, ffn, C.byref(lo)),
         "ibert_encoder_layer_workspace_layout")
    return lo


def ibert_encoder_layer_i(weights: LayerWeights, quant: LayerQuant, x, y, batch, seq, hidden, heads, ffn,
                          workspace, stream=None):
    _chk(lib().ibert_encoder_layer_i(C.byref(weights), C.byref(quant), _dp(x), _dp(y), batch, seq, hidden, heads, ffn,
                                     _dp(workspace), workspace.numel() * workspace.element_size(), _stream(stream)),
         "ibert_encoder_layer_i")


def ibert_encoder_layer_masked_i(weights: LayerWeights, quant: LayerQuant, x, y, batch, seq, hidden, heads, ffn, key_lens,
                                 workspace, stream=None):
    _chk(lib().ibert_encoder_layer_masked_i(C.byref(weights), C.byref(quant), _dp(x), _dp(y), batch, seq, hidden, heads,
                                            ffn, _dp(key_lens), _dp(workspace),
                                            workspace.numel() * workspace.element_size(), _stream(stream)),
         "ibert_encoder_layer_masked_i")


def ibert_static_scratch_bytes() -> int:
    return int(lib().ibert_static_scratch_bytes())


def ibert_static_scratch_init():
    _chk(lib().ibert_static_scratch_init(), "ibert_static_scratch_init")


def ibert_encoder_layer_static_i(weights: LayerWeights, quant: LayerQuant, x, y, batch, seq, hidden, heads, ffn,
                                 key_lens=None, stream=None):
    _chk(lib().ibert_encoder_layer_static_i(C.byref(weights), C.byref(quant), _dp(x), _dp(y), batch, seq, hidden, heads,
                                            ffn, _dp(key_lens), _stream(stream)), "ibert_encoder_layer_static_i")


def ibert_encoder_masked_i(weights, quant, n_layers: int, x, y, batch, seq, hidden, heads, ffn, key_lens, workspace,
                           stream=None):
    _chk(lib().ibert_encoder_masked_i(weights, quant, n_layers, _dp(x), _dp(y), batch, seq, hidden, heads, ffn,
                                      _dp(key_lens), _dp(workspace), workspace.numel() * workspace.element_size(),
                                      _stream(stream)), "ibert_encoder_masked_i")


def ibert_encoder_i(weights, quant, n_layers: int, x, y, batch, seq, hidden, heads, ffn, workspace, stream=None):
    """weights / quant: ctypes arrays (LayerWeights * n, LayerQuant * n)."""
    _chk(lib().ibert_encoder_i(weights, quant, n_layers, _dp(x), _dp(y), batch, seq, hidden, heads, ffn,
                               _dp(workspace), workspace.numel() * workspace.element_size(), _stream(stream)),
         "ibert_encoder_i")


def ibert_profile_begin(capacity: int):
    _chk(lib().ibert_profile_begin(capacity), "ibert_profile_begin")


def ibert_profile_end(capacity: int):
    """Returns a list of (step, ms, ops, bytes, kernel)."""
    recs = (ProfileRecord * capacity)()
    n = C.c_int32(0)
    _chk(lib().ibert_profile_end(recs, capacity, C.byref(n)), "ibert_profile_end")
    return [(r.step, r.ms, r.ops, r.bytes, r.kernel.decode()) for r in recs[:n.value]]


# ------------------------------------------------------------------------- model marshalling
_W_I8 = ("w_qkv", "w_o", "w_1", "w_2")


class DeviceLayer:
    """One layer's integer parameters resident on the GPU (built only through the library's host helpers)."""

    def __init__(self, raw: dict, sc: dict, hidden: int, heads: int, seq: int, device):
        import torch
        H = hidden
        host = {}
        host["w_qkv"], host["b_qkv"] = raw["w_qkv"], raw["b_qkv"]
        parts = [ibert_channel_dyadics_from_scales(sc["S_x"], raw["sw_qkv"][i * H:(i + 1) * H], sc[k])
                 for i, k in enumerate(("S_q", "S_k", "S_v"))]
        host["m_qkv"] = np.concatenate([p[0] for p in parts])
        host["s_qkv"] = np.concatenate([p[1] for p in parts])
        host["w_o"], host["b_o"] = raw["w_o"], raw["b_o"]
        host["m_o"], host["s_o"] = ibert_channel_dyadics_from_scales(sc["S_ctx"], raw["sw_o"], sc["S_r1"])
        host["ln1_gamma_q"], host["ln1_beta_q"], ln1 = ibert_layernorm_params_from_float(raw["gamma1"], raw["beta1"], sc["S_h1"])
        host["w_1"], host["b_1"] = raw["w_1"], raw["b_1"]
        host["m_1"], host["s_1"] = ibert_channel_dyadics_from_scales(sc["S_h1"], raw["sw_1"], sc["S_g_in"])
        host["w_2"], host["b_2"] = raw["w_2"], raw["b_2"]
        host["m_2"], host["s_2"] = ibert_channel_dyadics_from_scales(sc["S_g_out"], raw["sw_2"], sc["S_r2"])
        host["ln2_gamma_q"], host["ln2_beta_q"], ln2 = ibert_layernorm_params_from_float(raw["gamma2"], raw["beta2"], sc["S_y"])
        self.host = host
        self.tensors = {}
        self.weights = LayerWeights()
        for name, _ in LayerWeights._fields_:
            dt = np.int8 if name in _W_I8 else np.int32
            t = torch.from_numpy(np.ascontiguousarray(host[name], dtype=dt)).to(device)
            self.tensors[name] = t
            setattr(self.weights, name, t.data_ptr())
        self.quant = ibert_layer_quant_from_scales(sc, seq, hidden // heads)
        self.quant.ln1_shift, self.quant.ln2_shift = ln1, ln2
