"""Helpers for the GPU parity tests: numpy in, HIP library through the C ABI, numpy out."""
import sys

import numpy as np
import torch

from paper_2101_01321_amd import binding as B, synth

DEV = torch.device("cuda:0")


def say(msg):
    """Name the case before its GPU step (flushed, so a fault still leaves the name behind)."""
    print("[gpu-case] " + msg, file=sys.stderr, flush=True)


def to_dev(a, dtype=None):
    a = np.ascontiguousarray(a, dtype=dtype)
    return torch.from_numpy(a).to(DEV)


def gemm(desc_kwargs, A, W, bias=None, mult=None, shift=None, residual=None, out_elems=None, offsets=None):
    """Flat-buffer GEMM call.  desc_kwargs: fields of GemmDesc (requant / residual_dy as (m, s) tuples).
    offsets: optional dict of element offsets {'A':..,'W':..,'C':..,'R':..} applied to the device pointers."""
    d = B.GemmDesc()
    for k, v in desc_kwargs.items():
        if k in ("requant", "residual_dy"):
            setattr(d, k, B.Dyadic(*v))
        else:
            setattr(d, k, v)
    offsets = offsets or {}
    i8 = d.out_dtype == B.I8
    tA, tW = to_dev(A, np.int8).reshape(-1), to_dev(W, np.int8).reshape(-1)
    tb = None if bias is None else to_dev(bias, np.int32)
    tm = None if mult is None else to_dev(mult, np.int32)
    ts = None if shift is None else to_dev(shift, np.int32)
    tR = None if residual is None else to_dev(residual, np.int8).reshape(-1)
    sentinel = 77
    out_t = torch.int8 if i8 else (torch.int16 if d.out_dtype == B.I16 else torch.int32)
    tC = torch.full((out_elems + offsets.get("C", 0),), sentinel, dtype=out_t, device=DEV)

    def off(t, key):
        return None if t is None else t[offsets.get(key, 0):]
    B.ibert_gemm_i8_requant(d, off(tA, "A"), off(tW, "W"), tb, tm, ts, off(tR, "R"), off(tC, "C"))
    torch.cuda.synchronize()
    return tC[offsets.get("C", 0):].cpu().numpy()


def gemm_gelu(desc_kwargs, A, W, bias, mult, shift, gelu_params, out_elems, with_scratch=True):
    """Fused MatMul + GELU call (dense INT8 output).  Returns (output, scratch-or-None) as numpy."""
    d = B.GemmDesc()
    for k, v in desc_kwargs.items():
        setattr(d, k, B.Dyadic(*v) if k in ("requant", "residual_dy") else v)
    tA, tW = to_dev(A, np.int8).reshape(-1), to_dev(W, np.int8).reshape(-1)
    tb = None if bias is None else to_dev(bias, np.int32)
    tm = None if mult is None else to_dev(mult, np.int32)
    ts = None if shift is None else to_dev(shift, np.int32)
    tC = torch.full((out_elems + 16,), 77, dtype=torch.int8, device=DEV)
    tS = torch.full((out_elems,), -5, dtype=torch.int32, device=DEV) if with_scratch else None
    B.ibert_gemm_i8_gelu(d, tA, tW, tb, tm, ts, gelu_params, tC, tS)
    torch.cuda.synchronize()
    out = tC.cpu().numpy()
    assert np.all(out[out_elems:] == 77), "wrote past the end"
    return out[:out_elems], (None if tS is None else tS.cpu().numpy())


def attention(qkv, batch, seq, hidden, heads, scores_dy, softmax_params, ctx_dy, with_scratch=True, key_lens=None):
    """Steps 2-4 through ibert_attention_i (ibert_attention_masked_i with key_lens).  qkv: int8 [batch*seq, 3*hidden];
    returns ctx int8 [batch*seq, hidden]."""
    tq = to_dev(qkv, np.int8)
    tc = torch.full((batch * seq * hidden + 16,), 77, dtype=torch.int8, device=DEV)
    ts = None
    if with_scratch:
        ts = torch.zeros(B.ibert_attention_scratch_bytes(batch, seq, heads), dtype=torch.uint8, device=DEV)
    if key_lens is None:
        B.ibert_attention_i(tq, tc, batch, seq, hidden, heads, B.Dyadic(*scores_dy), softmax_params, B.Dyadic(*ctx_dy), ts)
    else:
        B.ibert_attention_masked_i(tq, tc, batch, seq, hidden, heads, B.Dyadic(*scores_dy), softmax_params,
                                   B.Dyadic(*ctx_dy), to_dev(key_lens, np.int32), ts)
    torch.cuda.synchronize()
    out = tc.cpu().numpy()
    assert np.all(out[batch * seq * hidden:] == 77), "wrote past the end"
    return out[:batch * seq * hidden].reshape(batch * seq, hidden)


def softmax(x, params, cols=None, ldx=None, ldy=None, x_off=0, y_off=0, key_lens=None, rows_per_len=1):
    x = np.ascontiguousarray(x, np.int32)
    rows = x.shape[0]
    ldx = x.shape[1] if ldx is None else ldx
    cols = x.shape[1] if cols is None else cols
    ldy = ldx if ldy is None else ldy
    tx = torch.zeros(rows * ldx + x_off, dtype=torch.int32, device=DEV)
    tx[x_off:].view(rows, ldx)[:, :x.shape[1]] = to_dev(x)
    i8 = params.out_dtype == B.I8
    ty = torch.full((rows * ldy + y_off,), 77, dtype=torch.int8 if i8 else torch.int32, device=DEV)
    if key_lens is None:
        B.ibert_softmax_i(tx[x_off:], ty[y_off:], rows, cols, ldx, ldy, params)
    else:
        B.ibert_softmax_masked_i(tx[x_off:], ty[y_off:], rows, cols, ldx, ldy, params, to_dev(key_lens, np.int32), rows_per_len)
    torch.cuda.synchronize()
    return ty[y_off:].view(rows, ldy).cpu().numpy()


def gelu(x, params, x_off=0, y_off=0):
    x = np.ascontiguousarray(x, np.int32).reshape(-1)
    tx = torch.zeros(x.size + x_off, dtype=torch.int32, device=DEV)
    tx[x_off:] = to_dev(x)
    ty = torch.full((x.size + y_off + 8,), 77, dtype=torch.int8, device=DEV)
    B.ibert_gelu_i(tx[x_off:], ty[y_off:], x.size, params)
    torch.cuda.synchronize()
    out = ty.cpu().numpy()
    assert np.all(out[y_off + x.size:] == 77), "wrote past the end"
    return out[y_off:y_off + x.size]


def hgelu(x, params, x_off=0, y_off=0):
    x = np.ascontiguousarray(x, np.int32).reshape(-1)
    tx = torch.zeros(x.size + x_off, dtype=torch.int32, device=DEV)
    tx[x_off:] = to_dev(x)
    ty = torch.full((x.size + y_off + 8,), 77, dtype=torch.int8, device=DEV)
    B.ibert_hgelu_i(tx[x_off:], ty[y_off:], x.size, params)
    torch.cuda.synchronize()
    out = ty.cpu().numpy()
    assert np.all(out[:y_off] == 77) and np.all(out[y_off + x.size:] == 77), "wrote outside the output"
    return out[y_off:y_off + x.size]


def layernorm(x, gamma_q, beta_q, shift, ldx=None, ldy=None, x_off=0, y_off=0, half=False):
    """ibert_layernorm_i, or ibert_layernorm_i16 on the same values stored as int16 (half=True)."""
    x = np.ascontiguousarray(x, np.int16 if half else np.int32)
    rows, Cc = x.shape
    ldx = Cc if ldx is None else ldx
    ldy = ldx if ldy is None else ldy
    tx = torch.zeros(rows * ldx + x_off, dtype=torch.int16 if half else torch.int32, device=DEV)
    tx[x_off:].view(rows, ldx)[:, :Cc] = to_dev(x)
    ty = torch.full((rows * ldy + y_off,), 77, dtype=torch.int8, device=DEV)
    call = B.ibert_layernorm_i16 if half else B.ibert_layernorm_i
    call(tx[x_off:], ty[y_off:], rows, Cc, ldx, ldy, to_dev(gamma_q, np.int32), to_dev(beta_q, np.int32), shift)
    torch.cuda.synchronize()
    return ty[y_off:].view(rows, ldy).cpu().numpy()


def embedding(ids, seq, tok, pos, tok_dy, pos_dy, gamma_q, beta_q, shift, ldy=None, y_off=0):
    """ibert_embedding_i; returns int8 [tokens, hidden]."""
    ids = np.ascontiguousarray(ids, np.int32)
    T, H = ids.size, tok.shape[1]
    ldy = H if ldy is None else ldy
    ty = torch.full((T * ldy + y_off + 16,), 77, dtype=torch.int8, device=DEV)
    B.ibert_embedding_i(to_dev(ids), to_dev(tok, np.int8), to_dev(pos, np.int8), T, seq, H, tok.shape[0], pos.shape[0],
                        B.Dyadic(*tok_dy), B.Dyadic(*pos_dy), to_dev(gamma_q, np.int32), to_dev(beta_q, np.int32), shift,
                        ty[y_off:], ldy)
    torch.cuda.synchronize()
    out = ty.cpu().numpy()
    assert np.all(out[:y_off] == 77) and np.all(out[y_off + T * ldy:] == 77), "wrote outside the output"
    body = out[y_off:y_off + T * ldy].reshape(T, ldy)
    assert np.all(body[:, H:] == 77), "wrote into the row padding"
    return body[:, :H]


def isqrt(n, method):
    """ibert_isqrt_i on a uint32 array."""
    n = np.ascontiguousarray(n, np.uint32)
    tn = torch.from_numpy(n.view(np.int32)).to(DEV)
    tr = torch.full((n.size + 8,), -1, dtype=torch.int32, device=DEV)
    B.ibert_isqrt_i(tn, tr, n.size, method)
    torch.cuda.synchronize()
    out = tr.cpu().numpy()
    assert np.all(out[n.size:] == -1), "wrote outside the output"
    return out[:n.size].view(np.uint32)


class DeviceModel:
    """All layers of a synthetic encoder resident on the GPU, plus workspace."""

    def __init__(self, cfg: synth.EncoderConfig, S_x: float, n_layers=None, seed=synth.SEED):
        self.cfg = cfg
        self.n_layers = cfg.layers if n_layers is None else n_layers
        self.scales = synth.model_scales(cfg, S_x)[:self.n_layers]
        self.layers = [B.DeviceLayer(synth.layer_raw(cfg, l, seed), self.scales[l], cfg.hidden, cfg.heads, cfg.seq, DEV)
                       for l in range(self.n_layers)]
        self.weights = (B.LayerWeights * self.n_layers)(*[l.weights for l in self.layers])
        self.quant = (B.LayerQuant * self.n_layers)(*[l.quant for l in self.layers])
        c = cfg
        self.ws_bytes = B.ibert_encoder_workspace_bytes(c.batch, c.seq, c.hidden, c.heads, c.ffn)
        self.ws = torch.zeros(self.ws_bytes, dtype=torch.uint8, device=DEV)
        self.layout = B.ibert_encoder_layer_workspace_layout(c.batch, c.seq, c.hidden, c.heads, c.ffn)

    def forward(self, x_q: torch.Tensor, key_lens=None) -> torch.Tensor:
        c = self.cfg
        y = torch.empty_like(x_q)
        if key_lens is None:
            B.ibert_encoder_i(self.weights, self.quant, self.n_layers, x_q, y, c.batch, c.seq, c.hidden, c.heads, c.ffn, self.ws)
        else:
            B.ibert_encoder_masked_i(self.weights, self.quant, self.n_layers, x_q, y, c.batch, c.seq, c.hidden, c.heads,
                                     c.ffn, key_lens, self.ws)
        return y

    def layer_forward(self, l: int, x_q: torch.Tensor, key_lens=None) -> torch.Tensor:
        c = self.cfg
        y = torch.empty_like(x_q)
        if key_lens is None:
            B.ibert_encoder_layer_i(self.layers[l].weights, self.layers[l].quant, x_q, y, c.batch, c.seq, c.hidden, c.heads,
                                    c.ffn, self.ws)
        else:
            B.ibert_encoder_layer_masked_i(self.layers[l].weights, self.layers[l].quant, x_q, y, c.batch, c.seq, c.hidden,
                                           c.heads, c.ffn, key_lens, self.ws)
        return y

    def set_route(self, route: int):
        """ibert_layer_quant.route of every layer (0 = every fusion; B.ROUTE_* flags)."""
        for l in range(self.n_layers):
            self.layers[l].quant.route = route
            self.quant[l].route = route

    def mark_unwritten(self):
        """Plants a pattern at the start of the INT32 tensors r1 and r2, to see afterwards whether a step wrote them."""
        for off in (self.layout.r1, self.layout.r2):
            self.ws[off:off + 16] = 0x7B

    def was_written(self, name: str) -> bool:
        off = getattr(self.layout, name)
        return not bool(torch.all(self.ws[off:off + 16] == 0x7B).item())

    def intermediates(self, r_half: bool = False) -> dict:
        """r_half: r1 / r2 were stored as int16 (the default route); they are returned widened."""
        c, lo = self.cfg, self.layout
        T, H, F, BH, L = c.tokens, c.hidden, c.ffn, c.batch * c.heads, c.seq
        spec = {"qkv": (lo.qkv, (T, 3 * H), torch.int8), "scores": (lo.scores, (BH, L, L), torch.int32),
                "probs": (lo.probs, (BH, L, L), torch.int8), "ctx": (lo.ctx, (T, H), torch.int8),
                "r1": (lo.r1, (T, H), torch.int32), "h1": (lo.h1, (T, H), torch.int8),
                "f1": (lo.f1, (T, F), torch.int32), "g": (lo.g, (T, F), torch.int8), "r2": (lo.r2, (T, H), torch.int32)}
        out = {}
        for k, (off, shape, dt) in spec.items():
            if r_half and k in ("r1", "r2"):
                n = int(np.prod(shape)) * 2
                out[k] = self.ws[off:off + n].view(torch.int16).view(*shape).cpu().numpy().astype(np.int32)
                continue
            n = int(np.prod(shape)) * (4 if dt == torch.int32 else 1)
            out[k] = self.ws[off:off + n].view(dt).view(*shape).cpu().numpy()
        return out
