"""The layer entry point that allocates nothing (its workspace is an array inside the library's device image) against the
entry point that takes a caller's workspace: same output bit for bit, on two calls in a row, the second one smaller."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from paper_2101_01321_amd import synth


def test_static_scratch_layer_equals_workspace_layer(gpu):
    import torch
    import gpu_util as G
    from paper_2101_01321_amd import binding as B
    B.lib()
    assert B.ibert_static_scratch_bytes() == 32 << 20
    B.ibert_static_scratch_init()
    first = synth.EncoderConfig("static_a", 384, 6, 1536, 128, 3, 1)          # 4.4 MB of intermediates, whole MatMul tiles
    second = synth.EncoderConfig("static_b", 192, 3, 320, 40, 2, 1)           # smaller and ragged: leaves most of the array stale
    for cfg, lens in ((first, None), (second, None), (first, (128, 17, 90))):
        assert B.ibert_encoder_layer_workspace_bytes(cfg.batch, cfg.seq, cfg.hidden, cfg.heads, cfg.ffn) <= B.ibert_static_scratch_bytes()
        x_q, S_x, _ = synth.input_activations(cfg)
        model = G.DeviceModel(cfg, S_x)
        tx = G.to_dev(x_q)
        tl = None if lens is None else G.to_dev(np.array(lens, np.int32))
        G.say("static-scratch layer %s lens=%s: workspace entry point" % (cfg.name, lens))
        want = model.layer_forward(0, tx, key_lens=tl)
        torch.cuda.synchronize()
        ty = torch.full_like(tx, 77)
        G.say("static-scratch layer %s lens=%s: static entry point" % (cfg.name, lens))
        B.ibert_encoder_layer_static_i(model.layers[0].weights, model.layers[0].quant, tx, ty, cfg.batch, cfg.seq, cfg.hidden,
                                       cfg.heads, cfg.ffn, key_lens=tl)
        torch.cuda.synchronize()
        got, ref = ty.cpu().numpy(), want.cpu().numpy()
        assert np.array_equal(got, ref), "%s: %d of %d elements differ" % (cfg.name, int((got != ref).sum()), ref.size)
        assert len(np.unique(ref)) > 20
    # a problem whose intermediates do not fit the array is refused before anything is launched
    big = synth.CONFIGS["base_b32"]
    x_q, S_x, _ = synth.input_activations(first)
    model = G.DeviceModel(first, S_x)
    t = torch.zeros(big.tokens, big.hidden, dtype=torch.int8, device=G.DEV)
    with pytest.raises(B.IbertError):
        B.ibert_encoder_layer_static_i(model.layers[0].weights, model.layers[0].quant, t, torch.empty_like(t), big.batch, big.seq,
                                       big.hidden, big.heads, big.ffn)
