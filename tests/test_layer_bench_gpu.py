"""The one-layer benchmark (a device's share of a transformer layer, Table 1 shapes): the
attention it runs is the library's ring, checked here against the oracle on the tensors the
layer actually fed it; the model it prints beside the measurement is Sec. 4's, checked by hand."""
import numpy as np
import pytest
import torch

from oracle import striped_attention as orc
from paper_2311_09431_amd import layer_bench as lb
from paper_2311_09431_amd import tms

SMALL = dict(n_vocab=0, d_model=256, d_ff=512, n_layer=1, n_head=2)


def test_one_layer_tms_by_hand():
    # 7B, 256k, N = 8, one layer: other = 2 (4 d^2 + 2 d d_ff), attention = 4 n_seq d per token
    d, dff, S, N = 4096, 11008, 262144, 8
    other, attn = 2 * (4 * d * d + 2 * d * dff), 4 * S * d
    want = (other + attn * (N - 0.5) / N) / (other + attn / 2)
    assert abs(lb.layer_tms("7B", S, N) - want) < 1e-12
    assert 1.76 < want < 1.77
    # without the logits term the one-layer figure is above the paper's whole-model one
    assert lb.layer_tms("7B", S, N) > tms.tms("7B", S, N, 1.0)


@pytest.mark.gpu
@pytest.mark.parametrize("layout", [0, 1])
def test_layer_attention_matches_the_oracle(layout):
    from paper_2311_09431_amd import binding as sa
    from paper_2311_09431_amd import inputs
    S, N = 2048, 4
    layer = lb.DeviceLayer(SMALL, S, N, layout)
    layer.step(lambda name: None)
    torch.cuda.synchronize()
    c, dev, H, d = layer.c, layer.dev, layer.H, layer.d
    un = (lambda x: orc.unstripe_permute(x, N, 2)) if layout == sa.STRIPED else (lambda x: x)
    # rows of the played device are rotated (they were projected here); the other devices' K, V
    # are synthetic and enter as they are
    Q, K, V = (un(inputs.to_f64(t)) for t in (layer.Qv, layer.Kv, layer.Vv))
    rows = [orc.global_position(dev, a, N, c, layout) for a in range(c)]
    scale = 1.0 / np.sqrt(d)
    got = layer.rows(layer.out).float().cpu().numpy()
    for h in range(H):
        want, _ = orc.causal_attention_rows(Q[0, h], K[0, h], V[0, h], scale, rows)
        assert np.abs(got[0, h] - want).max() <= 3e-2        # bf16 output: one more rounding
    assert all(torch.isfinite(t).all() for t in (layer.dQ, layer.dK, layer.dV))


@pytest.mark.gpu
def test_layer_bench_runs_and_reports():
    r = lb.run(SMALL, 4096, 4, reps=1)
    assert r["striped"]["layer_ms"] > 0 and r["ring"]["layer_ms"] > 0
    assert r["attention_only_limit"] == round(tms.attention_only_limit(4, 1024), 3)
