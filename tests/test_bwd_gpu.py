"""GPU parity of the backward ring step (dQ, dK, dV accumulated over the ring)
against the fp64 analytic gradient of causal attention, through the C ABI."""
import numpy as np
import pytest
import torch

from paper_2311_09431_amd import binding as sa
from paper_2311_09431_amd import inputs
from tests import helpers as hp

pytestmark = pytest.mark.gpu


def _tolerance(dtype, ref):
    # fp32 path: 1e-5 scaled by the gradient's magnitude; bf16 inputs with fp32
    # accumulation: 2e-2 * max(1, max|ref|) (the forward's bf16 bound, scaled)
    scale = max(1.0, float(np.max(np.abs(ref))))
    return (2e-5 if dtype == torch.float32 else 2e-2) * scale


def _check(B, H, S, d, N, layout, dtype, seed, use_driver=False):
    Q, K, V, dO = inputs.qkv(B, H, S, d, seed, dtype, with_dout=True)
    sc = 1.0 / np.sqrt(d)
    got = hp.ring_backward_gpu(Q.cuda(), K.cuda(), V.cuda(), dO.cuda(), N, layout, None, use_driver)
    torch.cuda.synchronize()
    want = hp.oracle_backward(Q, K, V, dO, sc)
    for name, g, w in zip(("dQ", "dK", "dV"), got, want):
        gh = hp.from_device_order_host(g.cpu().numpy(), N, layout)
        assert np.isfinite(gh).all()
        err = hp.max_abs_err(gh, w)
        assert err <= _tolerance(dtype, w), (name, err, hp.layout_name(layout))
        hp.check_grad(name + " " + hp.layout_name(layout), gh, w, dtype != torch.float32)


@pytest.mark.parametrize("layout", [sa.CONTIGUOUS, sa.STRIPED])
@pytest.mark.parametrize("B,H,S,d,N,dtype", [
    (1, 1, 256, 64, 4, torch.float32),
    (2, 2, 120, 32, 4, torch.float32),     # ragged c = 30
    (1, 1, 8, 4, 8, torch.float32),        # c = 1
    (1, 2, 192, 64, 4, torch.bfloat16),
    (1, 2, 96, 128, 4, torch.bfloat16),
    (1, 2, 128, 100, 4, torch.bfloat16),   # head dimension of Table 1's 3B model
])
def test_generic_backward(layout, B, H, S, d, N, dtype):
    _check(B, H, S, d, N, layout, dtype, seed=S + d + 1)


@pytest.mark.parametrize("layout", [sa.CONTIGUOUS, sa.STRIPED])
def test_backward_driver(layout):
    _check(1, 2, 128, 64, 4, layout, torch.float32, seed=3, use_driver=True)


def test_bwd_preprocess_matches_rowsum():
    o = inputs.gaussian((2, 2, 100, 64), 7).cuda()
    g = inputs.gaussian((2, 2, 100, 64), 8, torch.bfloat16).cuda()
    delta = torch.empty(2, 2, 100, device="cuda")
    sa.sa_bwd_preprocess(o, g, delta, sa.shard_shape(g, 100, delta))
    want = (inputs.to_f64(o) * inputs.to_f64(g)).sum(-1)
    assert hp.max_abs_err(delta.cpu().numpy(), want) <= 1e-4


@pytest.mark.parametrize("layout", [sa.CONTIGUOUS, sa.STRIPED])
@pytest.mark.parametrize("B,H,S,N", [
    (1, 2, 512, 4),      # c = 128
    (2, 1, 1024, 2),     # c = 512: tiles before, on and after the diagonal
    (1, 1, 1152, 3),     # c = 384
    (1, 2, 768, 1),      # N = 1
])
def test_mfma_bf16_backward(layout, B, H, S, N):
    _check(B, H, S, 128, N, layout, torch.bfloat16, seed=S + N + 5, use_driver=(N != 2))


@pytest.mark.parametrize("layout", [sa.CONTIGUOUS, sa.STRIPED])
@pytest.mark.parametrize("d", [100, 64, 72, 4, 124, 112, 116])
def test_mfma_bf16_backward_padded_head_dimension(layout, d):
    _check(1, 2, 768, d, 3, layout, torch.bfloat16, seed=2000 + d, use_driver=True)


def test_mfma_backward_is_deterministic():
    B, H, S, d, N = 1, 2, 1024, 128, 2
    Q, K, V, dO = (x.cuda() for x in inputs.qkv(B, H, S, d, 32, torch.bfloat16, with_dout=True))
    a = hp.ring_backward_gpu(Q, K, V, dO, N, sa.STRIPED, use_driver=True)
    b = hp.ring_backward_gpu(Q, K, V, dO, N, sa.STRIPED, use_driver=True)
    torch.cuda.synchronize()
    for x, y in zip(a, b):
        assert torch.equal(x, y)


@pytest.mark.parametrize("layout", [sa.CONTIGUOUS, sa.STRIPED])
@pytest.mark.parametrize("B,H,S,d,N", [
    (1, 2, 768, 256, 3),      # two 128-column halves, c = 256
    (2, 1, 1024, 256, 2),     # c = 512: tiles before, on and after the diagonal
    (1, 2, 768, 192, 3),      # second half padded
    (1, 1, 600, 256, 2),      # c = 300: ragged block
    (1, 2, 512, 136, 2),      # one chunk into the second half
])
def test_mfma_bf16_backward_head_dimension_above_128(layout, B, H, S, d, N):
    _check(B, H, S, d, N, layout, torch.bfloat16, seed=3000 + d + S, use_driver=True)
