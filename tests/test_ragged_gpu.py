"""Block sizes that are not a multiple of the matrix-core kernels' 128-row tiles (c >= 128):
the last query tile holds rows beyond the shard and the last key tiles keys beyond it.
Forward and backward against the fp64 oracle, both layouts, single steps and drivers."""
import numpy as np
import pytest
import torch

from oracle import striped_attention as orc
from paper_2311_09431_amd import binding as sa
from paper_2311_09431_amd import inputs
from tests import helpers as hp

pytestmark = pytest.mark.gpu


def _check(B, H, H_kv, c, N, d, layout, seed, use_driver=True, seq_major=False, guard=False):
    S = c * N
    Q = inputs.gaussian((B, H, S, d), seed, torch.bfloat16)
    K = inputs.gaussian((B, H_kv, S, d), seed + 1, torch.bfloat16)
    V = inputs.gaussian((B, H_kv, S, d), seed + 2, torch.bfloat16)
    dO = inputs.gaussian((B, H, S, d), seed + 3, torch.bfloat16)
    dev = [hp.to_device_order(x.cuda(), N, layout) for x in (Q, K, V, dO)]
    if seq_major:
        dev = [x.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3) for x in dev]
    Qp, Kp, Vp, Gp = dev
    O = torch.empty_like(Qp, dtype=torch.float32)
    LSE = torch.empty(B, H, S, dtype=torch.float32, device="cuda")
    delta = torch.empty_like(LSE)
    dQ = torch.empty_like(O)
    dK, dV = (torch.empty_like(Kp, dtype=torch.float32) for _ in range(2))
    shape = sa.shard_shape(Qp, c, LSE, None, kv=Kp if H_kv != H else None)
    if use_driver:
        sa.sa_ring_fwd(Qp, Kp, Vp, O, LSE, N, layout, shape)
        sa.sa_ring_bwd(Qp, Kp, Vp, Gp, O, LSE, delta, dQ, dK, dV, N, layout, shape)
    else:
        r = lambda t, i: t[:, :, i * c:]
        for j in range(N):
            sa.sa_state_init(r(O, j), r(LSE, j), shape)
        for _, j, k in orc.ring_schedule(N):
            sa.sa_attn_step_fwd(r(Qp, j), r(Kp, k), r(Vp, k), r(O, j), r(LSE, j), j, k, N, layout, shape)
        dQ.zero_(), dK.zero_(), dV.zero_()
        for j in range(N):
            sa.sa_bwd_preprocess(r(O, j), r(Gp, j), r(delta, j), shape)
        for _, j, k in orc.ring_schedule(N):
            sa.sa_attn_step_bwd(r(Qp, j), r(Kp, k), r(Vp, k), r(Gp, j), r(LSE, j), r(delta, j),
                                r(dQ, j), r(dK, k), r(dV, k), j, k, N, layout, shape)
    torch.cuda.synchronize()
    back = lambda t: hp.from_device_order_host(t.cpu().numpy(), N, layout)
    f = [inputs.to_f64(x) for x in (Q, K, V, dO)]
    sc = 1.0 / np.sqrt(d)
    Ow, Lw = orc.causal_attention_gqa(f[0], f[1], f[2], sc)
    assert np.isfinite(back(O)).all()
    assert hp.max_abs_err(back(O), Ow) <= 2e-2
    assert hp.max_abs_err(back(LSE), Lw) <= 1e-3
    for name, g, w in zip(("dQ", "dK", "dV"), (dQ, dK, dV), orc.causal_attention_gqa_grad(*f, sc)):
        hp.check_grad(name, back(g), w, True)


@pytest.mark.parametrize("layout", [sa.CONTIGUOUS, sa.STRIPED])
@pytest.mark.parametrize("c,N", [(129, 2), (200, 3), (255, 2), (130, 1), (1000, 2), (321, 4)])
def test_ragged_block_sizes_on_the_matrix_core_kernels(layout, c, N):
    _check(1, 2, 2, c, N, 128, layout, seed=c + N)


@pytest.mark.parametrize("layout", [sa.CONTIGUOUS, sa.STRIPED])
def test_ragged_with_everything_else(layout):
    # two batches, shared key/value heads, padded head dimension, both memory orders, single steps
    _check(2, 4, 2, 200, 2, 100, layout, seed=11, use_driver=False)
    _check(2, 4, 1, 333, 2, 64, layout, seed=12, seq_major=True)
    _check(1, 3, 3, 192, 3, 128, layout, seed=13, seq_major=True, use_driver=False)


def test_rows_beyond_the_shard_are_left_alone():
    # a shard of c = 200 rows inside tensors of 256 rows: rows 200..255 of every output keep
    # their contents (the last query / key tile covers them, nothing may be stored there)
    B, H, c, d = 1, 2, 200, 128
    full = [inputs.gaussian((B, H, 256, d), 70 + i, torch.bfloat16).cuda() for i in range(4)]
    Q, K, V, dO = full
    O = torch.full((B, H, 256, d), 7.0, device="cuda")
    LSE = torch.full((B, H, 256), 7.0, device="cuda")
    delta = torch.full((B, H, 256), 7.0, device="cuda")
    grads = [torch.full((B, H, 256, d), 7.0, device="cuda") for _ in range(3)]
    shape = sa.shard_shape(Q, c, LSE)
    for layout in (sa.STRIPED, sa.CONTIGUOUS):
        sa.sa_state_init(O, LSE, shape)
        sa.sa_attn_step_fwd(Q, K, V, O, LSE, 1, 0, 2, layout, shape)     # triangular / full
        sa.sa_bwd_preprocess(O, dO, delta, shape)
        sa.sa_attn_step_bwd(Q, K, V, dO, LSE, delta, *grads, 1, 0, 2, layout, shape)
        torch.cuda.synchronize()
        for t in (O, *grads):
            assert torch.all(t[:, :, c:] == 7.0) and torch.isfinite(t[:, :, :c]).all()
        assert torch.all(LSE[:, :, c:] == 7.0) and torch.all(delta[:, :, c:] == 7.0)
