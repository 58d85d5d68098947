"""GPU parity at the full benchmark sizes, in the launch configuration bench.py
times (ring driver, one device's share or the whole ring), on sampled outputs
the fp64 oracle computes one row at a time from the unpermuted inputs.

Forward: sampled rows of O and LSE.  Backward: dO is zero outside a sampled row
set R, so dQ is exactly zero outside R and dK/dV are the sums over R alone,
which the oracle computes from those rows; every K/V shard is still touched.
"""
import numpy as np
import pytest
import torch

from oracle import striped_attention as orc
from paper_2311_09431_amd import binding as sa
from paper_2311_09431_amd import inputs

pytestmark = pytest.mark.gpu

TOL_O, TOL_LSE = 2e-2, 1e-3


def _device_order(xs, N, layout):
    if layout == sa.CONTIGUOUS:
        return xs
    out = []
    for x in xs:
        y = torch.empty_like(x)
        sa.sa_stripe_permute(x, y, N)
        out.append(y)
    return out


def _global_pos(layout, dev, a, N, c):
    return a * N + dev if layout == sa.STRIPED else dev * c + a


def _local_rows(c, extra_seed):
    fixed = [0, 1, 31, 32, 127, 128, c // 2 - 1, c // 2, c - 129, c - 2, c - 1]
    rnd = np.random.default_rng(extra_seed).integers(0, c, 6).tolist()
    return sorted(set(fixed + rnd))


def _head_f64(x, h):
    return x[0, h].to("cpu").to(torch.float64).numpy()


@pytest.mark.parametrize("layout", [sa.STRIPED, sa.CONTIGUOUS])
def test_one_devices_share_at_256k_forward(layout):
    # seq 262144, N = 8 (32768-token shards), 32 heads, d = 128, bf16: all 8 steps of q_dev 7
    B, H, S, d, N, q_dev = 1, 32, 262144, 128, 8, 7
    c = S // N
    Q, K, V = inputs.qkv(B, H, S, d, 3, torch.bfloat16, device="cuda")
    Qp, Kp, Vp = _device_order([Q, K, V], N, layout)
    O = torch.empty(B, H, S, d, dtype=torch.float32, device="cuda")
    LSE = torch.empty(B, H, S, dtype=torch.float32, device="cuda")
    shape = sa.shard_shape(Qp, c, LSE)
    sa.sa_ring_fwd(Qp, Kp, Vp, O, LSE, N, layout, shape, q_dev_only=q_dev)
    torch.cuda.synchronize()
    rows = _local_rows(c, 11)
    scale = 1.0 / np.sqrt(d)
    for h in (0, H - 1):
        Qh, Kh, Vh = (_head_f64(x, h) for x in (Q, K, V))
        pos = [_global_pos(layout, q_dev, a, N, c) for a in rows]
        Ow, Lw = orc.causal_attention_rows(Qh, Kh, Vh, scale, pos)
        idx = torch.tensor([q_dev * c + a for a in rows], device="cuda")
        Og = O[0, h].index_select(0, idx).cpu().numpy()
        Lg = LSE[0, h].index_select(0, idx).cpu().numpy()
        assert np.isfinite(Og).all()
        assert np.abs(Og - Ow).max() <= TOL_O, (h, np.abs(Og - Ow).max())
        assert np.abs(Lg - Lw).max() <= TOL_LSE, (h, np.abs(Lg - Lw).max())


@pytest.mark.parametrize("layout", [sa.STRIPED, sa.CONTIGUOUS])
def test_forward_ring_sim_32k(layout):
    # seq 32768, N = 8 (4096-token shards), 16 heads: all 64 steps
    B, H, S, d, N = 1, 16, 32768, 128, 8
    c = S // N
    Q, K, V = inputs.qkv(B, H, S, d, 2, torch.bfloat16, device="cuda")
    Qp, Kp, Vp = _device_order([Q, K, V], N, layout)
    O = torch.empty(B, H, S, d, dtype=torch.float32, device="cuda")
    LSE = torch.empty(B, H, S, dtype=torch.float32, device="cuda")
    sa.sa_ring_fwd(Qp, Kp, Vp, O, LSE, N, layout, sa.shard_shape(Qp, c, LSE))
    torch.cuda.synchronize()
    assert torch.isfinite(LSE).all() and torch.isfinite(O).all()
    scale = 1.0 / np.sqrt(d)
    h = 5
    Qh, Kh, Vh = (_head_f64(x, h) for x in (Q, K, V))
    picks = [(dev, a) for dev in range(N) for a in (0, 1, 2047, 4095)] + [(3, 100), (6, 3000)]
    pos = [_global_pos(layout, dev, a, N, c) for dev, a in picks]
    Ow, Lw = orc.causal_attention_rows(Qh, Kh, Vh, scale, pos)
    idx = torch.tensor([dev * c + a for dev, a in picks], device="cuda")
    Og = O[0, h].index_select(0, idx).cpu().numpy()
    Lg = LSE[0, h].index_select(0, idx).cpu().numpy()
    assert np.abs(Og - Ow).max() <= TOL_O
    assert np.abs(Lg - Lw).max() <= TOL_LSE


def _sparse_dout(B, H, S, d, rows, seed):
    """dO that is N(0,1) on `rows` (positions in the ORIGINAL order) and zero elsewhere."""
    g = torch.zeros(B, H, S, d, dtype=torch.bfloat16, device="cuda")
    vals = inputs.gaussian((B, H, len(rows), d), seed, torch.bfloat16, device="cuda")
    g[:, :, torch.tensor(rows, device="cuda")] = vals
    return g


def _check_grads(name, got, want):
    tol = 2e-2 * max(1.0, float(np.abs(want).max()))
    err = float(np.abs(got - want).max())
    assert np.isfinite(got).all() and err <= tol, (name, err, tol)


@pytest.mark.parametrize("layout", [sa.STRIPED, sa.CONTIGUOUS])
def test_backward_131k_row_subsample(layout):
    # seq 131072, N = 8 (16384-token shards), 16 heads, bf16, saved LSE from the forward
    # ring; all 64 backward steps with dO restricted to a sampled row set R
    B, H, S, d, N = 1, 16, 131072, 128, 8
    c = S // N
    Q, K, V = inputs.qkv(B, H, S, d, 4, torch.bfloat16, device="cuda")
    r = np.random.default_rng(4)
    R = sorted(set([0, 1, c - 1, c, S // 2, S - c, S - 2, S - 1] + r.integers(0, S, 88).tolist()))
    dO = _sparse_dout(B, H, S, d, R, 44)
    Qp, Kp, Vp, dOp = _device_order([Q, K, V, dO], N, layout)
    O = torch.empty(B, H, S, d, dtype=torch.float32, device="cuda")
    LSE = torch.empty(B, H, S, dtype=torch.float32, device="cuda")
    shape = sa.shard_shape(Qp, c, LSE)
    sa.sa_ring_fwd(Qp, Kp, Vp, O, LSE, N, layout, shape)
    delta = torch.empty_like(LSE)
    dQ, dK, dV = (torch.empty_like(O) for _ in range(3))
    sa.sa_ring_bwd(Qp, Kp, Vp, dOp, O, LSE, delta, dQ, dK, dV, N, layout, shape)
    torch.cuda.synchronize()
    scale = 1.0 / np.sqrt(d)
    h = 9
    want = orc.causal_attention_grad(*(_head_f64(x, h) for x in (Q, K, V, dO)), scale, rows=R)
    for name, g, w in zip(("dQ", "dK", "dV"), (dQ, dK, dV), want):
        gh = g[0, h].cpu().numpy()
        if layout == sa.STRIPED:
            gh = orc.unstripe_permute(gh, N, 0)
        _check_grads(name, gh, w)
        if name == "dQ":
            outside = np.ones(S, bool)
            outside[R] = False
            assert np.all(gh[outside] == 0.0)        # dO = 0 there, so every term vanishes exactly


@pytest.mark.parametrize("layout", [sa.STRIPED, sa.CONTIGUOUS])
def test_one_devices_share_at_786k_forward_and_backward(layout):
    # seq 786432, N = 16 (49152-token shards), 8 heads: the 16 forward and 16 backward steps of
    # q_dev 15; dO restricted to sampled rows of that device
    B, H, S, d, N, q_dev = 1, 8, 786432, 128, 16, 15
    c = S // N
    Q, K, V = inputs.qkv(B, H, S, d, 5, torch.bfloat16, device="cuda")
    rows = _local_rows(c, 12)
    R = [_global_pos(layout, q_dev, a, N, c) for a in rows]
    dO = _sparse_dout(B, H, S, d, R, 55)
    Qp, Kp, Vp, dOp = _device_order([Q, K, V, dO], N, layout)
    O = torch.empty(B, H, S, d, dtype=torch.float32, device="cuda")
    LSE = torch.empty(B, H, S, dtype=torch.float32, device="cuda")
    shape = sa.shard_shape(Qp, c, LSE)
    sa.sa_ring_fwd(Qp, Kp, Vp, O, LSE, N, layout, shape, q_dev_only=q_dev)
    delta = torch.empty_like(LSE)
    dQ, dK, dV = (torch.empty_like(O) for _ in range(3))
    sa.sa_ring_bwd(Qp, Kp, Vp, dOp, O, LSE, delta, dQ, dK, dV, N, layout, shape, q_dev_only=q_dev)
    torch.cuda.synchronize()
    scale = 1.0 / np.sqrt(d)
    h = 3
    Qh, Kh, Vh, Gh = (_head_f64(x, h) for x in (Q, K, V, dO))
    Ow, Lw = orc.causal_attention_rows(Qh, Kh, Vh, scale, R)
    idx = torch.tensor([q_dev * c + a for a in rows], device="cuda")
    assert np.abs(O[0, h].index_select(0, idx).cpu().numpy() - Ow).max() <= TOL_O
    assert np.abs(LSE[0, h].index_select(0, idx).cpu().numpy() - Lw).max() <= TOL_LSE
    want = orc.causal_attention_grad(Qh, Kh, Vh, Gh, scale, rows=R)
    for name, g, w in zip(("dQ", "dK", "dV"), (dQ, dK, dV), want):
        gh = g[0, h].cpu().numpy()
        if layout == sa.STRIPED:
            gh = orc.unstripe_permute(gh, N, 0)
        _check_grads(name, gh, w)


@pytest.mark.parametrize("layout", [sa.STRIPED, sa.CONTIGUOUS])
def test_head_count_not_a_multiple_of_the_head_group(layout):
    # 10 heads x 64 query tiles = 640 workgroups: the large-grid order with a partial last
    # group of heads; batch 2 exercises the batch stride.  Forward and backward, sampled rows.
    B, H, S, d, N = 2, 5, 16384, 128, 2
    c = S // N
    Q, K, V = inputs.qkv(B, H, S, d, 6, torch.bfloat16, device="cuda")
    R = sorted(set([0, 1, 127, 128, c - 1, c, S - 1] + np.random.default_rng(6).integers(0, S, 25).tolist()))
    dO = _sparse_dout(B, H, S, d, R, 66)
    Qp, Kp, Vp, dOp = _device_order([Q, K, V, dO], N, layout)
    O = torch.empty(B, H, S, d, dtype=torch.float32, device="cuda")
    LSE = torch.empty(B, H, S, dtype=torch.float32, device="cuda")
    shape = sa.shard_shape(Qp, c, LSE)
    sa.sa_ring_fwd(Qp, Kp, Vp, O, LSE, N, layout, shape)
    delta = torch.empty_like(LSE)
    dQ, dK, dV = (torch.empty_like(O) for _ in range(3))
    sa.sa_ring_bwd(Qp, Kp, Vp, dOp, O, LSE, delta, dQ, dK, dV, N, layout, shape)
    torch.cuda.synchronize()
    scale = 1.0 / np.sqrt(d)
    un = (lambda x: orc.unstripe_permute(x, N, 0)) if layout == sa.STRIPED else (lambda x: x)
    for b, h in ((0, 0), (1, 4), (1, 2)):
        f64 = lambda x: x[b, h].to("cpu").to(torch.float64).numpy()
        Qh, Kh, Vh, Gh = f64(Q), f64(K), f64(V), f64(dO)
        Ow, Lw = orc.causal_attention_rows(Qh, Kh, Vh, scale, R)
        assert np.abs(un(O[b, h].cpu().numpy())[R] - Ow).max() <= TOL_O
        assert np.abs(un(LSE[b, h].cpu().numpy())[R] - Lw).max() <= TOL_LSE
        want = orc.causal_attention_grad(Qh, Kh, Vh, Gh, scale, rows=R)
        for name, g, w in zip(("dQ", "dK", "dV"), (dQ, dK, dV), want):
            _check_grads(name, un(g[b, h].cpu().numpy()), w)
