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


@pytest.mark.parametrize("d", [128, 100])
@pytest.mark.parametrize("layout", [sa.STRIPED, sa.CONTIGUOUS])
def test_one_devices_share_at_256k_forward(layout, d):
    # seq 262144, N = 8 (32768-token shards), 32 heads, bf16: all 8 steps of q_dev 7, at the head
    # dimension of Table 1's 1B / 7B models (128) and of its 3B model (100)
    B, H, S, N, q_dev = 1, 32, 262144, 8, 7
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


# Gradient criteria.  (i) max abs error <= 2e-2 * max(1, max|want|) per tensor, the forward's
# bf16 bound scaled by the gradient's magnitude.  (ii) ||got - want||_F <= 1e-2 ||want||_F per
# tensor: P and dS are rounded to bf16 (2^-9 relative, about 1e-3 rms) before the fp32-accumulated
# products, so a correct result sits near 2e-3 whatever the gradient's magnitude, and a dropped
# tile or term does not.  (iii) the same per 128-row tile with 2e-2, plus an absolute floor per
# element of a row that carries a gradient: 2e-6 rms for dK and dV (fp32 accumulation), 1e-3 rms
# for dQ, where dS = P (dP - delta) cancels on rows with few keys or one dominant key (row 0:
# exactly zero) and delta carries the forward's bf16 rounding of P (2^-9 of |dP|, against a
# difference that may be a few per cent of it).  Rows whose expected gradient is exactly zero
# (dO = 0 there, or keys no sampled query sees) must be exactly zero.
REL_TENSOR, REL_TILE, ABS_TILE_RMS, ABS_TILE_RMS_DQ = 1e-2, 2e-2, 2e-6, 1e-3


def _check_grads(name, got, want, tile=128, report=None, zero_rows=None):
    got = np.asarray(got, np.float64)
    assert np.isfinite(got).all(), name
    tol = 2e-2 * max(1.0, float(np.abs(want).max()))
    err = float(np.abs(got - want).max())
    assert err <= tol, (name, err, tol)
    rel = float(np.linalg.norm(got - want) / np.linalg.norm(want))
    assert rel <= REL_TENSOR, (name, "relative Frobenius error", rel)
    if zero_rows is not None:
        assert not np.any(want[zero_rows]) and not np.any(got[zero_rows]), (name, "rows that must be exactly zero")
    n, d = got.shape[0] // tile * tile, got.shape[1]
    g, w = got[:n].reshape(-1, tile * d), want[:n].reshape(-1, tile * d)
    num, den = np.linalg.norm(g - w, axis=1), np.linalg.norm(w, axis=1)
    signal_rows = np.any(want[:n] != 0.0, axis=1).reshape(-1, tile).sum(axis=1)
    floor = (ABS_TILE_RMS_DQ if name.startswith("dQ") else ABS_TILE_RMS) * np.sqrt(signal_rows * d)
    bound = REL_TILE * den + floor
    worst = int(np.argmax(num - bound))
    assert num[worst] <= bound[worst], (name, "tile", worst, num[worst], den[worst], bound[worst])
    if report is not None:
        report.append((name, "%.2e" % err, "%.2e" % rel, "%.2e" % float(np.max(num / np.maximum(den, 1e-300)))))


def _chunked_grad(Qh, Kh, Vh, Gh, scale, rows, chunk=512):
    """The oracle's matrix-form gradient summed over chunks of the (sorted) row set: the
    gradient is additive over disjoint sets of query rows."""
    rows = sorted(rows)
    tot = None
    for i in range(0, len(rows), chunk):
        part = orc.causal_attention_grad_matrix(Qh, Kh, Vh, Gh, scale, rows[i:i + chunk])[:3]
        tot = list(part) if tot is None else [t + q for t, q in zip(tot, part)]
    return tot


def test_backward_131k_row_subsample():
    # seq 131072, N = 8 (16384-token shards), 16 heads, bf16, saved LSE from the forward
    # ring; all 64 backward steps with dO restricted to a sampled row set: 4096 rows on the
    # head checked in full (the subsample the configuration names), 512 on the first and the
    # last head, 96 on the others.  One row in eight of a set has its query scaled by 3, so
    # that its softmax concentrates (top probability of a few per cent instead of 1e-5) and
    # key tiles far from the diagonal carry gradients of ordinary magnitude.
    B, H, S, d, N = 1, 16, 131072, 128, 8
    c = S // N
    Q, K, V = inputs.qkv(B, H, S, d, 4, torch.bfloat16, device="cuda")
    r = np.random.default_rng(4)
    base = [0, 1, c - 1, c, S // 2, S - c, S - 2, S - 1]
    n_rows = {0: 512, 9: 4096, H - 1: 512}
    R = {h: sorted(set(base + r.choice(S, n_rows.get(h, 96) - len(base), replace=False).tolist()))
         for h in range(H)}
    dO = torch.zeros(B, H, S, d, dtype=torch.bfloat16, device="cuda")
    for h in range(H):
        idx = torch.tensor(R[h], device="cuda")
        dO[0, h, idx] = inputs.gaussian((len(R[h]), d), 4400 + h, torch.bfloat16, device="cuda")
        sharp = idx[::8]
        Q[0, h, sharp] = (Q[0, h, sharp].float() * 3.0).to(torch.bfloat16)
    scale = 1.0 / np.sqrt(d)
    want = {h: _chunked_grad(*(_head_f64(x, h) for x in (Q, K, V, dO)), scale, R[h]) for h in n_rows}
    report = []
    for layout in (sa.STRIPED, sa.CONTIGUOUS):
        Qp, Kp, Vp, dOp = _device_order([Q, K, V, dO], N, layout)
        O = torch.empty(B, H, S, d, dtype=torch.float32, device="cuda")
        LSE = torch.empty(B, H, S, dtype=torch.float32, device="cuda")
        shape = sa.shard_shape(Qp, c, LSE)
        sa.sa_ring_fwd(Qp, Kp, Vp, O, LSE, N, layout, shape)
        delta = torch.empty_like(LSE)
        dQ, dK, dV = (torch.empty_like(O) for _ in range(3))
        sa.sa_ring_bwd(Qp, Kp, Vp, dOp, O, LSE, delta, dQ, dK, dV, N, layout, shape)
        torch.cuda.synchronize()
        for h in n_rows:
            for name, g, w in zip(("dQ", "dK", "dV"), (dQ, dK, dV), want[h]):
                gh = g[0, h].cpu().numpy()
                if layout == sa.STRIPED:
                    gh = orc.unstripe_permute(gh, N, 0)
                zero = np.ones(S, bool)
                if name == "dQ":
                    zero[R[h]] = False              # dO = 0 outside R: every term vanishes exactly
                else:
                    zero[:R[h][-1] + 1] = False     # no sampled query sees the keys after the last one
                _check_grads("%s head %d layout %d" % (name, h, layout), gh, w, report=report, zero_rows=zero)
        del Qp, Kp, Vp, dOp, O, LSE, dQ, dK, dV
    print("backward 131k subsample (name, max abs err, rel F, worst tile rel):", report)


def _index_in_device_order(pos, N, c, layout):
    pos = np.asarray(pos, np.int64)
    return (pos % N) * c + pos // N if layout == sa.STRIPED else pos


@pytest.mark.parametrize("d", [128, 100])
def test_dense_backward_at_256k_shards(d):
    # The shape bench.py times (32 heads, d = 128, 32768-token shards of a 262144-token
    # sequence, the large-grid workgroup order; and the same at the 3B model's d = 100, the
    # `3b` workload) with a DENSE dO, whole ring and one device's share, both layouts.  Against the oracle: dQ on sampled rows (dQ_i needs row i of dO
    # only) and dK, dV on the keys of the last 512 positions (only the queries at or after a
    # key see it).  Properties that hold for every row: sum_j dV_j = sum_i dO_i and
    # <Q, dQ> = <K, dK> per head, and striped == contiguous after un-permuting (two different
    # tile walks of the same sum).
    B, H, S, N, q_dev = 1, 32, 262144, 8, 7
    c = S // N
    Q, K, V, dO = inputs.qkv(B, H, S, d, 3, torch.bfloat16, device="cuda", with_dout=True)
    scale = 1.0 / np.sqrt(d)
    r = np.random.default_rng(33)
    q_rows = sorted(set([0, 1, 127, 128, c - 1, c, 3 * c + 77, S - c - 1, S - c, S - 129, S - 1]
                        + r.choice(S, 53, replace=False).tolist()))
    tail0 = S - 512
    tail = list(range(tail0, S))
    heads_q, heads_kv = (0, 7, 8, H - 1), (0, H - 1)     # first / last of a group of 8 heads
    want_q, want_tail = {}, {}
    for h in heads_q:
        Qh, Kh, Vh, Gh = (_head_f64(x, h) for x in (Q, K, V, dO))
        want_q[h] = orc.causal_attention_grad_matrix(Qh, Kh, Vh, Gh, scale, q_rows)[0][q_rows]
        if h in heads_kv:
            want_tail[h] = _chunked_grad(Qh, Kh, Vh, Gh, scale, tail, chunk=256)
    sum_dO = dO.double().sum(dim=2)                               # [B, H, d]
    report, unpermuted = [], {}
    for layout in (sa.STRIPED, sa.CONTIGUOUS):
        Qp, Kp, Vp, dOp = _device_order([Q, K, V, dO], N, layout)
        O = torch.empty(B, H, S, d, dtype=torch.float32, device="cuda")
        LSE = torch.empty(B, H, S, dtype=torch.float32, device="cuda")
        shape = sa.shard_shape(Qp, c, LSE)
        sa.sa_ring_fwd(Qp, Kp, Vp, O, LSE, N, layout, shape)
        delta = torch.empty_like(LSE)
        dQ, dK, dV = (torch.empty_like(O) for _ in range(3))
        sa.sa_ring_bwd(Qp, Kp, Vp, dOp, O, LSE, delta, dQ, dK, dV, N, layout, shape)
        torch.cuda.synchronize()
        assert all(bool(torch.isfinite(g).all()) for g in (dQ, dK, dV))
        qi = torch.tensor(_index_in_device_order(q_rows, N, c, layout), device="cuda")
        ti = torch.tensor(_index_in_device_order(tail, N, c, layout), device="cuda")
        for h in heads_q:
            got = dQ[0, h].index_select(0, qi).cpu().numpy()
            _check_grads("dQ rows head %d layout %d" % (h, layout), got, want_q[h], tile=8, report=report)
        for h in heads_kv:
            _, wk, wv = want_tail[h]
            _check_grads("dK tail head %d layout %d" % (h, layout),
                         dK[0, h].index_select(0, ti).cpu().numpy(), wk[tail0:], report=report)
            _check_grads("dV tail head %d layout %d" % (h, layout),
                         dV[0, h].index_select(0, ti).cpu().numpy(), wv[tail0:], report=report)
            # the tail queries' dQ is dense-exact too (every key of theirs is in the product)
            _check_grads("dQ tail head %d layout %d" % (h, layout),
                         dQ[0, h].index_select(0, ti).cpu().numpy(), want_tail[h][0][tail0:], report=report)
        # properties, every head
        col = dV.double().sum(dim=2)
        rel = ((col - sum_dO).norm(dim=-1) / sum_dO.norm(dim=-1)).max().item()
        assert rel <= 5e-3, ("sum_j dV_j = sum_i dO_i", rel)
        for h in range(H):
            qdq = (Qp[0, h].double() * dQ[0, h].double()).sum(dim=1)
            kdk = (Kp[0, h].double() * dK[0, h].double()).sum(dim=1)
            gap = abs(qdq.sum().item() - kdk.sum().item())
            ref = qdq.abs().sum().item()
            assert gap <= 1e-3 * ref, ("<Q,dQ> = <K,dK>", h, gap, ref)
        # one device's share, as bench.py runs it: the same steps for that device
        dQs, dKs, dVs = (torch.empty_like(O) for _ in range(3))
        sa.sa_ring_bwd(Qp, Kp, Vp, dOp, O, LSE, delta, dQs, dKs, dVs, N, layout, shape, q_dev_only=q_dev)
        torch.cuda.synchronize()
        assert torch.equal(dQs[:, :, q_dev * c:(q_dev + 1) * c], dQ[:, :, q_dev * c:(q_dev + 1) * c])
        own = [t for t in tail if (t % N if layout == sa.STRIPED else t // c) == q_dev]
        for h in heads_kv:
            Qh, Kh, Vh, Gh = (_head_f64(x, h) for x in (Q, K, V, dO))
            _, wk, wv = (want_tail[h] if len(own) == len(tail) else
                         _chunked_grad(Qh, Kh, Vh, Gh, scale, own, chunk=256))
            _check_grads("share dK tail head %d layout %d" % (h, layout),
                         dKs[0, h].index_select(0, ti).cpu().numpy(), wk[tail0:], report=report)
            _check_grads("share dV tail head %d layout %d" % (h, layout),
                         dVs[0, h].index_select(0, ti).cpu().numpy(), wv[tail0:], report=report)
        del dQs, dKs, dVs
        if layout == sa.STRIPED:
            outs = []
            for g in (dQ, dK, dV):
                u = torch.empty_like(g)
                sa.sa_unstripe_permute(g, u, N)      # the permutation kernel is bit-exact (its own tests)
                outs.append(u)
            unpermuted[layout] = outs
        else:
            unpermuted[layout] = [dQ, dK, dV]
        del Qp, Kp, Vp, dOp, O, LSE
    torch.cuda.synchronize()
    for name, a, b in zip(("dQ", "dK", "dV"), unpermuted[sa.STRIPED], unpermuted[sa.CONTIGUOUS]):
        blk = 1024
        x = a.view(B, H, S // blk, blk * d).double()
        y = b.view(B, H, S // blk, blk * d).double()
        rel = ((x - y).norm(dim=-1) / y.norm(dim=-1)).max().item()
        report.append((name + " striped vs contiguous, worst 1024-row block", rel))
        assert rel <= 1.5e-2, (name, "striped vs contiguous", rel)
    print("dense backward at 256k (name, max abs err, rel F, worst tile rel):", report)


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
