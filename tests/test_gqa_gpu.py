"""GPU parity of the ring steps with fewer key/value heads than query heads (grouped-query
and multi-query attention) against the fp64 oracle, forward and backward, on the generic
and the matrix-core kernels, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import striped_attention as orc
from paper_2311_09431_amd import binding as sa
from paper_2311_09431_amd import inputs
from tests import helpers as hp

pytestmark = pytest.mark.gpu

TOL_FWD = {torch.float32: (1e-5, 1e-5), torch.bfloat16: (2e-2, 1e-3)}


def _inputs(B, H, H_kv, S, d, seed, dtype):
    Q = inputs.gaussian((B, H, S, d), seed * 16, dtype)
    K = inputs.gaussian((B, H_kv, S, d), seed * 16 + 1, dtype)
    V = inputs.gaussian((B, H_kv, S, d), seed * 16 + 2, dtype)
    dO = inputs.gaussian((B, H, S, d), seed * 16 + 3, dtype)
    return Q, K, V, dO


def _run(Q, K, V, dO, N, layout, use_driver, seq_major=False):
    """Forward and backward ring on the GPU; everything returned in device order."""
    B, H, S, d = Q.shape
    c = S // N
    dev = [hp.to_device_order(x.cuda(), N, layout) for x in (Q, K, V, dO)]
    if seq_major:   # [B, S, heads, d] storage viewed as [B, heads, S, d]
        dev = [x.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3) for x in dev]
    Qp, Kp, Vp, dOp = dev
    O = torch.empty_like(Qp, dtype=torch.float32)
    LSE = torch.empty(B, H, S, dtype=torch.float32, device="cuda")
    delta = torch.empty_like(LSE)
    dQ = torch.empty_like(O)
    dK, dV = (torch.full_like(Kp, 7.0, dtype=torch.float32) for _ in range(2))
    shape = sa.shard_shape(Qp, c, LSE, None, kv=Kp)
    if use_driver:
        sa.sa_ring_fwd(Qp, Kp, Vp, O, LSE, N, layout, shape)
        sa.sa_ring_bwd(Qp, Kp, Vp, dOp, O, LSE, delta, dQ, dK, dV, N, layout, shape)
    else:
        r = lambda t, i: t[:, :, i * c:]
        for j in range(N):
            sa.sa_state_init(r(O, j), r(LSE, j), shape)
        for _, j, k in orc.ring_schedule(N):
            sa.sa_attn_step_fwd(r(Qp, j), r(Kp, k), r(Vp, k), r(O, j), r(LSE, j), j, k, N, layout, shape)
        dQ.zero_(), dK.zero_(), dV.zero_()
        for j in range(N):
            sa.sa_bwd_preprocess(r(O, j), r(dOp, j), r(delta, j), shape)
        for _, j, k in orc.ring_schedule(N):
            sa.sa_attn_step_bwd(r(Qp, j), r(Kp, k), r(Vp, k), r(dOp, j), r(LSE, j), r(delta, j),
                                r(dQ, j), r(dK, k), r(dV, k), j, k, N, layout, shape)
    torch.cuda.synchronize()
    return O, LSE, dQ, dK, dV


def _check(B, H, H_kv, S, d, N, layout, dtype, seed, use_driver=True, seq_major=False):
    Q, K, V, dO = _inputs(B, H, H_kv, S, d, seed, dtype)
    got = _run(Q, K, V, dO, N, layout, use_driver, seq_major)
    O, LSE, dQ, dK, dV = (hp.from_device_order_host(x.cpu().numpy(), N, layout) for x in got)
    f = [inputs.to_f64(x) for x in (Q, K, V, dO)]
    sc = 1.0 / np.sqrt(d)
    Ow, Lw = orc.causal_attention_gqa(f[0], f[1], f[2], sc)
    tol_o, tol_l = TOL_FWD[dtype]
    assert hp.max_abs_err(O, Ow) <= tol_o, ("O", hp.max_abs_err(O, Ow))
    assert hp.max_abs_err(LSE, Lw) <= tol_l, ("LSE", hp.max_abs_err(LSE, Lw))
    want = orc.causal_attention_gqa_grad(*f, sc)
    for name, g, w in zip(("dQ", "dK", "dV"), (dQ, dK, dV), want):
        hp.check_grad(name + " " + hp.layout_name(layout), g, w, dtype != torch.float32)


@pytest.mark.parametrize("layout", [sa.CONTIGUOUS, sa.STRIPED])
@pytest.mark.parametrize("B,H,H_kv,S,d,N,dtype", [
    (1, 4, 2, 120, 32, 4, torch.float32),      # ragged c = 30
    (2, 6, 1, 64, 8, 2, torch.float32),        # multi-query: one shared head
    (1, 4, 2, 96, 64, 4, torch.bfloat16),
    (2, 3, 3, 64, 16, 2, torch.float32),       # H_kv = H given explicitly
])
def test_generic_kernels(layout, B, H, H_kv, S, d, N, dtype):
    _check(B, H, H_kv, S, d, N, layout, dtype, seed=H * 7 + H_kv + S)
    _check(B, H, H_kv, S, d, N, layout, dtype, seed=H * 7 + H_kv + S + 1, use_driver=False)


@pytest.mark.parametrize("layout", [sa.CONTIGUOUS, sa.STRIPED])
@pytest.mark.parametrize("B,H,H_kv,S,d,N", [
    (1, 4, 2, 1024, 128, 4),       # c = 256
    (2, 4, 1, 768, 128, 3),        # multi-query, two batches
    (1, 8, 2, 512, 64, 2),         # groups of four, padded head dimension
    (1, 2, 2, 512, 128, 2),        # H_kv = H given explicitly
])
def test_mfma_kernels(layout, B, H, H_kv, S, d, N):
    _check(B, H, H_kv, S, d, N, layout, torch.bfloat16, seed=H + H_kv + S)


@pytest.mark.parametrize("layout", [sa.CONTIGUOUS, sa.STRIPED])
def test_mfma_kernels_step_by_step_and_sequence_major(layout):
    # [B, S, heads, d] storage: Q's rows are H * d apart, K's and V's H_kv * d
    _check(1, 4, 2, 512, 128, 2, layout, torch.bfloat16, seed=91, use_driver=False)
    _check(2, 4, 2, 768, 100, 3, layout, torch.bfloat16, seed=92, seq_major=True)
    _check(1, 4, 1, 96, 32, 4, layout, torch.float32, seed=93, seq_major=True)


def test_grouped_heads_equal_repeated_heads_bit_for_bit():
    # forward and dQ of the matrix-core kernels do the same arithmetic whether a key/value
    # head is shared or stored once per query head
    B, H, H_kv, S, d, N = 1, 4, 2, 1024, 128, 2
    Q, K, V, dO = _inputs(B, H, H_kv, S, d, 5, torch.bfloat16)
    g = H // H_kv
    a = _run(Q, K, V, dO, N, sa.STRIPED, True)
    b = _run(Q, K.repeat_interleave(g, 1), V.repeat_interleave(g, 1), dO, N, sa.STRIPED, True)
    for x, y in zip(a[:3], b[:3]):
        assert torch.equal(x, y)
    for x, y in zip(a[3:], b[3:]):      # shared-head gradients: the members' sum, up to fp32 rounding order
        ysum = y.view(B, H_kv, g, S, d).sum(2)
        assert hp.max_abs_err(x.cpu().numpy(), ysum.cpu().numpy()) <= 1e-4 * float(ysum.abs().max())


def test_argument_errors():
    Q = torch.zeros(1, 4, 128, 64, dtype=torch.bfloat16, device="cuda")
    K = torch.zeros(1, 3, 128, 64, dtype=torch.bfloat16, device="cuda")
    O = torch.zeros(1, 4, 128, 64, device="cuda")
    L = torch.zeros(1, 4, 128, device="cuda")
    shape = sa.shard_shape(Q, 128, L, None, kv=K)        # 3 does not divide 4
    with pytest.raises(sa.StripedAttnError) as e:
        sa.sa_attn_step_fwd(Q, K, K, O, L, 0, 0, 1, sa.STRIPED, shape)
    assert e.value.status == -2
    K2 = torch.zeros(1, 2, 128, 64, dtype=torch.bfloat16, device="cuda")
    shape = sa.shard_shape(Q, 128, L, None, kv=K2)
    shape.kv_stride_h = 64                                # heads would overlap
    with pytest.raises(sa.StripedAttnError) as e:
        sa.sa_attn_step_fwd(Q, K2, K2, O, L, 0, 0, 1, sa.STRIPED, shape)
    assert e.value.status == -2
    shape = sa.shard_shape(Q, 64, L, None, kv=K2[:, :, :64])   # ring extent: K/V hold 64 rows per head
    shape.kv_stride_h = 64 * 64
    with pytest.raises(sa.StripedAttnError) as e:
        sa.sa_ring_fwd(Q, K2, K2, O, L, 2, sa.STRIPED, shape)
    assert e.value.status == -2
