"""Memory orders other than [B, H, rows, d]: the ABI takes batch, head and row strides, so a
[B, rows, H, d] tensor (heads interleaved within a row step, the usual order of attention
inputs) goes through unchanged.  Same oracle, same tolerances as the contiguous cases."""
import numpy as np
import pytest
import torch

from paper_2311_09431_amd import binding as sa
from paper_2311_09431_amd import inputs
from tests import helpers as hp

pytestmark = pytest.mark.gpu


def _seq_major(x):
    """[B, H, S, d] values stored as [B, S, H, d]; returns (storage, [B, H, S, d] view)."""
    store = x.permute(0, 2, 1, 3).contiguous()
    return store, store.permute(0, 2, 1, 3)


def _empty_like_view(B, H, S, d, dtype):
    store = torch.empty(B, S, H, d, dtype=dtype, device="cuda")
    return store, store.permute(0, 2, 1, 3)


@pytest.mark.parametrize("layout", [sa.CONTIGUOUS, sa.STRIPED])
@pytest.mark.parametrize("B,H,S,d,N,dtype,use_driver", [
    (2, 3, 1024, 128, 4, torch.bfloat16, True),    # matrix-core kernels, row pitch 3 * 256 bytes
    (1, 2, 768, 100, 3, torch.bfloat16, False),    # padded head dimension and a row pitch
    (2, 2, 120, 32, 4, torch.float32, True),       # generic kernels
])
def test_seq_major_forward_and_backward(layout, B, H, S, d, N, dtype, use_driver):
    c = S // N
    Q, K, V, dO = (x.cuda() for x in inputs.qkv(B, H, S, d, S + d + N, dtype, with_dout=True))
    stores, views = [], []
    for x in (Q, K, V, dO):
        st, _ = _seq_major(x)
        if layout == sa.STRIPED:                    # permute along the sequence axis of [B, S, H, d]
            dst = torch.empty_like(st)
            sa.sa_stripe_permute(st, dst, N, seq_axis=1)
            st = dst
        stores.append(st)
        views.append(st.permute(0, 2, 1, 3))
    Qv, Kv, Vv, Gv = views
    _, O = _empty_like_view(B, H, S, d, torch.float32)
    LSE = torch.empty(B, H, S, dtype=torch.float32, device="cuda")
    delta = torch.empty_like(LSE)
    grads = [_empty_like_view(B, H, S, d, torch.float32)[1] for _ in range(3)]
    shape = sa.shard_shape(Qv, c, LSE)
    assert shape.stride_h == d and shape.stride_s == H * d
    if use_driver:
        sa.sa_ring_fwd(Qv, Kv, Vv, O, LSE, N, layout, shape)
        sa.sa_ring_bwd(Qv, Kv, Vv, Gv, O, LSE, delta, *grads, N, layout, shape)
    else:
        r = lambda t, dev: t[:, :, dev * c:]
        for j in range(N):
            sa.sa_state_init(r(O, j), r(LSE, j), shape)
        for j in range(N):
            for k in range(N):
                sa.sa_attn_step_fwd(r(Qv, j), r(Kv, k), r(Vv, k), r(O, j), r(LSE, j), j, k, N, layout, shape)
        for g in grads:
            g.zero_()
        for j in range(N):
            sa.sa_bwd_preprocess(r(O, j), r(Gv, j), r(delta, j), shape)
        for j in range(N):
            for k in range(N):
                sa.sa_attn_step_bwd(r(Qv, j), r(Kv, k), r(Vv, k), r(Gv, j), r(LSE, j), r(delta, j),
                                    r(grads[0], j), r(grads[1], k), r(grads[2], k), j, k, N, layout, shape)
    out_store, out = _empty_like_view(B, H, S, d, dtype)
    for j in range(N):
        sa.sa_finalize(O[:, :, j * c:], out[:, :, j * c:], shape)
    torch.cuda.synchronize()

    scale = 1.0 / np.sqrt(d)
    Oref, Lref = hp.oracle_forward(Q, K, V, scale)
    gref = hp.oracle_backward(Q, K, V, dO, scale)
    back = lambda t: hp.from_device_order_host(t.contiguous().cpu().float().numpy(), N, layout)
    bf16 = dtype == torch.bfloat16
    assert hp.max_abs_err(back(O), Oref) <= (2e-2 if bf16 else 1e-5)
    assert hp.max_abs_err(hp.from_device_order_host(LSE.cpu().numpy(), N, layout), Lref) <= (1e-3 if bf16 else 1e-5)
    assert hp.max_abs_err(back(out), Oref) <= (3e-2 if bf16 else 1e-5)      # one more bf16 rounding
    for g, w in zip(grads, gref):
        hp.check_grad("gradient", back(g), w, bf16)


def test_rows_that_overlap_are_rejected():
    x = torch.zeros(1, 256, 2, 128, dtype=torch.bfloat16, device="cuda")
    lse = torch.zeros(1, 2, 256, device="cuda")
    o = torch.zeros(1, 256, 2, 128, device="cuda")
    good = sa.shard_shape(x.permute(0, 2, 1, 3), 128, lse)
    for field, value in [("stride_s", 64), ("stride_s", 130), ("stride_h", 64), ("stride_s", 200)]:
        bad = sa.SaShape.from_buffer_copy(good)
        setattr(bad, field, value)
        with pytest.raises(sa.StripedAttnError) as e:
            sa.sa_state_init(o.permute(0, 2, 1, 3), lse, bad)
        assert e.value.status in (-2, -6)


@pytest.mark.parametrize("layout", [sa.CONTIGUOUS, sa.STRIPED])
@pytest.mark.parametrize("d,pitch", [(100, 128), (64, 128), (36, 40), (124, 136), (192, 256), (136, 144)])
def test_gap_between_rows_may_hold_anything(layout, d, pitch):
    # Rows of d elements at a pitch of more than d, the gap filled with NaN (what an
    # uninitialised buffer may hold): the matrix-core kernels compute 64, 112, 128 or 256 columns
    # and must neither read the gap into a product nor write into it.
    B, H, S, N = 1, 2, 768, 3
    c = S // N
    Q, K, V, dO = (x.cuda() for x in inputs.qkv(B, H, S, d, 900 + d, torch.bfloat16, with_dout=True))

    def padded(x, dtype, fill):
        store = torch.full((B, H, S, pitch), fill, dtype=dtype, device="cuda")
        view = store[..., :d]
        if x is not None:
            view.copy_(x)
        return store, view

    ins = []
    for x in (Q, K, V, dO):
        if layout == sa.STRIPED:
            y = torch.empty_like(x)
            sa.sa_stripe_permute(x, y, N)
            x = y
        ins.append(padded(x, torch.bfloat16, float("nan"))[1])
    Qv, Kv, Vv, Gv = ins
    O_store, O = padded(None, torch.float32, float("nan"))
    LSE = torch.empty(B, H, S, dtype=torch.float32, device="cuda")
    delta = torch.empty_like(LSE)
    g_stores, grads = zip(*(padded(None, torch.float32, float("nan")) for _ in range(3)))
    shape = sa.shard_shape(Qv, c, LSE)
    assert shape.stride_s == pitch
    sa.sa_ring_fwd(Qv, Kv, Vv, O, LSE, N, layout, shape)
    sa.sa_ring_bwd(Qv, Kv, Vv, Gv, O, LSE, delta, *grads, N, layout, shape)
    torch.cuda.synchronize()
    for st in (O_store,) + tuple(g_stores):
        assert bool(torch.isnan(st[..., d:]).all())          # the gap is left alone
    scale = 1.0 / np.sqrt(d)
    Oref, Lref = hp.oracle_forward(Q, K, V, scale)
    back = lambda t: hp.from_device_order_host(t.contiguous().cpu().float().numpy(), N, layout)
    assert hp.max_abs_err(back(O), Oref) <= 2e-2
    assert hp.max_abs_err(hp.from_device_order_host(LSE.cpu().numpy(), N, layout), Lref) <= 1e-3
    for g, w in zip(grads, hp.oracle_backward(Q, K, V, dO, scale)):
        hp.check_grad("gradient", back(g), w, True)
