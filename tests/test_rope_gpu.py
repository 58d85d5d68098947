"""Rotary embedding with explicit position ids on the GPU, and the paper's remark about it
(Sec. 2.3): permute the position ids with the tokens and every token is embedded as before."""
import numpy as np
import pytest
import torch

from oracle import striped_attention as orc
from paper_2311_09431_amd import binding as sa
from paper_2311_09431_amd import inputs
from tests import helpers as hp

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("B,H,S,d,per_batch", [(2, 3, 64, 128, False), (2, 2, 50, 100, True), (1, 1, 7, 4, False)])
def test_rope_matches_the_oracle(dtype, B, H, S, d, per_batch):
    x = inputs.gaussian((B, H, S, d), 5, dtype).cuda()
    rng = np.random.default_rng(S)
    ids = rng.integers(0, 786432, size=(B, S) if per_batch else (S,)).astype(np.int32)
    ids.flat[0] = 786431                                  # the largest position of the workloads
    pos = torch.from_numpy(ids).cuda()
    y = torch.empty_like(x)
    shape = sa.shard_shape(x, S)
    sa.sa_rope(x, y, pos, shape)
    want = orc.rope(inputs.to_f64(x), ids[:, None, :] if per_batch else ids)
    tol = 1e-6 if dtype == torch.float32 else 2 ** -8      # one rounding of values of size <= 4
    assert hp.max_abs_err(y.cpu().float().numpy(), want) <= tol * max(1.0, float(np.abs(want).max()))
    # inverse = transpose, in place
    sa.sa_rope(y, y, pos, shape, inverse=True)
    assert hp.max_abs_err(y.cpu().float().numpy(), inputs.to_f64(x)) <= 2 * tol * max(1.0, float(np.abs(want).max()))


def test_rope_on_a_sequence_major_tensor():
    B, H, S, d = 2, 3, 40, 64
    x = inputs.gaussian((B, H, S, d), 9, torch.bfloat16).cuda()
    store = x.permute(0, 2, 1, 3).contiguous()
    view = store.permute(0, 2, 1, 3)
    pos = torch.arange(S, dtype=torch.int32, device="cuda") * 1000
    y = torch.empty_like(x)
    sa.sa_rope(x, y, pos, sa.shard_shape(x, S))
    sa.sa_rope(view, view, pos, sa.shard_shape(view, S))
    torch.cuda.synchronize()
    assert torch.equal(view.contiguous(), y)


@pytest.mark.parametrize("N", [2, 4, 8])
def test_permuting_the_position_ids_with_the_tokens(N):
    # rope in the striped layout with ids permuted by the same kernel == stripe(rope(original))
    B, H, S, d = 1, 2, 256, 128
    x = inputs.gaussian((B, H, S, d), 3, torch.bfloat16).cuda()
    ids = torch.arange(S, dtype=torch.int32, device="cuda")
    ids_p = torch.empty_like(ids)
    sa.sa_stripe_permute(ids, ids_p, N, seq_axis=0)
    c = S // N
    assert ids_p.view(N, c).cpu().tolist() == [[a * N + dev for a in range(c)] for dev in range(N)]
    shape = sa.shard_shape(x, S)
    a = torch.empty_like(x)
    sa.sa_rope(x, a, ids, shape)
    a_p = torch.empty_like(x)
    sa.sa_stripe_permute(a, a_p, N)
    x_p = torch.empty_like(x)
    sa.sa_stripe_permute(x, x_p, N)
    b_p = torch.empty_like(x)
    sa.sa_rope(x_p, b_p, ids_p, shape)
    torch.cuda.synchronize()
    assert torch.equal(a_p, b_p)


def test_striped_ring_attention_on_rotated_inputs():
    # the whole path: permute tokens and ids, rotate Q and K shard-wise, ring attention,
    # un-permute; against the oracle's attention on rotated inputs in the original order
    B, H, S, d, N = 1, 2, 1024, 128, 4
    c = S // N
    Q, K, V = (t.cuda() for t in inputs.qkv(B, H, S, d, 77, torch.bfloat16))
    ids = torch.arange(S, dtype=torch.int32, device="cuda")
    ids_p = torch.empty_like(ids)
    sa.sa_stripe_permute(ids, ids_p, N, seq_axis=0)
    Qp, Kp, Vp = (hp.to_device_order(t, N, sa.STRIPED) for t in (Q, K, V))
    LSE = torch.empty(B, H, S, dtype=torch.float32, device="cuda")
    O = torch.empty(B, H, S, d, dtype=torch.float32, device="cuda")
    shard = sa.shard_shape(Qp, c, LSE)
    for dev in range(N):                                   # each device rotates its own shard
        for t in (Qp, Kp):
            sa.sa_rope(t[:, :, dev * c:], t[:, :, dev * c:], ids_p[dev * c:(dev + 1) * c], shard)
    sa.sa_ring_fwd(Qp, Kp, Vp, O, LSE, N, sa.STRIPED, shard)
    torch.cuda.synchronize()
    # the oracle consumes the SAME rotated bf16 bits (un-permuted on the host), so the
    # comparison isolates the attention; the rotation itself is checked above
    Qr = orc.unstripe_permute(inputs.to_f64(Qp), N, 2)
    Kr = orc.unstripe_permute(inputs.to_f64(Kp), N, 2)
    scale = 1.0 / np.sqrt(d)
    Ow, Lw = orc.causal_attention_bh(Qr, Kr, inputs.to_f64(V), scale)
    assert hp.max_abs_err(orc.unstripe_permute(O.cpu().numpy(), N, 2), Ow) <= 2e-2
    assert hp.max_abs_err(orc.unstripe_permute(LSE.cpu().numpy(), N, 2), Lw) <= 1e-3
    # and the rotated bits are what the oracle's rope gives for the original order
    want_q = orc.rope(inputs.to_f64(Q), np.arange(S))
    assert hp.max_abs_err(Qr, want_q) <= 2 ** -8 * max(1.0, float(np.abs(want_q).max()))


@pytest.mark.parametrize("layout", [sa.CONTIGUOUS, sa.STRIPED])
@pytest.mark.parametrize("d", [128, 64, 256])
def test_query_rotation_fused_into_the_forward_step(layout, d):
    # sa_attn_step_fwd_rope rotates the query rows as it loads them; keys are rotated once per
    # shard by sa_rope.  Against the oracle: rotate in fp64, round the rotated queries to bf16
    # (the precision in which the kernel hands them to the matrix cores), attention on that.
    B, H, S, N = 2, 2, 1024, 4
    c = S // N
    Q, K, V = inputs.qkv(B, H, S, d, 70 + d, torch.bfloat16)
    ids = np.arange(S, dtype=np.int32) * 700 + 3            # positions up to 7 * 10^5
    pos = torch.from_numpy(ids).cuda()
    Qp, Kp, Vp = (hp.to_device_order(x.cuda(), N, layout) for x in (Q, K, V))
    pos_p = pos
    if layout == sa.STRIPED:
        pos_p = torch.empty_like(pos)
        sa.sa_stripe_permute(pos, pos_p, N, seq_axis=0)      # the ids travel with the tokens
    full = sa.shard_shape(Kp, S)
    Kr = torch.empty_like(Kp)
    sa.sa_rope(Kp, Kr, pos_p, full)
    Qr = torch.empty_like(Qp)
    sa.sa_rope(Qp, Qr, pos_p, full)
    outs = []
    for fused in (True, False):
        O = torch.empty(B, H, S, d, dtype=torch.float32, device="cuda")
        LSE = torch.empty(B, H, S, dtype=torch.float32, device="cuda")
        shape = sa.shard_shape(Qp, c, LSE)
        r = lambda t, dev: t[:, :, dev * c:]
        for j in range(N):
            sa.sa_state_init(r(O, j), r(LSE, j), shape)
            for k in range(N):
                if fused:
                    sa.sa_attn_step_fwd_rope(r(Qp, j), r(Kr, k), r(Vp, k), r(O, j), r(LSE, j),
                                             pos_p[j * c:(j + 1) * c], j, k, N, layout, shape)
                else:
                    sa.sa_attn_step_fwd(r(Qr, j), r(Kr, k), r(Vp, k), r(O, j), r(LSE, j), j, k, N, layout, shape)
        outs.append((O, LSE))
    torch.cuda.synchronize()
    scale = 1.0 / np.sqrt(d)
    q_rot = torch.from_numpy(orc.rope(inputs.to_f64(Q), ids)).to(torch.bfloat16)
    k_rot = hp.from_device_order_host(inputs.to_f64(Kr), N, layout)       # the bits the kernel read
    Ow, Lw = orc.causal_attention_bh(inputs.to_f64(q_rot), k_rot, inputs.to_f64(V), scale)
    for O, LSE in outs:
        assert hp.max_abs_err(hp.from_device_order_host(O.cpu().numpy(), N, layout), Ow) <= 2e-2
        assert hp.max_abs_err(hp.from_device_order_host(LSE.cpu().numpy(), N, layout), Lw) <= 1e-3
    # fused and unfused differ only where the two sine / cosine evaluations round a rotated
    # query to neighbouring bf16 values
    assert hp.max_abs_err(outs[0][0].cpu().numpy(), outs[1][0].cpu().numpy()) <= 2e-3
    assert hp.max_abs_err(outs[0][1].cpu().numpy(), outs[1][1].cpu().numpy()) <= 5e-4


def test_fused_query_rotation_rejects_other_shapes():
    q = torch.zeros(1, 1, 256, 100, dtype=torch.bfloat16, device="cuda")
    o = torch.zeros(1, 1, 256, 100, device="cuda")
    lse = torch.zeros(1, 1, 256, device="cuda")
    pos = torch.zeros(256, dtype=torch.int32, device="cuda")
    with pytest.raises(sa.StripedAttnError) as e:
        sa.sa_attn_step_fwd_rope(q, q, q, o, lse, pos, 0, 0, 1, sa.STRIPED, sa.shard_shape(q, 256, lse))
    assert e.value.status == -2
