"""Shared plumbing of the GPU parity tests: seeded inputs -> HIP path through the
C ABI -> host arrays, and the oracle's answer for the same bits."""
import numpy as np
import torch

from oracle import striped_attention as orc
from paper_2311_09431_amd import binding as sa
from paper_2311_09431_amd import inputs


def layout_name(layout):
    return "striped" if layout == sa.STRIPED else "contiguous"


def to_device_order(x, N, layout):
    """[B,H,S,d] GPU tensor in original order -> device order (GPU permute kernel)."""
    if layout == sa.CONTIGUOUS:
        return x
    y = torch.empty_like(x)
    sa.sa_stripe_permute(x, y, N)
    return y


def from_device_order_host(x_np, N, layout, axis=2):
    """Undo the device order on the HOST with the oracle's inverse permutation."""
    return x_np if layout == sa.CONTIGUOUS else orc.unstripe_permute(x_np, N, axis)


def ring_forward_gpu(Q, K, V, N, layout, scale=None, use_driver=False, order=None):
    """Play all N*N steps on the GPU.  Q, K, V: GPU tensors in ORIGINAL order.
    Returns (O fp32, LSE fp32) as GPU tensors in device order."""
    B, H, S, d = Q.shape
    c = S // N
    Qp, Kp, Vp = (to_device_order(x, N, layout) for x in (Q, K, V))
    O = torch.empty(B, H, S, d, dtype=torch.float32, device=Q.device)
    LSE = torch.empty(B, H, S, dtype=torch.float32, device=Q.device)
    shape = sa.shard_shape(Qp, c, LSE, scale)
    if use_driver:
        sa.sa_ring_fwd(Qp, Kp, Vp, O, LSE, N, layout, shape)
        return O, LSE
    for j in range(N):
        sa.sa_state_init(O[:, :, j * c:], LSE[:, :, j * c:], shape)
    pairs = order if order is not None else [(j, k) for _, j, k in orc.ring_schedule(N)]
    for j, k in pairs:
        sa.sa_attn_step_fwd(Qp[:, :, j * c:], Kp[:, :, k * c:], Vp[:, :, k * c:], O[:, :, j * c:],
                            LSE[:, :, j * c:], j, k, N, layout, shape)
    return O, LSE


def oracle_forward(Q, K, V, scale):
    """fp64 causal attention of the bits in Q, K, V (any device/dtype)."""
    return orc.causal_attention_bh(inputs.to_f64(Q), inputs.to_f64(K), inputs.to_f64(V), scale)


def max_abs_err(a, b):
    return float(np.max(np.abs(np.asarray(a, np.float64) - np.asarray(b, np.float64))))


def check_grad(name, got, want, bf16):
    """Gradient criteria shared by the parity tests: max abs error <= 2e-2 (bf16) or 2e-5
    (fp32) times max(1, max|want|), and ||got - want||_F <= 1e-2 (2e-5) ||want||_F, which
    does not loosen with the gradient's magnitude (bf16 rounding of P and dS is about 1e-3
    rms of every term; a dropped tile or term is of order one)."""
    got = np.asarray(got, np.float64)
    assert got.shape == want.shape and np.isfinite(got).all(), name
    err = max_abs_err(got, want)
    assert err <= (2e-2 if bf16 else 2e-5) * max(1.0, float(np.max(np.abs(want)))), (name, err)
    den = float(np.linalg.norm(want))
    if den > 0:
        rel = float(np.linalg.norm(got - want)) / den
        assert rel <= (1e-2 if bf16 else 2e-5), (name, "relative", rel)


def ring_backward_gpu(Q, K, V, dO, N, layout, scale=None, use_driver=False):
    """Forward ring, then all N*N backward steps.  Inputs in ORIGINAL order on the
    GPU; returns (dQ, dK, dV) fp32 GPU tensors in device order."""
    B, H, S, d = Q.shape
    c = S // N
    Qp, Kp, Vp, dOp = (to_device_order(x, N, layout) for x in (Q, K, V, dO))
    O = torch.empty(B, H, S, d, dtype=torch.float32, device=Q.device)
    LSE = torch.empty(B, H, S, dtype=torch.float32, device=Q.device)
    shape = sa.shard_shape(Qp, c, LSE, scale)
    sa.sa_ring_fwd(Qp, Kp, Vp, O, LSE, N, layout, shape)
    delta = torch.empty_like(LSE)
    dQ, dK, dV = (torch.empty_like(O) for _ in range(3))
    if use_driver:
        sa.sa_ring_bwd(Qp, Kp, Vp, dOp, O, LSE, delta, dQ, dK, dV, N, layout, shape)
        return dQ, dK, dV
    dQ.zero_(), dK.zero_(), dV.zero_()
    for j in range(N):
        sa.sa_bwd_preprocess(O[:, :, j * c:], dOp[:, :, j * c:], delta[:, :, j * c:], shape)
    for _, j, k in orc.ring_schedule(N):
        r = lambda t, dev: t[:, :, dev * c:]
        sa.sa_attn_step_bwd(r(Qp, j), r(Kp, k), r(Vp, k), r(dOp, j), r(LSE, j), r(delta, j),
                            r(dQ, j), r(dK, k), r(dV, k), j, k, N, layout, shape)
    return dQ, dK, dV


def oracle_backward(Q, K, V, dO, scale, rows=None):
    return orc.causal_attention_grad_bh(inputs.to_f64(Q), inputs.to_f64(K), inputs.to_f64(V),
                                        inputs.to_f64(dO), scale, rows)
