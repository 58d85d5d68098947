"""GPU parity of the forward ring step against the fp64 oracle (full causal
attention of the unpermuted sequence), through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import striped_attention as orc
from paper_2311_09431_amd import binding as sa
from paper_2311_09431_amd import inputs
from tests import helpers as hp

pytestmark = pytest.mark.gpu

# tolerances: fp32 configuration 1e-5 on O and LSE; bf16 inputs with fp32
# accumulation 2e-2 on O and 1e-3 on LSE
TOL = {torch.float32: (1e-5, 1e-5), torch.bfloat16: (2e-2, 1e-3)}


def _check_ring(B, H, S, d, N, layout, dtype, seed, scale=None, use_driver=False, order=None):
    Q, K, V = inputs.qkv(B, H, S, d, seed, dtype)
    sc = scale if scale else 1.0 / np.sqrt(d)
    O, LSE = hp.ring_forward_gpu(Q.cuda(), K.cuda(), V.cuda(), N, layout, scale, use_driver, order)
    torch.cuda.synchronize()
    Oh = hp.from_device_order_host(O.cpu().numpy(), N, layout)
    Lh = hp.from_device_order_host(LSE.cpu().numpy(), N, layout)
    Ow, Lw = hp.oracle_forward(Q, K, V, sc)
    tol_o, tol_l = TOL[dtype]
    assert np.isfinite(Oh).all() and np.isfinite(Lh).all()
    assert hp.max_abs_err(Oh, Ow) <= tol_o, (hp.max_abs_err(Oh, Ow), hp.layout_name(layout))
    assert hp.max_abs_err(Lh, Lw) <= tol_l, (hp.max_abs_err(Lh, Lw), hp.layout_name(layout))


@pytest.mark.parametrize("layout", [sa.CONTIGUOUS, sa.STRIPED])
def test_tiny_fp32_config(layout):
    # batch 1, 1 head, head_dim 64, seq 256, N = 4 (64-token shards), fp32, 4 x 4 steps
    _check_ring(1, 1, 256, 64, 4, layout, torch.float32, seed=1)


@pytest.mark.parametrize("layout", [sa.CONTIGUOUS, sa.STRIPED])
@pytest.mark.parametrize("B,H,S,d,N,dtype", [
    (2, 3, 120, 32, 4, torch.float32),     # ragged: c = 30, not a multiple of anything
    (1, 2, 66, 8, 2, torch.float32),
    (1, 1, 8, 4, 8, torch.float32),        # c = 1: striped steps with kv_dev > q_dev see nothing
    (1, 2, 200, 128, 1, torch.float32),    # N = 1: plain causal attention
    (1, 2, 256, 256, 4, torch.float32),    # largest head dimension
    (2, 2, 192, 64, 4, torch.bfloat16),    # bf16 storage on the generic path
    (1, 2, 96, 128, 4, torch.bfloat16),    # d = 128 but c = 24: not MFMA-eligible
    (1, 2, 256, 100, 4, torch.bfloat16),   # head dimension of Table 1's 3B model (3200 / 32)
])
def test_generic_shapes(layout, B, H, S, d, N, dtype):
    _check_ring(B, H, S, d, N, layout, dtype, seed=S + d)


@pytest.mark.parametrize("layout", [sa.CONTIGUOUS, sa.STRIPED])
def test_driver_and_step_order(layout):
    _check_ring(1, 2, 128, 64, 4, layout, torch.float32, seed=9, use_driver=True)
    pairs = [(j, k) for j in range(4) for k in range(4)]
    np.random.default_rng(1).shuffle(pairs)
    _check_ring(1, 2, 128, 64, 4, layout, torch.float32, seed=9, order=pairs)


@pytest.mark.parametrize("layout", [sa.CONTIGUOUS, sa.STRIPED])
def test_single_steps_match_the_ring_oracle(layout):
    # each (j, k) step on its own against the oracle's step with the mask taken
    # from original token positions, starting from a non-trivial running state
    B, H, S, d, N = 1, 1, 96, 32, 4
    c = S // N
    Q, K, V = inputs.qkv(B, H, S, d, 21, torch.float32)
    Qn, Kn, Vn = (inputs.to_f64(x)[0, 0] for x in (Q, K, V))
    scale = 0.3
    for j in range(N):
        for k in range(N):
            qs, ks = slice(j * c, (j + 1) * c), slice(k * c, (k + 1) * c)
            prev = (k + 1) % N                       # some other block as the earlier state
            O0, L0 = orc.ring_step_fwd(np.zeros((c, d)), np.full(c, -np.inf), Qn[qs],
                                       Kn[prev * c:(prev + 1) * c], Vn[prev * c:(prev + 1) * c],
                                       j, prev, N, layout, scale)
            Ow, Lw = orc.ring_step_fwd(O0, L0, Qn[qs], Kn[ks], Vn[ks], j, k, N, layout, scale)
            Og = torch.from_numpy(O0).float().cuda()[None, None].contiguous()
            Lg = torch.from_numpy(L0).float().cuda()[None, None].contiguous()
            Qg, Kg, Vg = Q.cuda(), K.cuda(), V.cuda()
            shape = sa.shard_shape(Qg, c, None, scale)
            shape.stat_stride_b = shape.stat_stride_h = c
            oshape = sa.SaShape.from_buffer_copy(shape)
            # q/k/v live in the [1,1,S,d] tensor, o/lse in their own [1,1,c,(d)] tensors
            sa.sa_attn_step_fwd(Qg[:, :, qs], Kg[:, :, ks], Vg[:, :, ks], Og, Lg, j, k, N, layout,
                                oshape)
            torch.cuda.synchronize()
            Lh = Lg.cpu().numpy()[0, 0]
            both_inf = np.isneginf(Lh) & np.isneginf(Lw)
            assert (np.isneginf(Lh) == np.isneginf(Lw)).all(), (j, k)
            assert hp.max_abs_err(Og.cpu().numpy()[0, 0], Ow) <= 1e-5, (j, k)
            if not both_inf.all():
                assert hp.max_abs_err(Lh[~both_inf], Lw[~both_inf]) <= 1e-5, (j, k)


def test_finalize_rounds_to_storage_dtype():
    x = inputs.gaussian((2, 2, 64, 128), 5).cuda()
    shape = sa.shard_shape(x.to(torch.bfloat16), 64)
    out = torch.empty_like(x, dtype=torch.bfloat16)
    sa.sa_finalize(x, out, shape)
    assert torch.equal(out, x.to(torch.bfloat16))
    shape32 = sa.shard_shape(x, 64)
    out32 = torch.empty_like(x)
    sa.sa_finalize(x, out32, shape32)
    assert torch.equal(out32, x)


@pytest.mark.parametrize("layout", [sa.CONTIGUOUS, sa.STRIPED])
@pytest.mark.parametrize("B,H,S,N", [
    (1, 2, 512, 4),      # c = 128: one query tile, two key tiles per step
    (2, 2, 1024, 4),     # c = 256
    (1, 3, 2048, 2),     # c = 1024: 8 query tiles, several unmasked tiles before the diagonal
    (1, 1, 1152, 3),     # c = 384: odd number of query tiles
    (1, 2, 1024, 1),     # N = 1
])
def test_mfma_bf16_ring(layout, B, H, S, N):
    # bf16, d = 128, c % 128 == 0: the matrix-core kernel
    _check_ring(B, H, S, 128, N, layout, torch.bfloat16, seed=S + N, use_driver=(N == 4))


@pytest.mark.parametrize("layout", [sa.CONTIGUOUS, sa.STRIPED])
@pytest.mark.parametrize("d", [100, 64, 72, 4, 124, 112, 116])
def test_mfma_bf16_padded_head_dimension(layout, d):
    # d < 128 runs on the matrix-core kernel that computes 64, 112 or 128 columns; 100 is the
    # head dimension of Table 1's 3B model (half a 16-byte chunk at the row end), 72 ends on a
    # chunk, 124 leaves one group of four, 4 is the smallest, 112 is the widest that skips the
    # last 16-column step of the contractions over d and 116 the narrowest that does not
    _check_ring(1, 2, 1024, d, 4, layout, torch.bfloat16, seed=1000 + d, use_driver=True)


@pytest.mark.parametrize("layout", [sa.CONTIGUOUS, sa.STRIPED])
@pytest.mark.parametrize("B,H,S,d,N", [
    (1, 2, 1024, 256, 4),     # two 128-column halves of K and V per tile
    (2, 1, 2048, 256, 2),     # c = 1024: unmasked tiles before the diagonal
    (1, 2, 768, 192, 3),      # second half padded
    (1, 1, 600, 256, 2),      # c = 300: ragged block
    (1, 2, 512, 136, 2),      # one chunk into the second half
])
def test_mfma_bf16_head_dimension_above_128(layout, B, H, S, d, N):
    _check_ring(B, H, S, d, N, layout, torch.bfloat16, seed=4000 + d + S, use_driver=True)


@pytest.mark.parametrize("layout", [sa.CONTIGUOUS, sa.STRIPED])
def test_mfma_bf16_scale_and_order(layout):
    pairs = [(j, k) for j in range(4) for k in range(4)]
    np.random.default_rng(2).shuffle(pairs)
    _check_ring(1, 2, 1024, 128, 4, layout, torch.bfloat16, seed=77, scale=0.05, order=pairs)


def test_mfma_matches_generic_kernel_on_large_scores():
    # unit-variance q.k with scale 1 gives scores of magnitude ~ sqrt(128): a hard
    # softmax, checked against the oracle with the same tolerances
    _check_ring(1, 1, 512, 128, 2, sa.STRIPED, torch.bfloat16, seed=5, scale=1.0)


@pytest.mark.parametrize("layout", [sa.CONTIGUOUS, sa.STRIPED])
def test_mfma_scores_far_above_the_running_reference(layout):
    # q.k of magnitude ~ 50-250 nats with scale 1: exp2 of a score against a reference that
    # lags behind overflows fp32, and every later block may bring a much larger maximum; the
    # kernel must notice from the row sums, redo the sub-tile against its row maximum and
    # stay within tolerance (LSE ~ 200: the 1e-3 bound is 40 ulp of fp32 there)
    B, H, S, d, N = 1, 2, 1024, 128, 4
    Q, K, V = inputs.qkv(B, H, S, d, 4242, torch.bfloat16)
    Q, K = (Q * 2).to(torch.bfloat16), (K * 2).to(torch.bfloat16)
    O, LSE = hp.ring_forward_gpu(Q.cuda(), K.cuda(), V.cuda(), N, layout, 1.0, True)
    torch.cuda.synchronize()
    Oh = hp.from_device_order_host(O.cpu().numpy(), N, layout)
    Lh = hp.from_device_order_host(LSE.cpu().numpy(), N, layout)
    Ow, Lw = hp.oracle_forward(Q, K, V, 1.0)
    assert np.isfinite(Oh).all() and np.isfinite(Lh).all()
    assert float(np.max(Lw)) > 150.0                      # the case is what it claims to be
    assert hp.max_abs_err(Oh, Ow) <= 2e-2 and hp.max_abs_err(Lh, Lw) <= 1e-3
    # all-zero queries: every score equals the reference-free value 0, uniform attention
    O2, LSE2 = hp.ring_forward_gpu((Q * 0).cuda(), K.cuda(), V.cuda(), N, layout, 1.0, True)
    torch.cuda.synchronize()
    Ow2, Lw2 = hp.oracle_forward(Q * 0, K, V, 1.0)
    assert hp.max_abs_err(hp.from_device_order_host(O2.cpu().numpy(), N, layout), Ow2) <= 2e-2
    assert hp.max_abs_err(hp.from_device_order_host(LSE2.cpu().numpy(), N, layout), Lw2) <= 1e-3


def test_mfma_forward_is_deterministic_and_honours_the_stream():
    # no atomics anywhere: two runs give the same bits; and the work goes to the caller's stream
    B, H, S, d, N = 1, 2, 1024, 128, 4
    Q, K, V = (x.cuda() for x in inputs.qkv(B, H, S, d, 31, torch.bfloat16))
    O1, L1 = hp.ring_forward_gpu(Q, K, V, N, sa.STRIPED, use_driver=True)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        O2, L2 = hp.ring_forward_gpu(Q, K, V, N, sa.STRIPED, use_driver=True)
    side.synchronize()
    torch.cuda.synchronize()
    assert torch.equal(O1, O2) and torch.equal(L1, L2)
