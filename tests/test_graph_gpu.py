"""The ring drivers only launch kernels on the caller's stream (no allocation, no
synchronisation, no memset nodes when no timings are asked for), so a whole forward +
backward pass can be recorded into a HIP graph.  Every replay must reproduce the eager
result bit for bit (the kernels are deterministic)."""
import pytest
import torch

from paper_2311_09431_amd import binding as sa
from paper_2311_09431_amd import inputs

pytestmark = pytest.mark.gpu


def _buffers(B, H, S, d, seed):
    Q, K, V, dO = (x.cuda() for x in inputs.qkv(B, H, S, d, seed, torch.bfloat16, with_dout=True))
    perm = [torch.empty_like(x) for x in (Q, K, V, dO)]
    O = torch.empty(B, H, S, d, dtype=torch.float32, device="cuda")
    LSE = torch.empty(B, H, S, dtype=torch.float32, device="cuda")
    out = torch.empty(B, H, S, d, dtype=torch.bfloat16, device="cuda")
    delta = torch.empty_like(LSE)
    grads = [torch.empty_like(O) for _ in range(3)]
    return (Q, K, V, dO), perm, O, LSE, out, delta, grads


def _one_pass(orig, perm, O, LSE, out, delta, grads, N, c, shape):
    for x, y in zip(orig, perm):
        sa.sa_stripe_permute(x, y, N)
    sa.sa_ring_fwd(perm[0], perm[1], perm[2], O, LSE, N, sa.STRIPED, shape)
    for j in range(N):
        sa.sa_finalize(O[:, :, j * c:], out[:, :, j * c:], shape)
    sa.sa_ring_bwd(perm[0], perm[1], perm[2], perm[3], O, LSE, delta, *grads, N, sa.STRIPED, shape)


@pytest.mark.parametrize("S,d", [(1024, 128), (240, 64)])      # matrix-core and generic kernels
def test_forward_backward_pass_replays_from_a_graph(S, d):
    B, H, N = 1, 2, 4
    c = S // N
    bufs = _buffers(B, H, S, d, 41)
    orig, perm, O, LSE, out, delta, grads = bufs
    shape = sa.shard_shape(perm[0], c, LSE)
    _one_pass(*bufs, N, c, shape)
    torch.cuda.synchronize()
    want = [t.clone() for t in (O, LSE, out, *grads)]

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        _one_pass(*bufs, N, c, shape)
    for replay in range(3):
        for t in (O, LSE, out, delta, *grads, *perm):     # eager work between the replays
            t.fill_(float(replay + 1))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip((O, LSE, out, *grads), want):
            assert torch.equal(got, ref), replay
    # new inputs in the same buffers: the graph reads them at replay time
    fresh = inputs.qkv(B, H, S, d, 42, torch.bfloat16, with_dout=True)
    for x, y in zip(orig, fresh):
        x.copy_(y)
    graph.replay()
    torch.cuda.synchronize()
    replayed = [t.clone() for t in (O, LSE, out, *grads)]
    _one_pass(*bufs, N, c, shape)
    torch.cuda.synchronize()
    for got, ref in zip(replayed, (O, LSE, out, *grads)):
        assert torch.equal(got, ref)
