"""GPU parity of sa_stripe_permute / sa_unstripe_permute: bit-exact against the
oracle's permutation for every row width class the kernel dispatches on."""
import numpy as np
import pytest
import torch

from oracle import striped_attention as orc
from paper_2311_09431_amd import binding as sa

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("outer,S,inner,N,dtype", [
    (2, 16, 1, 4, torch.uint8),          # 1-byte rows
    (3, 24, 1, 8, torch.int16),          # 2-byte rows
    (2, 4096, 1, 8, torch.int32),        # token / position ids
    (2, 1000, 1, 4, torch.int64),        # targets
    (1, 48, 3, 16, torch.int16),         # 6-byte rows
    (4, 2048, 128, 8, torch.bfloat16),   # 256-byte rows (Q/K/V, d = 128)
    (2, 512, 64, 4, torch.float32),      # fp32 rows, d = 64
    (1, 12, 5, 1, torch.uint8),          # N = 1: identity
    (2, 96, 128, 96, torch.bfloat16),    # c = 1
    (3, 1000, 128, 5, torch.bfloat16),   # 256-byte rows, 1000 rows of 5 devices
    (2, 84, 1024, 7, torch.float32),     # 4096-byte rows
    (2, 520, 4, 8, torch.float32),       # 16-byte rows: a single chunk
    (2, 60, 100, 4, torch.bfloat16),     # 200-byte rows (d = 100): 8-byte chunks
    (2, 64, 96, 4, torch.bfloat16),      # 192-byte rows: 12 chunks of 16 bytes
])
def test_permute_bit_exact(outer, S, inner, N, dtype):
    g = torch.Generator().manual_seed(S + inner)
    x = torch.randint(0, 250, (outer, S, inner), generator=g, dtype=torch.int64)
    if dtype in (torch.bfloat16, torch.float32):
        x = x.to(torch.float32).to(dtype)
    else:
        x = x.to(dtype)
    xg = x.cuda()
    yg = torch.empty_like(xg)
    sa.sa_stripe_permute(xg, yg, N, seq_axis=1)
    want = orc.stripe_permute(x.view(torch.uint8).numpy().reshape(outer, S, -1), N, 1)
    got = yg.cpu().view(torch.uint8).numpy().reshape(outer, S, -1)
    assert np.array_equal(got, want)
    zg = torch.empty_like(xg)
    sa.sa_unstripe_permute(yg, zg, N, seq_axis=1)
    assert torch.equal(zg, xg)
    want_inv = orc.unstripe_permute(x.view(torch.uint8).numpy().reshape(outer, S, -1), N, 1)
    sa.sa_unstripe_permute(xg, zg, N, seq_axis=1)
    assert np.array_equal(zg.cpu().view(torch.uint8).numpy().reshape(outer, S, -1), want_inv)


def test_permute_empty_and_errors():
    x = torch.zeros(0, 8, 4, device="cuda")
    sa.sa_stripe_permute(x, torch.empty_like(x), 4, seq_axis=1)      # outer = 0: no-op
    x = torch.zeros(1, 10, 4, device="cuda")
    with pytest.raises(sa.StripedAttnError):
        sa.sa_stripe_permute(x, torch.empty_like(x), 4, seq_axis=1)  # 10 % 4 != 0
    with pytest.raises(sa.StripedAttnError):
        sa.sa_stripe_permute(x, x, 2, seq_axis=1)                    # in place
