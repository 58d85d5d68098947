"""Pins for the stripe permutation, GetMask, Work(i, j) and tile skipping."""
import os

import numpy as np
import pytest

from oracle import striped_attention as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _lines(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [l.split("#")[0].split() for l in f if l.split("#")[0].strip()]


def test_paper_stripe_example():
    for N, dev, *tokens in _lines("stripe_example.txt"):
        N, dev, tokens = int(N), int(dev), [int(t) for t in tokens]
        S = 4 * N
        permuted = orc.stripe_permute(np.arange(S), N, 0)
        c = S // N
        assert list(permuted[dev * c: dev * c + len(tokens)]) == tokens


@pytest.mark.parametrize("S,N", [(16, 4), (24, 8), (12, 1), (10, 2), (48, 16)])
def test_permutation_closed_form_and_inverse(S, N):
    c = S // N
    x = np.arange(S * 3).reshape(S, 3)
    p = orc.stripe_permute(x, N, 0)
    # token t = a*N + dev sits at row dev*c + a: a transposition of a [c, N] grid
    np.testing.assert_array_equal(p, x.reshape(c, N, 3).transpose(1, 0, 2).reshape(S, 3))
    np.testing.assert_array_equal(orc.unstripe_permute(p, N, 0), x)
    np.testing.assert_array_equal(orc.stripe_permute(orc.unstripe_permute(x, N, 0), N, 0), x)
    for t in range(S):
        assert p[(t % N) * c + t // N, 0] == x[t, 0]
    y = np.arange(2 * S * 2).reshape(2, S, 2)
    np.testing.assert_array_equal(orc.stripe_permute(y, N, 1)[1], orc.stripe_permute(y[1], N, 0))


def test_permutation_rejects_ragged():
    with pytest.raises(ValueError):
        orc.stripe_source_index(10, 4)


@pytest.mark.parametrize("S,N", [(16, 4), (12, 3), (8, 8)])   # (16, 4) is the Fig. 2/3 case
def test_get_mask_is_the_block_of_C(S, N):
    c = S // N
    C = orc.causal_mask(S)
    allowed_full = np.isfinite(C)
    src = orc.stripe_source_index(S, N)
    allowed_perm = allowed_full[np.ix_(src, src)]        # C seen in permuted order
    total = {orc.CONTIGUOUS: 0, orc.STRIPED: 0}
    for j in range(N):
        for k in range(N):
            blk = (slice(j * c, (j + 1) * c), slice(k * c, (k + 1) * c))
            m = orc.get_mask(j, k, N, c, orc.CONTIGUOUS)
            np.testing.assert_array_equal(m, allowed_full[blk])     # Sec. 2.2: entry (j,k) of C
            m = orc.get_mask(j, k, N, c, orc.STRIPED)
            np.testing.assert_array_equal(m, allowed_perm[blk])
            total[orc.CONTIGUOUS] += orc.work(j, k, N, c, orc.CONTIGUOUS)
            total[orc.STRIPED] += orc.work(j, k, N, c, orc.STRIPED)
    assert total[orc.CONTIGUOUS] == total[orc.STRIPED] == S * (S + 1) // 2


@pytest.mark.parametrize("N,c", [(4, 4), (8, 5), (2, 16)])
def test_work_formula(N, c):
    # Sec. 2.3: Work(i, j) = c(c+1)/2 if i >= j else c(c-1)/2 for Striped Attention;
    # Ring Attention has a device with c^2 on every round after the first (Sec. 1, 2.3).
    for i in range(N):
        for j in range(N):
            want = c * (c + 1) // 2 if i >= j else c * (c - 1) // 2
            assert orc.work(i, j, N, c, orc.STRIPED) == want
    ring = orc.worst_device_work_per_round(N, c, orc.CONTIGUOUS)
    assert ring[0] == c * (c + 1) // 2 and all(w == c * c for w in ring[1:])
    striped = orc.worst_device_work_per_round(N, c, orc.STRIPED)
    assert all(w == c * (c + 1) // 2 for w in striped)
    # in the limit the ratio of the two sums tends to 2 (Sec. 2.3, last paragraph)
    assert sum(ring) / sum(striped) == pytest.approx(
        (c * (c + 1) / 2 + (N - 1) * c * c) / (N * c * (c + 1) / 2))


def test_speedup_limit_approaches_two():
    N, c = 64, 512
    ring = sum(orc.worst_device_work_per_round(N, c, orc.CONTIGUOUS))
    striped = sum(orc.worst_device_work_per_round(N, c, orc.STRIPED))
    assert 1.95 < ring / striped < 2.0


def test_paper_tiling_examples():
    for c, tq, tk, kind, full, part, empty, pct in _lines("tiling_examples.txt"):
        c, tq, tk = int(c), int(tq), int(tk)
        if kind == "causal":
            allowed = orc.get_mask(1, 1, 2, c, orc.CONTIGUOUS)
        else:
            allowed = orc.get_mask(0, 1, 2, c, orc.STRIPED)
        got = orc.classify_tiles(allowed, tq, tk)
        for g, w in zip(got, (int(full), int(part), int(empty))):
            if w >= 0:
                assert g == w
        assert int(100 * got[2] / sum(got)) == int(pct)
    # a fully unmasked block computes every tile (Sec. 2.2.1, last sentence)
    assert orc.classify_tiles(orc.get_mask(1, 0, 2, 1536, orc.CONTIGUOUS), 512, 512) == (9, 0, 0)
    assert orc.classify_tiles(orc.get_mask(0, 1, 2, 1536, orc.CONTIGUOUS), 512, 512) == (0, 0, 9)
