"""Pins for the ring functions: the N-step ring, unpermuted, equals full causal
attention for both layouts (the paper's exactness claim, Sec. 1), in any step
order; the merge is the lazy-softmax algebra; the ring gradient equals the
full gradient."""
import numpy as np
import pytest

from oracle import striped_attention as orc


def _rand(S, d, seed, n=3):
    r = np.random.default_rng(seed)
    return tuple(r.standard_normal((S, d)) for _ in range(n))


@pytest.mark.parametrize("layout", [orc.CONTIGUOUS, orc.STRIPED])
@pytest.mark.parametrize("S,N,d", [(16, 4, 4), (24, 3, 5), (32, 8, 8), (9, 1, 3)])
def test_ring_equals_full_causal_attention(layout, S, N, d):
    Q, K, V = _rand(S, d, S + N)
    scale = 0.6
    O, L = orc.causal_attention(Q, K, V, scale)
    if layout == orc.STRIPED:
        Qp, Kp, Vp = (orc.stripe_permute(x, N, 0) for x in (Q, K, V))
    else:
        Qp, Kp, Vp = Q, K, V
    Or, Lr = orc.ring_attention(Qp, Kp, Vp, N, layout, scale)
    if layout == orc.STRIPED:
        Or, Lr = orc.unstripe_permute(Or, N, 0), orc.unstripe_permute(Lr, N, 0)
    np.testing.assert_allclose(Or, O, atol=1e-12)
    np.testing.assert_allclose(Lr, L, atol=1e-12)


@pytest.mark.parametrize("layout", [orc.CONTIGUOUS, orc.STRIPED])
def test_step_order_does_not_matter(layout):
    S, N, d = 20, 4, 3
    Q, K, V = _rand(S, d, 2)
    base = orc.ring_attention(Q, K, V, N, layout, 0.5)
    pairs = [(j, k) for j in range(N) for k in range(N)]
    np.random.default_rng(0).shuffle(pairs)
    other = orc.ring_attention(Q, K, V, N, layout, 0.5, order=pairs)
    np.testing.assert_allclose(other[0], base[0], atol=1e-12)
    np.testing.assert_allclose(other[1], base[1], atol=1e-12)


def test_schedule_is_algorithm_1():
    N = 4
    sched = orc.ring_schedule(N)
    assert sched[:N] == [(0, j, j) for j in range(N)]          # round 0: own block
    assert sched[N:2 * N] == [(1, 0, 3), (1, 1, 0), (1, 2, 1), (1, 3, 2)]
    assert sorted((j, k) for _, j, k in sched) == [(j, k) for j in range(N) for k in range(N)]


def test_merge_is_softmax_over_the_union_of_key_sets():
    c, d = 6, 4
    Q, _, _ = _rand(c, d, 3)
    K, V = _rand(10, d, 4, n=2)
    everything = np.ones((c, 10), bool)
    O, L = orc.attention_fragment(Q, K, V, everything, 0.7)
    O1, L1 = orc.attention_fragment(Q, K[:3], V[:3], everything[:, :3], 0.7)
    O2, L2 = orc.attention_fragment(Q, K[3:], V[3:], everything[:, 3:], 0.7)
    Om, Lm = orc.merge(O1, L1, O2, L2)
    np.testing.assert_allclose(Om, O, atol=1e-13)
    np.testing.assert_allclose(Lm, L, atol=1e-13)
    Om2, Lm2 = orc.merge(O2, L2, O1, L1)                        # commutative
    np.testing.assert_allclose(Om2, Om, atol=1e-15)
    # textbook check of the fragment itself
    s = 0.7 * Q @ K.T
    w = np.exp(s) / np.exp(s).sum(axis=1, keepdims=True)
    np.testing.assert_allclose(O, w @ V, atol=1e-13)
    np.testing.assert_allclose(L, np.log(np.exp(s).sum(axis=1)), atol=1e-13)


def test_merge_identity_and_empty_rows():
    O1 = np.arange(6.0).reshape(3, 2)
    L1 = np.array([0.5, -2.0, 3.0])
    zero, ninf = np.zeros((3, 2)), np.full(3, -np.inf)
    Om, Lm = orc.merge(zero, ninf, O1, L1)
    np.testing.assert_array_equal(Om, O1)
    np.testing.assert_array_equal(Lm, L1)
    Om, Lm = orc.merge(zero, ninf, zero, ninf)
    assert np.all(Om == 0) and np.all(np.isneginf(Lm))
    # striped step with j < k: local row 0 sees no key of that block
    Q, K, V = _rand(4, 2, 5)
    Of, Lf = orc.attention_fragment(Q, K, V, orc.get_mask(0, 1, 2, 4, orc.STRIPED), 1.0)
    assert np.all(Of[0] == 0) and np.isneginf(Lf[0]) and np.all(np.isfinite(Lf[1:]))
    # contiguous step with j < k: nothing at all
    Of, Lf = orc.attention_fragment(Q, K, V, orc.get_mask(0, 1, 2, 4, orc.CONTIGUOUS), 1.0)
    assert np.all(Of == 0) and np.all(np.isneginf(Lf))


@pytest.mark.parametrize("layout", [orc.CONTIGUOUS, orc.STRIPED])
@pytest.mark.parametrize("S,N,d", [(16, 4, 4), (18, 3, 2)])
def test_ring_gradient_equals_full_gradient(layout, S, N, d):
    Q, K, V, dO = _rand(S, d, 6, n=4)
    scale = 0.45
    want = orc.causal_attention_grad(Q, K, V, dO, scale)
    if layout == orc.STRIPED:
        ins = [orc.stripe_permute(x, N, 0) for x in (Q, K, V, dO)]
    else:
        ins = [Q, K, V, dO]
    got = orc.ring_attention_grad(*ins, N, layout, scale)
    if layout == orc.STRIPED:
        got = [orc.unstripe_permute(g, N, 0) for g in got]
    for g, w in zip(got, want):
        np.testing.assert_allclose(g, w, atol=1e-12)
