"""Pins for the forward oracle (Sec. 2.1): brute-force S x S softmax with the
mask matrix C, closed forms, and a library causal SDPA in fp64."""
import numpy as np
import pytest
import torch

from oracle import striped_attention as orc


def _rand(S, d, seed):
    r = np.random.default_rng(seed)
    return r.standard_normal((S, d)), r.standard_normal((S, d)), r.standard_normal((S, d))


def _brute(Q, K, V, scale):
    """Softmax(scale Q K^T + C) V with the matrices materialised and a naive
    exp / row-sum (no max subtraction): a different code shape from the oracle."""
    S = Q.shape[0]
    C = np.zeros((S, S))
    for i in range(S):
        for j in range(S):
            if i < j:                       # Sec. 2.1: C_ij = -inf iff i < j
                C[i, j] = -np.inf
    E = np.exp(scale * (Q @ K.T) + C)
    den = E.sum(axis=1)
    return (E / den[:, None]) @ V, np.log(den)


@pytest.mark.parametrize("S,d,scale", [(1, 1, 1.0), (2, 3, 0.5), (7, 4, 1.0), (16, 8, 0.35),
                                       (33, 5, 0.7)])
def test_matches_brute_force(S, d, scale):
    Q, K, V = _rand(S, d, S * 100 + d)
    O, L = orc.causal_attention(Q, K, V, scale)
    Ob, Lb = _brute(Q, K, V, scale)
    np.testing.assert_allclose(O, Ob, rtol=0, atol=1e-12)
    np.testing.assert_allclose(L, Lb, rtol=0, atol=1e-12)


def test_softmax_rows_sum_to_one_and_upper_triangle_is_zero():
    S = 24
    Q, K, _ = _rand(S, 6, 3)
    P, _ = orc.causal_attention(Q, K, np.eye(S), 0.4)      # V = I  =>  O = P
    np.testing.assert_allclose(P.sum(axis=1), np.ones(S), atol=1e-14)
    assert np.all(P[np.triu_indices(S, 1)] == 0.0)
    assert np.all(P[np.tril_indices(S)] > 0.0)


def test_zero_queries_give_prefix_means_and_log_counts():
    S, d = 40, 5
    _, K, V = _rand(S, d, 4)
    O, L = orc.causal_attention(np.zeros((S, d)), K, V, 1.0)
    want = np.cumsum(V, axis=0) / np.arange(1, S + 1)[:, None]
    np.testing.assert_allclose(O, want, atol=1e-13)
    np.testing.assert_allclose(L, np.log(np.arange(1, S + 1)), atol=1e-13)


def test_constant_values_and_first_row():
    S, d = 19, 7
    Q, K, V = _rand(S, d, 5)
    O, _ = orc.causal_attention(Q, K, np.ones((S, d)), 0.3)
    np.testing.assert_allclose(O, np.ones((S, d)), atol=1e-14)
    O, L = orc.causal_attention(Q, K, V, 0.3)
    np.testing.assert_allclose(O[0], V[0], atol=1e-15)
    np.testing.assert_allclose(L[0], 0.3 * Q[0] @ K[0], atol=1e-14)


def test_scale_is_applied_to_the_scores():
    Q, K, V = _rand(12, 4, 6)
    O1, L1 = orc.causal_attention(Q, K, V, 0.25)
    O2, L2 = orc.causal_attention(0.25 * Q, K, V, 1.0)
    np.testing.assert_allclose(O1, O2, atol=1e-13)
    np.testing.assert_allclose(L1, L2, atol=1e-13)


def test_operands_are_not_transposed_or_swapped():
    # one-hot rows make every term readable: query i = e_i, key j = w_j * e_i-th column
    S = 5
    Q = np.eye(S)
    K = np.arange(1, S * S + 1, dtype=float).reshape(S, S) / 10.0
    V = np.arange(S * 3, dtype=float).reshape(S, 3)
    O, L = orc.causal_attention(Q, K, V, 1.0)
    for i in range(S):
        s = K[: i + 1, i]                     # score of (i, j) = K[j, i]
        w = np.exp(s) / np.exp(s).sum()
        np.testing.assert_allclose(O[i], w @ V[: i + 1], atol=1e-13)
        np.testing.assert_allclose(L[i], np.log(np.exp(s).sum()), atol=1e-13)


@pytest.mark.parametrize("S,d", [(17, 8), (64, 16)])
def test_matches_library_causal_sdpa_fp64(S, d):
    Q, K, V = _rand(S, d, 7)
    scale = 1.0 / np.sqrt(d)
    O, _ = orc.causal_attention(Q, K, V, scale)
    t = lambda x: torch.from_numpy(x)[None, None]
    ref = torch.nn.functional.scaled_dot_product_attention(t(Q), t(K), t(V), is_causal=True,
                                                           scale=scale)[0, 0].numpy()
    np.testing.assert_allclose(O, ref, atol=1e-12)


def test_rows_subset_and_batched_wrapper():
    Q, K, V = _rand(30, 4, 8)
    O, L = orc.causal_attention(Q, K, V, 0.5)
    rows = [0, 7, 29]
    Or, Lr = orc.causal_attention_rows(Q, K, V, 0.5, rows)
    np.testing.assert_array_equal(Or, O[rows])
    np.testing.assert_array_equal(Lr, L[rows])
    Ob, Lb = orc.causal_attention_bh(np.stack([Q, K])[None], np.stack([K, V])[None],
                                     np.stack([V, Q])[None], 0.5)
    assert Ob.shape == (1, 2, 30, 4) and Lb.shape == (1, 2, 30)
    np.testing.assert_array_equal(Ob[0, 0], O)
    np.testing.assert_array_equal(Lb[0, 1], orc.causal_attention(K, V, Q, 0.5)[1])
