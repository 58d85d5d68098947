"""Pins for the backward oracle: central finite differences, library autograd in
fp64, and invariants of the softmax gradient.  (The paper gives no backward
pass; the oracle is the analytic gradient of the Sec. 2.1 definition.)"""
import numpy as np
import pytest
import torch

from oracle import striped_attention as orc


def _rand(S, d, seed, n=4):
    r = np.random.default_rng(seed)
    return tuple(r.standard_normal((S, d)) for _ in range(n))


def _loss(Q, K, V, dO, scale):
    O, _ = orc.causal_attention(Q, K, V, scale)
    return float((O * dO).sum())


@pytest.mark.parametrize("S,d,scale", [(3, 2, 1.0), (9, 4, 0.5), (16, 3, 0.8)])
def test_finite_differences(S, d, scale):
    Q, K, V, dO = _rand(S, d, S + d)
    grads = orc.causal_attention_grad(Q, K, V, dO, scale)
    eps = 1e-6
    for which, g in enumerate(grads):
        num = np.zeros_like(g)
        for idx in np.ndindex(*g.shape):
            args = [Q.copy(), K.copy(), V.copy()]
            args[which][idx] += eps
            up = _loss(*args, dO, scale)
            args[which][idx] -= 2 * eps
            dn = _loss(*args, dO, scale)
            num[idx] = (up - dn) / (2 * eps)
        np.testing.assert_allclose(g, num, atol=2e-8, rtol=1e-7)


@pytest.mark.parametrize("S,d", [(20, 8), (48, 16)])
def test_matches_library_autograd_fp64(S, d):
    Q, K, V, dO = _rand(S, d, 11)
    scale = 1.0 / np.sqrt(d)
    dQ, dK, dV = orc.causal_attention_grad(Q, K, V, dO, scale)
    tq, tk, tv = (torch.from_numpy(x).clone().requires_grad_(True) for x in (Q, K, V))
    s = scale * tq @ tk.T
    s = s.masked_fill(torch.triu(torch.ones(S, S, dtype=torch.bool), 1), float("-inf"))
    (torch.softmax(s, dim=1) @ tv).backward(torch.from_numpy(dO))
    np.testing.assert_allclose(dQ, tq.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(dK, tk.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(dV, tv.grad.numpy(), atol=1e-12)


def test_invariants():
    Q, K, V, dO = _rand(25, 6, 12)
    dQ, dK, dV = orc.causal_attention_grad(Q, K, V, dO, 0.4)
    # every softmax row sums to one => columns of P^T dO add up to the rows of dO
    np.testing.assert_allclose(dV.sum(axis=0), dO.sum(axis=0), atol=1e-12)
    # dQ = scale dS K and dK = scale dS^T Q => <Q, dQ> = <K, dK> = scale sum(dS * S)
    np.testing.assert_allclose((Q * dQ).sum(), (K * dK).sum(), atol=1e-12)
    # row 0 attends only to key 0: its softmax is the constant 1 => dQ_0 = 0
    np.testing.assert_allclose(dQ[0], 0.0, atol=1e-14)
    # the last key is seen only by the last query
    assert np.all(dV[-1] != 0)


def test_rows_subset_equals_zeroed_dout():
    Q, K, V, dO = _rand(21, 4, 13)
    rows = [0, 5, 6, 20]
    dOz = np.zeros_like(dO)
    dOz[rows] = dO[rows]
    a = orc.causal_attention_grad(Q, K, V, dO, 0.6, rows=rows)
    b = orc.causal_attention_grad(Q, K, V, dOz, 0.6)
    for x, y in zip(a, b):
        np.testing.assert_allclose(x, y, atol=1e-14)
    mask = np.ones(21, bool)
    mask[rows] = False
    assert np.all(a[0][mask] == 0)


@pytest.mark.parametrize("S,d,rows", [
    (21, 4, [0, 5, 6, 20]),
    (40, 8, list(range(40))),
    (33, 5, [32]),
    (17, 3, [3, 16, 9]),           # unsorted
])
def test_matrix_form_over_a_row_set_equals_the_row_by_row_gradient(S, d, rows):
    Q, K, V, dO = _rand(S, d, 14 + S)
    a = orc.causal_attention_grad(Q, K, V, dO, 0.7, rows=rows)
    dQ, dK, dV, O, LSE = orc.causal_attention_grad_matrix(Q, K, V, dO, 0.7, rows)
    for x, y in zip(a, (dQ, dK, dV)):
        np.testing.assert_allclose(x, y, atol=1e-13)
    Ow, Lw = orc.causal_attention_rows(Q, K, V, 0.7, rows)
    np.testing.assert_allclose(O, Ow, atol=1e-13)
    np.testing.assert_allclose(LSE, Lw, atol=1e-13)


def test_matrix_form_finite_differences_and_additivity():
    S, d, scale = 10, 3, 0.9
    Q, K, V, dO = _rand(S, d, 99)
    rows = [2, 7, 9]
    dOz = np.zeros_like(dO)
    dOz[rows] = dO[rows]
    grads = orc.causal_attention_grad_matrix(Q, K, V, dO, scale, rows)[:3]
    eps = 1e-6
    for which, g in enumerate(grads):
        num = np.zeros_like(g)
        for idx in np.ndindex(*g.shape):
            args = [Q.copy(), K.copy(), V.copy()]
            args[which][idx] += eps
            up = _loss(*args, dOz, scale)
            args[which][idx] -= 2 * eps
            dn = _loss(*args, dOz, scale)
            num[idx] = (up - dn) / (2 * eps)
        np.testing.assert_allclose(g, num, atol=2e-8, rtol=1e-7)
    # additive over disjoint row sets; dQ rows do not depend on the other rows' dO
    a = orc.causal_attention_grad_matrix(Q, K, V, dO, scale, [2, 7])
    b = orc.causal_attention_grad_matrix(Q, K, V, dO, scale, [9])
    for x, y, z in zip(a[:3], b[:3], grads):
        np.testing.assert_allclose(x + y, z, atol=1e-14)
    full = orc.causal_attention_grad(Q, K, V, dO, scale)
    np.testing.assert_allclose(grads[0][rows], full[0][rows], atol=1e-14)
    # keys at or after position j0 are seen only by queries at or after j0
    j0 = 6
    tail = orc.causal_attention_grad_matrix(Q, K, V, dO, scale, list(range(j0, S)))
    np.testing.assert_allclose(tail[1][j0:], full[1][j0:], atol=1e-14)
    np.testing.assert_allclose(tail[2][j0:], full[2][j0:], atol=1e-14)
