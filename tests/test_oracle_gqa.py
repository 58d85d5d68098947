"""Pins for the oracle's grouped-head attention (fewer key/value heads than query
heads; an extension, not in the paper): the library's grouped causal attention
and its autograd in fp64, central finite differences on a shared head, and the
special cases H_kv = H (plain multi-head attention) and repeated heads."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import striped_attention as orc


def _rand(B, H, H_kv, S, d, seed):
    r = np.random.default_rng(seed)
    return (r.standard_normal((B, H, S, d)), r.standard_normal((B, H_kv, S, d)),
            r.standard_normal((B, H_kv, S, d)), r.standard_normal((B, H, S, d)))


def test_head_mapping_is_by_consecutive_groups():
    assert [orc.kv_head_of(h, 8, 2) for h in range(8)] == [0, 0, 0, 0, 1, 1, 1, 1]
    assert [orc.kv_head_of(h, 4, 4) for h in range(4)] == [0, 1, 2, 3]
    assert [orc.kv_head_of(h, 3, 1) for h in range(3)] == [0, 0, 0]


@pytest.mark.parametrize("H,H_kv", [(4, 2), (6, 1), (3, 3)])
def test_matches_library_grouped_attention_and_autograd(H, H_kv):
    B, S, d = 2, 24, 8
    Q, K, V, dO = _rand(B, H, H_kv, S, d, H * 10 + H_kv)
    scale = 0.37
    O, _ = orc.causal_attention_gqa(Q, K, V, scale)
    dQ, dK, dV = orc.causal_attention_gqa_grad(Q, K, V, dO, scale)
    tq, tk, tv = (torch.from_numpy(x).clone().requires_grad_(True) for x in (Q, K, V))
    to = F.scaled_dot_product_attention(tq, tk, tv, is_causal=True, scale=scale, enable_gqa=True)
    to.backward(torch.from_numpy(dO))
    np.testing.assert_allclose(O, to.detach().numpy(), atol=1e-12)
    np.testing.assert_allclose(dQ, tq.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(dK, tk.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(dV, tv.grad.numpy(), atol=1e-12)


def test_equal_head_counts_reduce_to_multi_head_attention():
    Q, K, V, dO = _rand(1, 3, 3, 17, 4, 5)
    O, L = orc.causal_attention_gqa(Q, K, V, 0.5)
    Ow, Lw = orc.causal_attention_bh(Q, K, V, 0.5)
    assert np.array_equal(O, Ow) and np.array_equal(L, Lw)
    for g, w in zip(orc.causal_attention_gqa_grad(Q, K, V, dO, 0.5),
                    orc.causal_attention_grad_bh(Q, K, V, dO, 0.5)):
        assert np.array_equal(g, w)


def test_equals_multi_head_attention_on_repeated_heads_with_summed_gradients():
    B, H, H_kv, S, d = 1, 6, 2, 13, 4
    Q, K, V, dO = _rand(B, H, H_kv, S, d, 9)
    g = H // H_kv
    Kr, Vr = np.repeat(K, g, axis=1), np.repeat(V, g, axis=1)
    O, L = orc.causal_attention_gqa(Q, K, V, 0.6)
    Ow, Lw = orc.causal_attention_bh(Q, Kr, Vr, 0.6)
    np.testing.assert_allclose(O, Ow, atol=1e-15)
    np.testing.assert_allclose(L, Lw, atol=1e-15)
    dQ, dK, dV = orc.causal_attention_gqa_grad(Q, K, V, dO, 0.6)
    dQw, dKw, dVw = orc.causal_attention_grad_bh(Q, Kr, Vr, dO, 0.6)
    np.testing.assert_allclose(dQ, dQw, atol=1e-14)
    np.testing.assert_allclose(dK, dKw.reshape(B, H_kv, g, S, d).sum(2), atol=1e-13)
    np.testing.assert_allclose(dV, dVw.reshape(B, H_kv, g, S, d).sum(2), atol=1e-13)


def test_finite_differences_on_a_shared_head():
    B, H, H_kv, S, d = 1, 4, 2, 5, 2
    Q, K, V, dO = _rand(B, H, H_kv, S, d, 3)
    scale, eps = 0.9, 1e-6
    _, dK, dV = orc.causal_attention_gqa_grad(Q, K, V, dO, scale)

    def loss(K_, V_):
        return float((orc.causal_attention_gqa(Q, K_, V_, scale)[0] * dO).sum())

    for grad, which in ((dK, 0), (dV, 1)):
        for idx in np.ndindex(*grad.shape):
            up, dn = [K.copy(), V.copy()], [K.copy(), V.copy()]
            up[which][idx] += eps
            dn[which][idx] -= eps
            num = (loss(*up) - loss(*dn)) / (2 * eps)
            assert abs(num - grad[idx]) <= 2e-8 + 1e-7 * abs(num)
