"""Pins of the oracle's rotary embedding and of the paper's remark about it (Sec. 2.3: with a
position embedding such as RoPE the position ids are permuted together with the tokens)."""
import numpy as np
import pytest

from oracle import striped_attention as orc


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def test_position_zero_is_the_identity_and_norms_are_kept():
    x = _rand((3, 5, 8), 1)
    assert np.allclose(orc.rope(x, np.zeros(5)), x)
    y = orc.rope(x, np.arange(5) * 37)
    half = 4
    assert np.allclose(x[..., :half] ** 2 + x[..., half:] ** 2, y[..., :half] ** 2 + y[..., half:] ** 2)


def test_against_complex_multiplication():
    # each pair (x_i, x_{i+d/2}) is the complex number x_i + j x_{i+d/2} times exp(j pos theta_i)
    d, rows, base = 12, 7, 500.0
    x = _rand((rows, d), 2)
    pos = np.array([0, 1, 2, 10, 100, 1000, 12345])
    z = x[:, : d // 2] + 1j * x[:, d // 2:]
    theta = base ** (-2.0 * np.arange(d // 2) / d)
    w = z * np.exp(1j * pos[:, None] * theta[None, :])
    want = np.concatenate([w.real, w.imag], axis=1)
    assert np.allclose(orc.rope(x, pos, base), want, atol=1e-12)


def test_scores_depend_on_the_position_difference_only():
    d = 16
    q, k = _rand((1, d), 3), _rand((1, d), 4)
    s = lambda m, n: float((orc.rope(q, [m]) @ orc.rope(k, [n]).T)[0, 0])
    assert s(5, 3) == pytest.approx(s(105, 103), abs=1e-10)
    assert s(7, 7) == pytest.approx(float((q @ k.T)[0, 0]), abs=1e-12)
    assert abs(s(5, 3) - s(5, 4)) > 1e-3


def test_inverse_is_the_transpose():
    x, g = _rand((6, 10), 5), _rand((6, 10), 6)
    pos = np.arange(6) * 3 + 1
    assert np.allclose(orc.rope(orc.rope(x, pos), pos, inverse=True), x)
    # <rope(x), g> == <x, rope^T(g)>
    assert np.sum(orc.rope(x, pos) * g) == pytest.approx(np.sum(x * orc.rope(g, pos, inverse=True)))


@pytest.mark.parametrize("N", [2, 4])
def test_permuting_tokens_and_position_ids_together_commutes_with_rope(N):
    # Sec. 2.3: permute the position ids with the tokens and every token is embedded as before
    S, d = 16, 8
    x = _rand((2, S, d), 7)
    ids = np.arange(S)
    a = orc.stripe_permute(orc.rope(x, ids), N, axis=1)
    b = orc.rope(orc.stripe_permute(x, N, axis=1), orc.stripe_permute(ids, N, axis=0))
    assert np.array_equal(a, b)
    # and the permuted ids are a*N + dev on device dev, local row a
    c = S // N
    got = orc.stripe_permute(ids, N, axis=0).reshape(N, c)
    assert all(got[dev, a] == a * N + dev for dev in range(N) for a in range(c))


def test_causal_attention_with_rope_is_permutation_consistent():
    # attention on striped, rotated inputs equals rotated attention in the original order
    S, d, N = 16, 8, 4
    q, k, v = (_rand((S, d), 10 + i) for i in range(3))
    ids = np.arange(S)
    O, _ = orc.causal_attention(orc.rope(q, ids), orc.rope(k, ids), v, 0.3)
    qp, kp, vp = (orc.stripe_permute(t, N, axis=0) for t in (q, k, v))
    idp = orc.stripe_permute(ids, N, axis=0)
    Op, _ = orc.ring_attention(orc.rope(qp, idp), orc.rope(kp, idp), vp, N, orc.STRIPED, 0.3)
    assert np.allclose(orc.unstripe_permute(Op, N, axis=0), O, atol=1e-12)
