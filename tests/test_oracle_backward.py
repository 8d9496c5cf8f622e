"""Pins for the oracle's Alg. 2 (backward of one softmax block with entropy): finite differences of the
forward definitions, and the special cases that have closed forms."""
import numpy as np
import pytest

from oracle import vmonarch_oracle as O


def _problem(seed, nq, nk, d, with_dh=True):
    rng = np.random.default_rng(seed)
    Q, K, V = rng.normal(size=(nq, d)), rng.normal(size=(nk, d)), rng.normal(size=(nk, d))
    sc = 0.2 + rng.random(nq)
    dO = rng.normal(size=(nq, d))
    dH = rng.normal(size=nq) if with_dh else None
    return Q, K, V, sc, dO, dH


def _loss(Q, K, V, sc, dO, dH):
    Oo, lse, H = O.entropy_attention(Q, K, V, sc)
    return float((dO * Oo).sum() + (0.0 if dH is None else (dH * H).sum()))


@pytest.mark.parametrize("with_dh", [False, True])
@pytest.mark.parametrize("nq,nk,d", [(5, 7, 4), (3, 12, 6), (8, 2, 3)])
def test_backward_matches_central_differences(nq, nk, d, with_dh):
    Q, K, V, sc, dO, dH = _problem(10 * nq + nk, nq, nk, d, with_dh)
    Oo, lse, H = O.entropy_attention(Q, K, V, sc)
    dQ, dK, dV = O.entropy_attention_backward(Q, K, V, Oo, dO, lse, H, dH, sc)
    h = 1e-6
    for name, X, G in (("Q", Q, dQ), ("K", K, dK), ("V", V, dV)):
        num = np.zeros_like(X)
        for idx in np.ndindex(*X.shape):
            old = X[idx]
            X[idx] = old + h
            lp = _loss(Q, K, V, sc, dO, dH)
            X[idx] = old - h
            lm = _loss(Q, K, V, sc, dO, dH)
            X[idx] = old
            num[idx] = (lp - lm) / (2 * h)
        np.testing.assert_allclose(G, num, rtol=2e-6, atol=2e-7, err_msg=name)


def test_entropy_term_is_what_distinguishes_the_two_gradients():
    Q, K, V, sc, dO, dH = _problem(3, 6, 9, 5, True)
    Oo, lse, H = O.entropy_attention(Q, K, V, sc)
    with_h = O.entropy_attention_backward(Q, K, V, Oo, dO, lse, H, dH, sc)
    without = O.entropy_attention_backward(Q, K, V, Oo, dO, lse, H, None, sc)
    zero = O.entropy_attention_backward(Q, K, V, Oo, dO, lse, H, np.zeros(6), sc)
    assert np.abs(with_h[0] - without[0]).max() > 1e-3
    np.testing.assert_array_equal(with_h[2], without[2])      # dV has no entropy term
    for a, b in zip(without, zero):
        np.testing.assert_allclose(a, b, atol=1e-15)


def test_single_key_block_has_no_logit_gradient():
    """With one key the softmax is identically 1 and the entropy identically 0: dQ = dK = 0, dV = sum_i dO_i."""
    Q, K, V, sc, dO, dH = _problem(4, 5, 1, 3, True)
    Oo, lse, H = O.entropy_attention(Q, K, V, sc)
    dQ, dK, dV = O.entropy_attention_backward(Q, K, V, Oo, dO, lse, H, dH, sc)
    np.testing.assert_allclose(dQ, 0.0, atol=1e-14)
    np.testing.assert_allclose(dK, 0.0, atol=1e-14)
    np.testing.assert_allclose(dV[0], dO.sum(axis=0), atol=1e-14)


def test_gradient_is_orthogonal_to_a_common_shift_of_the_keys():
    """Adding one vector u to every key shifts every logit of row i by the same amount, which changes neither
    the softmax nor its entropy: sum_l dK[l] . u = 0 for every u, i.e. the key gradients sum to zero."""
    Q, K, V, sc, dO, dH = _problem(5, 7, 11, 4, True)
    Oo, lse, H = O.entropy_attention(Q, K, V, sc)
    _, dK, _ = O.entropy_attention_backward(Q, K, V, Oo, dO, lse, H, dH, sc)
    np.testing.assert_allclose(dK.sum(axis=0), 0.0, atol=1e-12)


def test_forward_statistics_against_brute_force():
    Q, K, V, sc, _, _ = _problem(6, 4, 9, 5)
    Oo, lse, H = O.entropy_attention(Q, K, V, sc)
    for i in range(4):
        z = np.array([sc[i] * float(Q[i] @ K[l]) for l in range(9)])
        p = np.exp(z) / np.exp(z).sum()
        assert abs(lse[i] - np.log(np.exp(z).sum())) < 1e-12
        assert abs(H[i] + (p * np.log(p)).sum()) < 1e-12
        np.testing.assert_allclose(Oo[i], p @ V, atol=1e-12)
