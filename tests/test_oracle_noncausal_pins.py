"""Pins of the non-causal oracle (Section 2.2: Attn = D^-1 phi'(Q) phi'(K)^T V with
D = diag(1 + phi'(Q) phi'(K)^T 1)) against things that are not the oracle: the matrix formula
typed out in numpy on explicit Kronecker features, the already pinned causal oracle on the one
row where both coincide, and structural facts (key order does not matter; one key gives a
closed form; exact features give polynomial attention)."""
import numpy as np
import pytest

import oracle


def draw(nq, nk, d, dv, r, p, seed):
    rng = np.random.default_rng(seed)
    Q, K = rng.standard_normal((nq, d)) * 0.7, rng.standard_normal((nk, d)) * 0.7
    V = rng.standard_normal((nk, dv))
    G = rng.standard_normal(oracle.g_len(d, r, p)) if p > 2 else None
    return Q, K, V, G


@pytest.mark.parametrize("p,r", [(2, 5), (4, 6), (8, 4)])
def test_matrix_formula_with_explicit_kronecker_features(p, r):
    Q, K, V, G = draw(7, 11, 5, 3, r, p, seed=p)
    mq, mk = oracle.sketch(Q, G, r, p), oracle.sketch(K, G, r, p)
    phi = lambda m: np.einsum("ia,ib->iab", m, m).reshape(m.shape[0], -1)      # m (x) m, index a r + b
    A = phi(mq) @ phi(mk).T
    assert (A >= -1e-12).all()
    want = (A @ V) / (1.0 + A @ np.ones((K.shape[0], 1)))
    np.testing.assert_allclose(oracle.attn_noncausal(Q, K, V, G, p, r), want, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(oracle.attn_noncausal(Q, K, V, G, p, r, explicit_features=True), want,
                               rtol=1e-11, atol=1e-13)


def test_last_row_of_the_causal_oracle_sees_every_key_too():
    n, d, dv, r, p = 16, 6, 4, 5, 4
    Q, K, V, G = draw(n, n, d, dv, r, p, seed=3)
    causal = oracle.attn_def(Q, K, V, G, p, r, 4, local=oracle.LOCAL_SKETCH)
    np.testing.assert_allclose(oracle.attn_noncausal(Q, K, V, G, p, r)[n - 1], causal[n - 1], rtol=1e-12, atol=1e-14)
    # and an earlier row differs: it must not be masked
    assert np.abs(oracle.attn_noncausal(Q, K, V, G, p, r)[0] - causal[0]).max() > 1e-3


def test_key_order_does_not_matter_and_queries_are_independent():
    Q, K, V, G = draw(6, 13, 5, 3, 4, 4, seed=5)
    base = oracle.attn_noncausal(Q, K, V, G, 4, 4)
    perm = np.random.default_rng(0).permutation(K.shape[0])
    np.testing.assert_allclose(oracle.attn_noncausal(Q, K[perm], V[perm], G, 4, 4), base, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(oracle.attn_noncausal(Q[2:4], K, V, G, 4, 4), base[2:4], rtol=1e-13, atol=1e-15)


def test_single_key_closed_form_and_exact_features():
    Q, K, V, G = draw(5, 1, 4, 3, 3, 4, seed=9)
    w = (oracle.sketch(Q, G, 3, 4) @ oracle.sketch(K, G, 3, 4).T) ** 2        # n x 1
    np.testing.assert_allclose(oracle.attn_noncausal(Q, K, V, G, 4, 3), (w / (1.0 + w)) * V, rtol=1e-12)
    Q, K, V, _ = draw(6, 9, 4, 3, 3, 4, seed=10)
    A = (Q @ K.T) ** 4
    np.testing.assert_allclose(oracle.attn_noncausal(Q, K, V, None, 4, 3, feat=oracle.FEAT_EXACT),
                               (A @ V) / (1.0 + A.sum(1, keepdims=True)), rtol=1e-12)


def test_with_learned_sketches_is_the_same_formula_on_those_sketches():
    d, r = 8, 4
    rng = np.random.default_rng(2)
    Q, K, V = rng.standard_normal((5, d)), rng.standard_normal((7, d)), rng.standard_normal((7, 3))
    P = rng.standard_normal(oracle.learned_len(d, r, 4)) * 0.3
    mq, mk = oracle.sketch_learned(Q, P, r, 4), oracle.sketch_learned(K, P, r, 4)
    A = (mq @ mk.T) ** 2
    np.testing.assert_allclose(oracle.attn_noncausal(Q, K, V, P, 4, r, learned=True),
                               (A @ V) / (1.0 + A.sum(1, keepdims=True)), rtol=1e-12)
