"""Pins for the gradient functions of the float64 oracle (CPU only).

Nothing here comes from the GPU path.  The gradient oracle is checked against (a) central
finite differences of the *forward* oracle, (b) reverse-mode automatic differentiation of a
forward written independently with dense torch operations, (c) closed forms for one and two
tokens, (d) structural facts: causality, linearity in dO, zero gradient of a constant loss,
block-size invariance where the forward has it.
"""
import numpy as np
import pytest
import torch

import oracle


def draw(n, d, dv, r, p, seed, unit=True):
    rng = np.random.default_rng(seed)
    Q, K = rng.standard_normal((n, d)), rng.standard_normal((n, d))
    if unit:
        Q /= np.linalg.norm(Q, axis=1, keepdims=True)
        K /= np.linalg.norm(K, axis=1, keepdims=True)
    V = rng.standard_normal((n, dv))
    dO = rng.standard_normal((n, dv))
    G = rng.standard_normal(oracle.g_len(d, r, p)) if p > 2 else None
    return Q, K, V, G, dO


def loss(Q, K, V, G, dO, p, r, b, feat, local):
    return float((oracle.attn_def(Q, K, V, G, p, r, b, feat=feat, local=local) * dO).sum())


def finite_difference(args, which, p, r, b, feat, local, h=1e-6):
    Q, K, V, G, dO = args
    base = [Q, K, V]
    out = np.zeros_like(base[which])
    for idx in np.ndindex(*out.shape):
        plus = [a.copy() for a in base]
        minus = [a.copy() for a in base]
        plus[which][idx] += h
        minus[which][idx] -= h
        out[idx] = (loss(*plus, G, dO, p, r, b, feat, local) - loss(*minus, G, dO, p, r, b, feat, local)) / (2 * h)
    return out


@pytest.mark.parametrize("p,feat,local", [
    (4, oracle.FEAT_SKETCH, oracle.LOCAL_EXACT), (4, oracle.FEAT_SKETCH, oracle.LOCAL_SKETCH),
    (8, oracle.FEAT_SKETCH, oracle.LOCAL_EXACT), (2, oracle.FEAT_SKETCH, oracle.LOCAL_EXACT),
    (16, oracle.FEAT_SKETCH, oracle.LOCAL_SKETCH), (4, oracle.FEAT_EXACT, oracle.LOCAL_EXACT)])
def test_gradient_matches_central_differences_of_the_forward_oracle(p, feat, local):
    n, d, dv, r, b = 8, 3, 2, 4, 4
    args = draw(n, d, dv, r, p, seed=10 + p)
    Q, K, V, G, dO = args
    dQ, dK, dV = oracle.attn_bwd(Q, K, V, G, dO, p, r, b, feat=feat, local=local)
    for which, got in enumerate((dQ, dK, dV)):
        want = finite_difference(args, which, p, r, b, feat, local)
        scale = max(1.0, np.abs(want).max())
        assert np.abs(got - want).max() <= 2e-6 * scale, (which, np.abs(got - want).max())


def torch_sketch(x, G, d, r, p):
    """Algorithm 1 with dense torch operations (written for this test; float64)."""
    deg = p // 2
    if deg == 1:
        return x
    nf = p // 2
    gf = [G[i * d * r:(i + 1) * d * r].reshape(d, r) for i in range(nf)]
    off = nf * d * r
    gi = [G[off + i * r * r: off + (i + 1) * r * r].reshape(r, r) for i in range(max(nf - 2, 0))]
    state = {"f": 0, "i": 0}

    def rec(degree):
        if degree == 1:
            return x
        m1 = rec(degree // 2)
        m2 = rec(degree // 2)
        if degree // 2 == 1:
            g1, g2 = gf[state["f"]], gf[state["f"] + 1]
            state["f"] += 2
        else:
            g1, g2 = gi[state["i"]], gi[state["i"] + 1]
            state["i"] += 2
        return (m1 @ g1) * (m2 @ g2) / np.sqrt(r)
    return rec(deg)


def torch_forward(Q, K, V, G, p, r, b, local_exact):
    n, d = Q.shape
    mq, mk = torch_sketch(Q, G, d, r, p), torch_sketch(K, G, d, r, p)
    W = (mq @ mk.T) ** 2
    if local_exact:
        blk = torch.arange(n) // b
        same = blk[:, None] == blk[None, :]
        W = torch.where(same, (Q @ K.T) ** p, W)
    W = torch.tril(W)
    return (W @ V) / (1.0 + W.sum(1, keepdim=True))


@pytest.mark.parametrize("p,local", [(4, oracle.LOCAL_EXACT), (8, oracle.LOCAL_EXACT),
                                     (4, oracle.LOCAL_SKETCH), (16, oracle.LOCAL_EXACT)])
def test_gradient_matches_autograd_of_an_independent_dense_forward(p, local):
    n, d, dv, r, b = 24, 6, 5, 8, 8
    Q, K, V, G, dO = draw(n, d, dv, r, p, seed=3 + p)
    tq, tk, tv = (torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (Q, K, V))
    tg = torch.tensor(G, dtype=torch.float64)
    out = torch_forward(tq, tk, tv, tg, p, r, b, local == oracle.LOCAL_EXACT)
    # the dense forward itself agrees with the oracle's forward
    np.testing.assert_allclose(out.detach().numpy(), oracle.attn_def(Q, K, V, G, p, r, b, local=local),
                               rtol=1e-10, atol=1e-12)
    (out * torch.tensor(dO)).sum().backward()
    dQ, dK, dV = oracle.attn_bwd(Q, K, V, G, dO, p, r, b, local=local)
    for got, want in ((dQ, tq.grad), (dK, tk.grad), (dV, tv.grad)):
        want = want.numpy()
        assert np.abs(got - want).max() <= 1e-10 * max(1.0, np.abs(want).max())


def test_one_token_closed_form():
    # o = w v / (1 + w), w = <q,k>^p: do/dv = w/(1+w), do/dw = v/(1+w)^2, dw/dq = p <q,k>^{p-1} k
    p = 4
    q, k = np.array([[0.6, -0.3, 0.2]]), np.array([[0.5, 0.4, -0.7]])
    v, dO = np.array([[1.5, -2.0]]), np.array([[0.3, 0.7]])
    s = float((q @ k.T)[0, 0])
    w = s ** p
    dw = float((dO * v).sum()) / (1 + w) ** 2
    dQ, dK, dV = oracle.attn_bwd(q, k, v, None, dO, p, 4, 1, feat=oracle.FEAT_EXACT)
    np.testing.assert_allclose(dV, dO * w / (1 + w), rtol=1e-13)
    np.testing.assert_allclose(dQ, dw * p * s ** (p - 1) * k, rtol=1e-12)
    np.testing.assert_allclose(dK, dw * p * s ** (p - 1) * q, rtol=1e-12)


def test_sketch_gradient_against_jacobian_by_differences():
    d, r = 5, 6
    for p in (4, 8, 16):
        rng = np.random.default_rng(p)
        X = rng.standard_normal((3, d)) * 0.7
        G = rng.standard_normal(oracle.g_len(d, r, p))
        dM = rng.standard_normal((3, r))
        got = oracle.sketch_bwd(X, G, r, p, dM)
        want = np.zeros_like(X)
        h = 1e-6
        for idx in np.ndindex(*X.shape):
            xp, xm = X.copy(), X.copy()
            xp[idx] += h
            xm[idx] -= h
            want[idx] = ((oracle.sketch(xp, G, r, p) - oracle.sketch(xm, G, r, p)) * dM).sum() / (2 * h)
        assert np.abs(got - want).max() <= 1e-6 * max(1.0, np.abs(want).max()), p
    # base case p = 2: m(x) = x
    np.testing.assert_array_equal(oracle.sketch_bwd(X, None, r, 2, X * 2.0), X * 2.0)


def test_structure_causality_linearity_constant_loss():
    n, d, dv, r, p, b = 16, 4, 3, 4, 4, 4
    Q, K, V, G, dO = draw(n, d, dv, r, p, seed=5)
    dQ, dK, dV = oracle.attn_bwd(Q, K, V, G, dO, p, r, b)
    # linear in dO
    dQ2, dK2, dV2 = oracle.attn_bwd(Q, K, V, G, -2.5 * dO, p, r, b)
    np.testing.assert_allclose(dQ2, -2.5 * dQ, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(dV2, -2.5 * dV, rtol=1e-12, atol=1e-14)
    # causality: a loss on rows < m cannot reach queries, keys or values at positions >= m
    m = 9
    dOm = dO.copy()
    dOm[m:] = 0.0
    dQm, dKm, dVm = oracle.attn_bwd(Q, K, V, G, dOm, p, r, b)
    assert np.abs(dQm[m:]).max() == 0 and np.abs(dKm[m:]).max() == 0 and np.abs(dVm[m:]).max() == 0
    # a query row only feels the loss on its own row
    dOi = np.zeros_like(dO)
    dOi[5] = dO[5]
    dQi, _, _ = oracle.attn_bwd(Q, K, V, G, dOi, p, r, b)
    assert np.abs(np.delete(dQi, 5, axis=0)).max() == 0
    np.testing.assert_allclose(dQi[5], oracle.attn_bwd(Q, K, V, G, dO, p, r, b)[0][5], rtol=1e-12)
    # V == constant vector c: o_i = c (1 - 1/D_i), so for dO orthogonal to c every gradient
    # with respect to Q and K vanishes
    c = np.array([1.0, 2.0, -1.0])
    Vc = np.tile(c, (n, 1))
    dOo = np.tile(np.array([2.0, 0.0, 2.0]), (n, 1))       # <dOo, c> = 0
    dQc, dKc, _ = oracle.attn_bwd(Q, K, Vc, G, dOo, p, r, b)
    assert np.abs(dQc).max() <= 1e-13 and np.abs(dKc).max() <= 1e-13


def test_block_size_invariance_of_the_gradient_where_the_forward_has_it():
    n, d, dv, r, p = 16, 4, 3, 4, 4
    Q, K, V, G, dO = draw(n, d, dv, r, p, seed=6)
    ref = oracle.attn_bwd(Q, K, V, G, dO, p, r, n, local=oracle.LOCAL_SKETCH)
    for b in (1, 2, 4, 8):
        got = oracle.attn_bwd(Q, K, V, G, dO, p, r, b, local=oracle.LOCAL_SKETCH)
        for x, y in zip(got, ref):
            np.testing.assert_allclose(x, y, rtol=1e-11, atol=1e-13)
    # with exact in-block weights the gradient legitimately depends on b
    a = oracle.attn_bwd(Q, K, V, G, dO, p, r, 4)[0]
    c = oracle.attn_bwd(Q, K, V, G, dO, p, r, 8)[0]
    assert np.abs(a - c).max() > 1e-6


def test_batch_driver_matches_single_units():
    B, H, n, d, dv, r, p, b = 2, 3, 8, 4, 3, 4, 4, 4
    rng = np.random.default_rng(8)
    Q, K = rng.standard_normal((B, H, n, d)), rng.standard_normal((B, H, n, d))
    V, dO = rng.standard_normal((B, H, n, dv)), rng.standard_normal((B, H, n, dv))
    G = rng.standard_normal((H, oracle.g_len(d, r, p)))
    dQ, dK, dV, threads = oracle.attn_bwd_batch(Q, K, V, G, dO, p, r, b)
    assert threads >= 1
    for bi in range(B):
        for h in range(H):
            want = oracle.attn_bwd(Q[bi, h], K[bi, h], V[bi, h], G[h], dO[bi, h], p, r, b)
            for got, w in zip((dQ[bi, h], dK[bi, h], dV[bi, h]), want):
                np.testing.assert_allclose(got, w, rtol=1e-13, atol=1e-15)


def test_row_restricted_gradient_against_finite_differences_and_the_full_sums():
    """attn_bwd_rows: dQ rows of listed queries and dK / dV rows whose whole tail of queries is
    listed.  Pinned two ways: against the full pair loop (itself pinned above), and directly
    against central differences of the forward oracle for a loss that only involves the listed
    output rows (dO zero elsewhere makes the restricted sums the whole gradient)."""
    rng = np.random.default_rng(77)
    n, d, dv, r, p, b = 24, 6, 5, 4, 4, 8
    Q, K = rng.standard_normal((n, d)) * 0.6, rng.standard_normal((n, d)) * 0.6
    V, dO = rng.standard_normal((n, dv)), rng.standard_normal((n, dv))
    G = rng.standard_normal(oracle.g_len(d, r, p))
    tail = 10                                           # keys >= tail have every later query listed
    rows = [3, 7] + list(range(tail, n))
    dQ, dK, dV = oracle.attn_bwd_rows(Q, K, V, G, dO, p, r, b, rows)
    fQ, fK, fV = oracle.attn_bwd(Q, K, V, G, dO, p, r, b)
    np.testing.assert_allclose(dQ[rows], fQ[rows], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(dK[tail:], fK[tail:], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(dV[tail:], fV[tail:], rtol=1e-12, atol=1e-14)
    assert not np.allclose(dK[:tail], fK[:tail])        # earlier keys are partial sums, as documented
    # loss over the listed rows only: its full gradient is what the restricted call returns
    dO_m = np.zeros_like(dO)
    dO_m[rows] = dO[rows]
    loss = lambda q_, k_, v_: float((oracle.attn_def(q_, k_, v_, G, p, r, b) * dO_m).sum())
    eps = 1e-6
    for (name, X, got) in (("Q", Q, dQ), ("K", K, dK), ("V", V, dV)):
        for (i, c) in ((3, 1), (12, 0), (n - 1, 2), (5, 3)):
            Xp, Xm = X.copy(), X.copy()
            Xp[i, c] += eps
            Xm[i, c] -= eps
            args_p = {"Q": (Xp, K, V), "K": (Q, Xp, V), "V": (Q, K, Xp)}[name]
            args_m = {"Q": (Xm, K, V), "K": (Q, Xm, V), "V": (Q, K, Xm)}[name]
            fd = (loss(*args_p) - loss(*args_m)) / (2 * eps)
            np.testing.assert_allclose(got[i, c], fd, rtol=2e-6, atol=1e-8, err_msg="%s[%d,%d]" % (name, i, c))
