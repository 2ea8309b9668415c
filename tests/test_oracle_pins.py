"""Pins for the float64 oracle: every check here compares it with something the paper
or plain mathematics fixes (hand-worked cases, brute force, closed forms, invariants),
never with the GPU path and never with a retyped copy of the oracle's own loops."""
import json
import os

import numpy as np
import pytest

import oracle
from oracle import FEAT_EXACT, FEAT_SKETCH, LOCAL_EXACT, LOCAL_SKETCH

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "hand_worked.json")))


def unit_rows(rng, n, d):
    x = rng.standard_normal((n, d))
    return x / np.linalg.norm(x, axis=1, keepdims=True)


def brute_poly_attention(Q, K, V, p):
    """Section 2.1/3: D^-1 lt((QK^T)^p) V with D = diag(1 + lt((QK^T)^p) 1), in numpy."""
    W = np.tril((Q @ K.T) ** p)
    return (W @ V) / (1.0 + W.sum(1, keepdims=True))


def brute_weights_attention(W, V):
    W = np.tril(W)
    return (W @ V) / (1.0 + W.sum(1, keepdims=True))


# ---------------------------------------------------------------- hand-worked cases
def test_matrix_counts_match_theorem():
    L = oracle.lib()
    for p, (nf, ni) in ((int(k), v) for k, v in GOLD["matrix_counts"].items() if k[0] != "_"):
        assert L.psf_oracle_num_g_first(p) == nf
        assert L.psf_oracle_num_g_inner(p) == ni


def test_sketch_p4_hand_worked():
    g = GOLD["sketch_p4"]
    G = np.concatenate([np.ravel(g["G1"]), np.ravel(g["G2"])])
    M = oracle.sketch(np.array(g["x"]), G, g["r"], g["p"])
    np.testing.assert_allclose(M * np.sqrt(2.0), g["m_times_sqrt2"], rtol=0, atol=1e-14)
    np.testing.assert_allclose(oracle.self_tensor(M) * 2.0, g["phi_times_2"], rtol=0, atol=1e-14)


def test_sketch_p8_hand_worked():
    g = GOLD["sketch_p8"]
    G = np.concatenate([np.ravel(g[k]) for k in ("G1", "G2", "G3", "G4", "G5", "G6")])
    M = oracle.sketch(np.array(g["x"]), G, g["r"], g["p"])
    np.testing.assert_allclose(M * np.sqrt(2.0), g["m_times_sqrt2"], rtol=0, atol=1e-13)


@pytest.mark.parametrize("fn", ["def", "block"])
def test_attention_n2_hand_worked(fn):
    g = GOLD["attention_n2"]
    Q, K, V = np.array(g["q"]), np.array(g["k"]), np.array(g["v"])
    want = np.array(g["o_numer"]) / np.array(g["o_denom"])
    for b in (1, 2):
        if fn == "def":
            O, W = oracle.attn_def(Q, K, V, None, g["p"], 1, b, feat=FEAT_EXACT,
                                   return_weights=True)
            np.testing.assert_allclose(W, g["weights"], atol=1e-15)
        else:
            O = oracle.attn_block(Q, K, V, None, g["p"], 1, b, feat=FEAT_EXACT)
        np.testing.assert_allclose(O[:, 0], want, atol=1e-15)


# ---------------------------------------------------------------- P1 brute force, exact features
@pytest.mark.parametrize("d,p", [(4, 4), (3, 4), (8, 2), (2, 8), (5, 2)])
def test_exact_features_vs_brute_force(d, p):
    rng = np.random.default_rng(10 + d + p)
    n, b = 48, 8
    Q, K, V = unit_rows(rng, n, d) * 1.3, unit_rows(rng, n, d) * 0.9, rng.standard_normal((n, 5))
    want = brute_poly_attention(Q, K, V, p)
    got_block = oracle.attn_block(Q, K, V, None, p, 1, b, feat=FEAT_EXACT)   # explicit x^{(x)p}
    got_def = oracle.attn_def(Q, K, V, None, p, 1, b, feat=FEAT_EXACT)
    np.testing.assert_allclose(got_block, want, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(got_def, want, rtol=1e-11, atol=1e-13)


def test_power_tensor_inner_product_identity():
    # <x,y>^p = <x^{(x)p}, y^{(x)p}>  (Section 2.2) and the Kronecker index order (Section 1.2)
    rng = np.random.default_rng(3)
    X, Y = rng.standard_normal((6, 3)), rng.standard_normal((6, 3))
    for p in (1, 2, 3, 4):
        PX, PY = oracle.power_tensor(X, p), oracle.power_tensor(Y, p)
        np.testing.assert_allclose((PX * PY).sum(1), (X * Y).sum(1) ** p, rtol=1e-12)
    P3 = oracle.power_tensor(X, 3)
    np.testing.assert_allclose(P3, np.einsum("ia,ib,ic->iabc", X, X, X).reshape(6, -1), rtol=1e-14)
    np.testing.assert_allclose(oracle.self_tensor(X), np.einsum("ia,ib->iab", X, X).reshape(6, -1),
                               rtol=1e-14)


# ---------------------------------------------------------------- P2 block-size invariance
@pytest.mark.parametrize("feat,local,p", [(FEAT_EXACT, LOCAL_EXACT, 4), (FEAT_SKETCH, LOCAL_SKETCH, 4),
                                          (FEAT_SKETCH, LOCAL_SKETCH, 8)])
def test_block_size_invariance(feat, local, p):
    rng = np.random.default_rng(21)
    n, d, r = 64, 4, 6
    Q, K, V = unit_rows(rng, n, d), unit_rows(rng, n, d), rng.standard_normal((n, 3))
    G = rng.standard_normal(oracle.g_len(d, r, p))
    outs = [oracle.attn_block(Q, K, V, G, p, r, b, feat=feat, local=local)
            for b in (1, 2, 4, 8, 16, 32, 64)]
    for o in outs[1:]:
        np.testing.assert_allclose(o, outs[0], rtol=1e-10, atol=1e-13)


def test_local_exact_depends_on_block_size_as_defined():
    # With exact in-block weights the set of exact pairs is defined by b (Section 3.2), so the
    # output changes with b, and equals brute force over the mixed weight matrix.
    rng = np.random.default_rng(22)
    n, d, r, p = 32, 6, 5, 4
    Q, K, V = unit_rows(rng, n, d), unit_rows(rng, n, d), rng.standard_normal((n, 4))
    G = rng.standard_normal(oracle.g_len(d, r, p))
    MQ, MK = oracle.sketch(Q, G, r, p), oracle.sketch(K, G, r, p)
    outs = {}
    for b in (4, 16):
        blk = np.arange(n) // b
        W = np.where(blk[:, None] == blk[None, :], (Q @ K.T) ** p, (MQ @ MK.T) ** 2)
        want = brute_weights_attention(W, V)
        for fn in (oracle.attn_def, oracle.attn_block):
            got = fn(Q, K, V, G, p, r, b, feat=FEAT_SKETCH, local=LOCAL_EXACT)
            np.testing.assert_allclose(got, want, rtol=1e-10, atol=1e-13)
        outs[b] = want
    assert np.abs(outs[4] - outs[16]).max() > 1e-3


# ---------------------------------------------------------------- P3 single block
@pytest.mark.parametrize("d,p", [(64, 4), (128, 8)])
def test_single_block_is_quadratic_polynomial_attention(d, p):
    rng = np.random.default_rng(31)
    n, r = 40, 8
    Q, K, V = unit_rows(rng, n, d), unit_rows(rng, n, d), rng.standard_normal((n, 7))
    want = brute_poly_attention(Q, K, V, p)
    for seed in (0, 1):                        # independent of the sketch matrices
        G = np.random.default_rng(seed).standard_normal(oracle.g_len(d, r, p))
        got = oracle.attn_def(Q, K, V, G, p, r, n, feat=FEAT_SKETCH, local=LOCAL_EXACT)
        np.testing.assert_allclose(got, want, rtol=1e-11, atol=1e-14)


# ---------------------------------------------------------------- P4 definition == block algorithm
@pytest.mark.parametrize("local", [LOCAL_EXACT, LOCAL_SKETCH])
@pytest.mark.parametrize("p", [4, 8, 16])
def test_definition_equals_block_algorithm(local, p):
    rng = np.random.default_rng(41 + p)
    n, d, r, b = 48, 5, 7, 12
    Q, K, V = unit_rows(rng, n, d), unit_rows(rng, n, d), rng.standard_normal((n, 3))
    G = rng.standard_normal(oracle.g_len(d, r, p))
    o_def = oracle.attn_def(Q, K, V, G, p, r, b, local=local)
    o_exp = oracle.attn_def(Q, K, V, G, p, r, b, local=local, explicit_features=True)
    o_blk = oracle.attn_block(Q, K, V, G, p, r, b, local=local)
    np.testing.assert_allclose(o_exp, o_def, rtol=1e-10, atol=1e-13)   # <m,m>^2 = <m(x)m, m(x)m>
    np.testing.assert_allclose(o_blk, o_def, rtol=1e-10, atol=1e-13)
    rows = [0, 5, 11, 12, 47]
    np.testing.assert_allclose(oracle.attn_def(Q, K, V, G, p, r, b, local=local, rows=rows),
                               o_def[rows], rtol=0, atol=0)


def test_sketched_weights_against_numpy_for_documented_g_layout():
    # Pins the *interface*: G is [d x r] row-major, G1 then G2; weights are (m_q . m_k)^2.
    rng = np.random.default_rng(43)
    n, d, r, p = 20, 6, 4, 4
    Q, K, V = unit_rows(rng, n, d), unit_rows(rng, n, d), rng.standard_normal((n, 2))
    G = rng.standard_normal(2 * d * r)
    G1, G2 = G[:d * r].reshape(d, r), G[d * r:].reshape(d, r)
    MQ = (Q @ G1) * (Q @ G2) / np.sqrt(r)
    MK = (K @ G1) * (K @ G2) / np.sqrt(r)
    np.testing.assert_allclose(oracle.sketch(Q, G, r, p), MQ, rtol=1e-12, atol=1e-15)
    O, W = oracle.attn_def(Q, K, V, G, p, r, n // 4, local=LOCAL_SKETCH, return_weights=True)
    np.testing.assert_allclose(W, np.tril((MQ @ MK.T) ** 2), rtol=1e-11, atol=1e-15)
    np.testing.assert_allclose(O, brute_weights_attention(W, V), rtol=1e-11, atol=1e-14)


# ---------------------------------------------------------------- P5 p = 2
def test_degree_two_is_deterministic_and_exact():
    # Algorithm 1's base case: degree 1 returns its input, so phi'(x) = x (x) x and the
    # "sketched" attention is exactly degree-2 polynomial attention.
    rng = np.random.default_rng(51)
    n, d = 32, 64
    Q, K, V = unit_rows(rng, n, d), unit_rows(rng, n, d), rng.standard_normal((n, 3))
    np.testing.assert_array_equal(oracle.sketch(Q, None, 9, 2), Q)
    want = brute_poly_attention(Q, K, V, 2)
    for local in (LOCAL_EXACT, LOCAL_SKETCH):
        np.testing.assert_allclose(oracle.attn_def(Q, K, V, None, 2, 9, 8, local=local), want,
                                   rtol=1e-11, atol=1e-14)
    np.testing.assert_allclose(oracle.attn_block(Q, K, V, None, 2, 9, 8, local=LOCAL_SKETCH), want,
                               rtol=1e-10, atol=1e-13)


# ---------------------------------------------------------------- P6 non-negativity, convex hull
@pytest.mark.parametrize("p", [4, 8])
def test_nonnegative_weights_and_convex_hull(p):
    rng = np.random.default_rng(61)
    n, d, r, b = 64, 8, 4, 16
    Q, K = unit_rows(rng, n, d) * 2.0, unit_rows(rng, n, d) * 2.0
    V = rng.standard_normal((n, 5))
    G = rng.standard_normal(oracle.g_len(d, r, p))
    for local in (LOCAL_EXACT, LOCAL_SKETCH):
        O, W = oracle.attn_def(Q, K, V, G, p, r, b, local=local, return_weights=True)
        assert (W >= 0).all() and np.triu(W, 1).max() == 0.0          # Theorem 1.1 item 1
        running_max = np.maximum.accumulate(np.abs(V).max(1))
        assert (np.abs(O).max(1) <= running_max + 1e-12).all()


# ---------------------------------------------------------------- P7 closed forms
def test_closed_forms_row0_ones_linearity_homogeneity():
    rng = np.random.default_rng(71)
    n, d, r, b, p = 40, 6, 5, 8, 4
    Q, K, V = unit_rows(rng, n, d), unit_rows(rng, n, d), rng.standard_normal((n, 3))
    G = rng.standard_normal(oracle.g_len(d, r, p))
    O, W = oracle.attn_def(Q, K, V, G, p, r, b, return_weights=True)
    w00 = float(Q[0] @ K[0]) ** p                      # same block -> exact weight
    np.testing.assert_allclose(O[0], w00 * V[0] / (1.0 + w00), rtol=1e-12)
    ones = oracle.attn_def(Q, K, np.ones((n, 1)), G, p, r, b)
    np.testing.assert_allclose(ones[:, 0], 1.0 - 1.0 / (1.0 + W.sum(1)), rtol=1e-12)
    V2 = rng.standard_normal((n, 3))
    O2 = oracle.attn_def(Q, K, V2, G, p, r, b)
    np.testing.assert_allclose(oracle.attn_def(Q, K, 2 * V - 3 * V2, G, p, r, b), 2 * O - 3 * O2,
                               rtol=1e-10, atol=1e-13)
    for pp in (4, 8, 16):                              # m(a x) = a^{p/2} m(x)
        Gp = rng.standard_normal(oracle.g_len(d, r, pp))
        np.testing.assert_allclose(oracle.sketch(1.5 * Q, Gp, r, pp),
                                   1.5 ** (pp // 2) * oracle.sketch(Q, Gp, r, pp), rtol=1e-11)


# ---------------------------------------------------------------- P8 Monte-Carlo moments
def _mc_pairs(c, d, r, p, seeds, rng):
    x = np.zeros(d); x[0] = 1.0
    y = np.zeros(d); y[0] = c; y[1] = np.sqrt(1 - c * c)
    X = np.stack([x, y])
    first = np.empty(seeds)
    glen = oracle.g_len(d, r, p)
    for s in range(seeds):
        M = oracle.sketch(X, rng.standard_normal(glen), r, p)
        first[s] = M[0] @ M[1]
    return first


@pytest.mark.parametrize("c", [0.0, 0.5, 1.0])
def test_monte_carlo_moments_degree4(c):
    r, d, seeds = 8, 5, 20000
    rng = np.random.default_rng(int(81 + 10 * c))
    s = _mc_pairs(c, d, r, 4, seeds, rng)
    want1 = c ** 2
    want2 = c ** 4 + ((1 + 2 * c ** 2) ** 2 - c ** 4) / r
    se1 = s.std(ddof=1) / np.sqrt(seeds)
    se2 = (s ** 2).std(ddof=1) / np.sqrt(seeds)
    assert abs(s.mean() - want1) < 4 * se1 + 1e-12          # <m(x),m(y)> is unbiased for c^2
    assert abs((s ** 2).mean() - want2) < 4.5 * se2 + 1e-12  # <phi',phi'> = <m,m>^2 carries var/r
    # and the estimator would not pass with a missing or doubled sqrt(1/r) at the node
    assert abs(s.mean() * r - want1) > 4 * se1 * r or c == 0.0


def test_monte_carlo_first_moment_degree8_and_bias_shrinks_with_r():
    # degree-4 sketch (p = 8): unbiased for c^4 only if the two halves use independent Gaussians
    c, d, seeds = 0.8, 4, 30000
    rng = np.random.default_rng(88)
    s = _mc_pairs(c, d, 16, 8, seeds, rng)
    batch = s.reshape(100, -1).mean(1)                       # batch means: heavy tails
    assert abs(batch.mean() - c ** 4) < 4 * batch.std(ddof=1) / np.sqrt(batch.size)
    # E<phi',phi'> -> c^p as r grows (degree 4, closed form above)
    errs = []
    for r in (4, 64):
        t = _mc_pairs(c, d, r, 4, 4000, rng)
        errs.append(abs((t ** 2).mean() - c ** 4))
    assert errs[1] < errs[0] / 4


# ---------------------------------------------------------------- P9 approximate matrix product slope
def test_amm_error_decays_like_inverse_sqrt_r():
    # Theorem 2.3: the degree-p/2 sketch has Frobenius error eps ~ r^-1/2 (slope -1/2 exactly,
    # its variance is 1/r per entry); Theorem 2.5: after self-tensoring the error is at most
    # sqrt(5) eps, so it must fall at least that fast.  The constants are not given: slopes only.
    rng = np.random.default_rng(91)
    n, d, p = 48, 8, 4
    Q, K = unit_rows(rng, n, d), unit_rows(rng, n, d)
    half, full = (Q @ K.T) ** (p // 2), (Q @ K.T) ** p
    rs, e_half, e_full = [4, 16, 64, 256], [], []
    for r in rs:
        a, c = [], []
        for _ in range(8):
            G = rng.standard_normal(oracle.g_len(d, r, p))
            MQ, MK = oracle.sketch(Q, G, r, p), oracle.sketch(K, G, r, p)
            a.append(np.linalg.norm(MQ @ MK.T - half) / n)    # ||Q^{(x)p/2}||_F = sqrt(n) for unit rows
            feat = oracle.self_tensor(MQ) @ oracle.self_tensor(MK).T if r <= 16 else (MQ @ MK.T) ** 2
            c.append(np.linalg.norm(feat - full) / n)
        e_half.append(np.mean(a))
        e_full.append(np.mean(c))
    s_half = np.polyfit(np.log(rs), np.log(e_half), 1)[0]
    s_full = np.polyfit(np.log(rs), np.log(e_full), 1)[0]
    assert -0.6 < s_half < -0.4, (s_half, e_half)
    assert s_full < -0.4, (s_full, e_full)
