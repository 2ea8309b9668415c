"""Pins for the learned-sketch oracle (Algorithm 2, Appendix D), CPU only.

Checked against: the same network assembled from torch's own layer_norm / gelu / matmul
routines (a re-call of library routines for every step), structural facts that follow from the
definition (parameter count of the appendix, invariance of f to positive rescaling of its input
because of the leading layer normalisation, the tanh bound |m| < sqrt(r), the small-signal limit
sqrt(r) tanh(z / sqrt(r)) -> z), the recursion order for p = 8, and the base case p = 2."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle


def draw_params(d, r, p, seed, w4_scale=1.0):
    """Synthetic parameters in the documented order; dense matrices N(0, 1/fan_in)."""
    rng = np.random.default_rng(seed)
    nets = []
    widths = [d] * (p // 2) + [r] * max(p // 2 - 2, 0)
    # consumption order of the recursion for p = 4: f1, f2 (input d); for p = 8: the two
    # first-level nodes (input d, d | d, d) and then the node (input r, r)
    for win in widths:
        hid = 8 * r
        nets.append(dict(
            g1=1.0 + 0.1 * rng.standard_normal(win), b1=0.1 * rng.standard_normal(win),
            W1=rng.standard_normal((win, hid)) / np.sqrt(win),
            g2=1.0 + 0.1 * rng.standard_normal(hid), b2=0.1 * rng.standard_normal(hid),
            W2=rng.standard_normal((hid, r)) / np.sqrt(hid),
            W3=rng.standard_normal((r, hid)) / np.sqrt(r),
            W4=w4_scale * rng.standard_normal((hid, r)) / np.sqrt(hid)))
    flat = np.concatenate([np.concatenate([n[k].reshape(-1) for k in ("g1", "b1", "W1", "g2", "b2", "W2", "W3", "W4")])
                           for n in nets])
    return nets, flat


def torch_net(x, n):
    t = lambda a: torch.tensor(a, dtype=torch.float64)
    u = F.layer_norm(x, (x.shape[-1],), t(n["g1"]), t(n["b1"]), eps=1e-6)
    h1 = F.gelu(u @ t(n["W1"]), approximate="tanh")
    v = F.layer_norm(h1, (h1.shape[-1],), t(n["g2"]), t(n["b2"]), eps=1e-6)
    h2 = v @ t(n["W2"])
    h3 = F.gelu(h2 @ t(n["W3"]), approximate="tanh")
    return h3 @ t(n["W4"])


def test_parameter_count_is_the_appendix_count_plus_layer_norms():
    for d, r in ((64, 64), (64, 32), (128, 64)):
        # p = 4: two networks of 8 h r + 24 r^2 dense parameters each (Appendix D)
        dense = 2 * (8 * d * r + 24 * r * r)
        norms = 2 * (2 * d + 2 * 8 * r)
        assert oracle.learned_len(d, r, 4) == dense + norms
        # p = 8: p - 2 = 6 networks, four on the input and two on r-vectors (32 r^2 each)
        dense8 = 4 * (8 * d * r + 24 * r * r) + 2 * (32 * r * r)
        norms8 = 4 * (2 * d + 16 * r) + 2 * (2 * r + 16 * r)
        assert oracle.learned_len(d, r, 8) == dense8 + norms8
    assert oracle.learned_len(64, 64, 2) == 0


@pytest.mark.parametrize("d,r", [(12, 4), (16, 8), (64, 16)])
def test_degree_4_against_torch_library_routines(d, r):
    nets, flat = draw_params(d, r, 4, seed=d + r)
    X = np.random.default_rng(1).standard_normal((7, d))
    x = torch.tensor(X)
    want = np.sqrt(r) * torch.tanh(torch_net(x, nets[0]) * torch_net(x, nets[1]) / np.sqrt(r))
    np.testing.assert_allclose(oracle.sketch_learned(X, flat, r, 4), want.numpy(), rtol=1e-10, atol=1e-12)


def test_degree_8_recursion_order_against_torch():
    d, r = 10, 6
    nets, flat = draw_params(d, r, 8, seed=5)
    # draw_params lists the four input-width networks first, then the two r-width ones; the
    # recursion consumes: left node (nets 0, 1), right node (nets 2, 3), then the root's pair
    X = np.random.default_rng(2).standard_normal((5, d))
    x = torch.tensor(X)
    node = lambda a, b2, inp: np.sqrt(r) * torch.tanh(torch_net(inp, a) * torch_net(inp, b2) / np.sqrt(r))
    # parameters are stored in consumption order: rebuild the flat vector accordingly
    order = [nets[0], nets[1], nets[2], nets[3], nets[4], nets[5]]
    flat = np.concatenate([np.concatenate([n[k].reshape(-1) for k in ("g1", "b1", "W1", "g2", "b2", "W2", "W3", "W4")])
                           for n in order])
    m1, m2 = node(nets[0], nets[1], x), node(nets[2], nets[3], x)
    want = np.sqrt(r) * torch.tanh(torch_net(m1, nets[4]) * torch_net(m2, nets[5]) / np.sqrt(r))
    np.testing.assert_allclose(oracle.sketch_learned(X, flat, r, 8), want.numpy(), rtol=1e-10, atol=1e-12)


def test_structure_scale_invariance_bound_and_small_signal_limit():
    d, r = 16, 8
    nets, flat = draw_params(d, r, 4, seed=9)
    X = np.random.default_rng(3).standard_normal((6, d))
    M = oracle.sketch_learned(X, flat, r, 4)
    # the leading layer normalisation removes positive rescaling of the input (up to its eps)
    np.testing.assert_allclose(oracle.sketch_learned(37.0 * X, flat, r, 4), M, rtol=1e-5, atol=1e-6)
    # tanh keeps every entry inside [-sqrt(r), sqrt(r)] however large the networks' outputs are
    big = oracle.sketch_learned(X, draw_params(d, r, 4, seed=9, w4_scale=1e3)[1], r, 4)
    assert np.abs(big).max() <= np.sqrt(r) and np.abs(big).max() > 0.9 * np.sqrt(r)
    # small signals pass through: sqrt(r) tanh(z / sqrt(r)) = z + O(z^3)
    tiny_nets, tiny = draw_params(d, r, 4, seed=9, w4_scale=1e-3)
    x = torch.tensor(X)
    z = (torch_net(x, tiny_nets[0]) * torch_net(x, tiny_nets[1])).numpy()
    np.testing.assert_allclose(oracle.sketch_learned(X, tiny, r, 4), z, rtol=1e-6, atol=1e-15)
    # base case p = 2: the sketch is the identity
    np.testing.assert_array_equal(oracle.sketch_learned(X, None, r, 2), X)


def test_attention_with_learned_sketches_is_the_definition_on_those_sketches():
    n, d, dv, r, b = 24, 12, 5, 4, 8
    _, flat = draw_params(d, r, 4, seed=11)
    rng = np.random.default_rng(4)
    Q, K, V = rng.standard_normal((n, d)), rng.standard_normal((n, d)), rng.standard_normal((n, dv))
    mq, mk = oracle.sketch_learned(Q, flat, r, 4), oracle.sketch_learned(K, flat, r, 4)
    W = (mq @ mk.T) ** 2
    blk = np.arange(n) // b
    W = np.tril(np.where(blk[:, None] == blk[None, :], (Q @ K.T) ** 4, W))
    want = (W @ V) / (1.0 + W.sum(1, keepdims=True))
    np.testing.assert_allclose(oracle.attn_def(Q, K, V, flat, 4, r, b, learned=True), want, rtol=1e-11, atol=1e-13)
