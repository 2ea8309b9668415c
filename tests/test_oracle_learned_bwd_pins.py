"""Pins for the gradient of the learned sketch (Algorithm 2) and of attention through it, CPU only.

The oracle's reverse pass (layer normalisation, gelu, tanh, the recursion) is checked against
two things that share none of its code: central finite differences of the forward oracle, in
float64, with respect to inputs and to every kind of parameter, and reverse-mode automatic
differentiation of the same network assembled from torch's own layer_norm / gelu / matmul /
tanh (the assembly test_oracle_learned_pins.py checks against the forward oracle)."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from test_oracle_learned_pins import draw_params


def torch_sketch(x, nets, r, p):
    """LearnablePolysketchWithNegativity(x, r, p/2) from torch routines; nets in the order the
    recursion consumes them: for p = 8 the four input-width networks come first in draw_params,
    the recursion uses (0, 1) for the left node, (2, 3) for the right node, then (4, 5)."""
    def net(z, nn_):
        u = F.layer_norm(z, (z.shape[-1],), nn_["g1"], nn_["b1"], eps=1e-6)
        h1 = F.gelu(u @ nn_["W1"], approximate="tanh")
        v = F.layer_norm(h1, (h1.shape[-1],), nn_["g2"], nn_["b2"], eps=1e-6)
        return F.gelu((v @ nn_["W2"]) @ nn_["W3"], approximate="tanh") @ nn_["W4"]
    node = lambda a, b_, na, nb: np.sqrt(r) * torch.tanh(net(a, na) * net(b_, nb) / np.sqrt(r))
    if p == 2:
        return x
    if p == 4:
        return node(x, x, nets[0], nets[1])
    assert p == 8
    return node(node(x, x, nets[0], nets[1]), node(x, x, nets[2], nets[3]), nets[4], nets[5])


KEYS = ("g1", "b1", "W1", "g2", "b2", "W2", "W3", "W4")


def to_torch(nets):
    return [{k: torch.tensor(n[k], dtype=torch.float64, requires_grad=True) for k in KEYS} for n in nets]


@pytest.mark.parametrize("d,r,p", [(6, 4, 4), (10, 6, 8), (12, 8, 4)])
def test_sketch_gradient_against_torch_autograd(d, r, p):
    nets, flat = draw_params(d, r, p, seed=3 * d + r + p)
    rng = np.random.default_rng(11)
    X, dM = rng.standard_normal((5, d)), rng.standard_normal((5, r))
    tn = to_torch(nets)
    x = torch.tensor(X, requires_grad=True)
    (torch_sketch(x, tn, r, p) * torch.tensor(dM)).sum().backward()
    dX, dP = oracle.sketch_learned_bwd(X, flat, r, p, dM)
    np.testing.assert_allclose(dX, x.grad.numpy(), rtol=1e-9, atol=1e-11)
    want = np.concatenate([np.concatenate([n[k].grad.numpy().reshape(-1) for k in KEYS]) for n in tn])
    np.testing.assert_allclose(dP, want, rtol=1e-9, atol=1e-11)


@pytest.mark.parametrize("p", [4, 8])
def test_sketch_gradient_against_central_differences(p):
    d, r = 7, 4
    nets, flat = draw_params(d, r, p, seed=21 + p)
    rng = np.random.default_rng(5)
    X, dM = rng.standard_normal((3, d)), rng.standard_normal((3, r))
    dX, dP = oracle.sketch_learned_bwd(X, flat, r, p, dM)
    loss = lambda X_, P_: float((oracle.sketch_learned(X_, P_, r, p) * dM).sum())
    eps = 1e-6
    for idx in [(0, 0), (1, 3), (2, d - 1)]:
        Xp, Xm = X.copy(), X.copy()
        Xp[idx] += eps
        Xm[idx] -= eps
        np.testing.assert_allclose(dX[idx], (loss(Xp, flat) - loss(Xm, flat)) / (2 * eps), rtol=2e-6, atol=1e-8)
    # one entry of every tensor of the first and of the last network (scales, biases, matrices)
    hid = 8 * r
    sizes = lambda win: [win, win, win * hid, hid, hid, hid * r, r * hid, hid * r]
    first = np.cumsum([0] + sizes(d))[:-1]
    last_start = flat.size - sum(sizes(d if p == 4 else r))
    last = last_start + np.cumsum([0] + sizes(d if p == 4 else r))[:-1]
    for pos in list(first + 1) + list(last + 2):
        Pp, Pm = flat.copy(), flat.copy()
        Pp[pos] += eps
        Pm[pos] -= eps
        np.testing.assert_allclose(dP[pos], (loss(X, Pp) - loss(X, Pm)) / (2 * eps), rtol=5e-6, atol=1e-8)


def test_degree_two_has_no_networks():
    X = np.random.default_rng(0).standard_normal((4, 5))
    dM = np.random.default_rng(1).standard_normal((4, 5))
    dX, dP = oracle.sketch_learned_bwd(X, np.zeros(0), 3, 2, dM)
    np.testing.assert_array_equal(dX, dM)
    assert dP.size == 0


@pytest.mark.parametrize("p,local", [(4, oracle.LOCAL_EXACT), (4, oracle.LOCAL_SKETCH), (8, oracle.LOCAL_EXACT)])
def test_attention_gradient_with_learned_sketches_against_torch_autograd(p, local):
    n, d, dv, r, b = 12, 6, 5, 4, 4
    nets, flat = draw_params(d, r, p, seed=40 + p)
    rng = np.random.default_rng(9)
    Q, K, V, dO = (rng.standard_normal(s) for s in ((n, d), (n, d), (n, dv), (n, dv)))
    tn = to_torch(nets)
    q, k, v = (torch.tensor(a, requires_grad=True) for a in (Q, K, V))
    mq, mk = torch_sketch(q, tn, r, p), torch_sketch(k, tn, r, p)
    W = (mq @ mk.T) ** 2
    if local == oracle.LOCAL_EXACT:
        same = (torch.arange(n)[:, None] // b) == (torch.arange(n)[None, :] // b)
        W = torch.where(same, (q @ k.T) ** p, W)
    W = torch.tril(W)
    O = (W @ v) / (1.0 + W.sum(1, keepdim=True))
    # the forward agrees with the forward oracle before its gradient is trusted
    np.testing.assert_allclose(oracle.attn_def(Q, K, V, flat, p, r, b, local=local, learned=True), O.detach().numpy(),
                               rtol=1e-9, atol=1e-12)
    (O * torch.tensor(dO)).sum().backward()
    dQ, dK, dV, dP = oracle.attn_bwd_learned(Q, K, V, flat, dO, p, r, b, local=local)
    np.testing.assert_allclose(dQ, q.grad.numpy(), rtol=1e-8, atol=1e-11)
    np.testing.assert_allclose(dK, k.grad.numpy(), rtol=1e-8, atol=1e-11)
    np.testing.assert_allclose(dV, v.grad.numpy(), rtol=1e-8, atol=1e-11)
    want = np.concatenate([np.concatenate([t[key].grad.numpy().reshape(-1) for key in KEYS]) for t in tn])
    np.testing.assert_allclose(dP, want, rtol=1e-8, atol=1e-11)


def test_attention_gradient_with_learned_sketches_against_central_differences():
    n, d, dv, r, b, p = 8, 5, 4, 4, 4, 4
    nets, flat = draw_params(d, r, p, seed=77)
    rng = np.random.default_rng(3)
    Q, K, V, dO = (rng.standard_normal(s) for s in ((n, d), (n, d), (n, dv), (n, dv)))
    dQ, dK, dV, dP = oracle.attn_bwd_learned(Q, K, V, flat, dO, p, r, b)
    loss = lambda Q_, K_, P_: float((oracle.attn_def(Q_, K_, V, P_, p, r, b, learned=True) * dO).sum())
    eps = 1e-6
    for idx in [(0, 0), (5, 2), (7, 4)]:
        Qp, Qm, Kp, Km = Q.copy(), Q.copy(), K.copy(), K.copy()
        Qp[idx] += eps
        Qm[idx] -= eps
        Kp[idx] += eps
        Km[idx] -= eps
        np.testing.assert_allclose(dQ[idx], (loss(Qp, K, flat) - loss(Qm, K, flat)) / (2 * eps), rtol=1e-5, atol=1e-9)
        np.testing.assert_allclose(dK[idx], (loss(Q, Kp, flat) - loss(Q, Km, flat)) / (2 * eps), rtol=1e-5, atol=1e-9)
    for pos in np.random.default_rng(4).integers(0, flat.size, size=12):
        Pp, Pm = flat.copy(), flat.copy()
        Pp[pos] += eps
        Pm[pos] -= eps
        np.testing.assert_allclose(dP[pos], (loss(Q, K, Pp) - loss(Q, K, Pm)) / (2 * eps), rtol=2e-5, atol=1e-9)
