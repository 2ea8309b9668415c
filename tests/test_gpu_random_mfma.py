"""GPU parity of the bf16 MFMA kernels on seeded random descriptors (through the C ABI, against
the float64 oracle).

The descriptor is drawn from the set the MFMA kernels admit -- d = dv in {64, 128}, r in {32, 64},
p in {2, 4, 8}, b in {256, 512, 1024}, one to four blocks, either in-block rule, shared or per-head
matrices, Gaussian or learned sketches, with or without the causal mask -- so that combinations
no hand-picked case names (degree 8 with the sketched in-block rule and three heads, a single
block with learned sketches, ...) are exercised too.  The forward results are compared on the
first and last rows of every block plus random rows of every unit, the gradients in full.
Tolerance 2e-2 (bf16 storage)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2310_01655_amd import binding as psf
from paper_2310_01655_amd import inputs
from parity import as_f64, assert_close, assert_close_scaled

pytestmark = pytest.mark.gpu


def draw_desc(seed):
    rng = np.random.default_rng(seed)
    c = dict(batch=int(rng.integers(1, 3)), heads=int(rng.integers(1, 4)),
             b=int(rng.choice([256, 512, 1024])), d=int(rng.choice([64, 64, 128])),
             r=int(rng.choice([32, 64])), p=int(rng.choice([2, 4, 4, 8])),
             local=int(rng.choice([psf.LOCAL_EXACT, psf.LOCAL_EXACT, psf.LOCAL_SKETCH])),
             per_head=bool(rng.integers(0, 2)), noncausal=bool(rng.integers(0, 4) == 0))
    c["n"] = c["b"] * int(rng.integers(1, 5))
    if c["p"] == 2:
        c["d"] = 64                               # the base case m(x) = x has MFMA kernels for d = 64
    c["learned"] = bool(c["p"] == 4 and c["d"] == 64 and rng.integers(0, 3) == 0)
    if c["learned"] or (c["d"] == 128 and c["r"] == 32):
        c["local"] = psf.LOCAL_EXACT              # the sketched rule has no MFMA kernel for these
    return c


def draw_inputs(c, seed):
    q, k, v = inputs.make_qkv(c["batch"], c["heads"], c["n"], c["d"], seed=seed, dtype="bf16")
    G = None
    if c["learned"]:
        G = inputs.make_learned_params(c["heads"], c["d"], c["r"], c["p"], per_head=c["per_head"], seed=seed + 1,
                                       dtype="bf16")
    elif c["p"] > 2:
        G = inputs.make_sketch_matrices(c["heads"], c["d"], c["r"], c["p"], per_head=c["per_head"], seed=seed + 1,
                                        dtype="bf16")
    desc = psf.make_desc(c["batch"], c["heads"], c["n"], c["d"], c["p"], c["r"], c["b"], "bf16",
                         local=c["local"], per_head=c["per_head"], learned=c["learned"])
    return q, k, v, G, desc


def sample_rows(c, seed):
    rng = np.random.default_rng(seed + 99)
    rows = set(int(x) for x in rng.integers(0, c["n"], size=24))
    for l in range(c["n"] // c["b"]):
        rows.update((l * c["b"], l * c["b"] + c["b"] - 1))
    return sorted(rows)


@pytest.mark.parametrize("seed", range(5000, 5024))
def test_mfma_forward_random_descriptor(seed):
    c = draw_desc(seed)
    q, k, v, G, desc = draw_inputs(c, seed)
    assert psf.kernel_path(desc) == 1, c
    dev = torch.device("cuda:0")
    args = [t.to(dev) if t is not None else None for t in (q, k, v, G)]
    fwd = psf.psf_noncausal_attn_fwd if c["noncausal"] else psf.psf_causal_attn_fwd
    O = fwd(desc, *args)
    torch.cuda.synchronize()
    got = O.float().cpu().numpy()
    assert np.isfinite(got).all()
    rows = sample_rows(c, seed)
    olocal = oracle.LOCAL_EXACT if c["local"] == psf.LOCAL_EXACT else oracle.LOCAL_SKETCH
    want = np.empty((c["batch"], c["heads"], len(rows), c["d"]))
    for bi in range(c["batch"]):
        for h in range(c["heads"]):
            g = None if G is None else as_f64(G[h if G.shape[0] > 1 else 0])
            Q1, K1, V1 = as_f64(q[bi, h]), as_f64(k[bi, h]), as_f64(v[bi, h])
            if c["noncausal"]:
                want[bi, h] = oracle.attn_noncausal(Q1[rows], K1, V1, g, c["p"], c["r"], learned=c["learned"])
            else:
                want[bi, h] = oracle.attn_def(Q1, K1, V1, g, c["p"], c["r"], c["b"], local=olocal, rows=rows,
                                              learned=c["learned"])
    print(c, assert_close(got[:, :, rows], want, "bf16", "mfma forward %s" % c))


@pytest.mark.parametrize("seed", list(range(6000, 6008)) + list(range(6100, 6112)))
def test_mfma_backward_random_descriptor(seed):
    rng = np.random.default_rng(seed)
    c = dict(batch=1, heads=int(rng.integers(1, 3)), b=int(rng.choice([256, 512])), d=64, p=4,
             r=int(rng.choice([32, 64])), per_head=bool(rng.integers(0, 2)), learned=False)
    c["n"] = c["b"] * int(rng.integers(1, 4))
    c["local"] = int(rng.choice([psf.LOCAL_EXACT, psf.LOCAL_SKETCH])) if c["r"] == 64 else psf.LOCAL_EXACT
    if seed >= 6100:                              # head width 128 and degree 8 (exact in-block weights)
        c["d"], c["p"] = int(rng.choice([64, 128, 128])), int(rng.choice([4, 8, 8]))
        if (c["d"], c["p"]) != (64, 4):
            c["local"] = psf.LOCAL_EXACT
    q, k, v, G, desc = draw_inputs(c, seed)
    assert psf.bwd_kernel_path(desc) == 3, c
    dO = inputs.make_dout(c["batch"], c["heads"], c["n"], c["d"], seed=seed, dtype="bf16")
    dev = torch.device("cuda:0")
    dQ, dK, dV = psf.psf_causal_attn_bwd(desc, *[t.to(dev) for t in (q, k, v, G, dO)])
    torch.cuda.synchronize()
    olocal = oracle.LOCAL_EXACT if c["local"] == psf.LOCAL_EXACT else oracle.LOCAL_SKETCH
    wQ, wK, wV, _ = oracle.attn_bwd_batch(as_f64(q), as_f64(k), as_f64(v), as_f64(G), as_f64(dO), c["p"], c["r"],
                                          c["b"], local=olocal)
    for name, got, want in (("dQ", dQ, wQ), ("dK", dK, wK), ("dV", dV, wV)):
        assert_close_scaled(got.float().cpu().numpy(), want, "bf16", "%s %s" % (name, c))
    print(c)


@pytest.mark.parametrize("seed", range(6200, 6208))
def test_mfma_learned_backward_random_descriptor(seed):
    """Learned sketches of degree 4 on the MFMA kernels: gradients with respect to Q, K, V in full
    and the parameter gradient of every set (summed over the units that share it)."""
    rng = np.random.default_rng(seed)
    c = dict(batch=int(rng.integers(1, 3)), heads=int(rng.integers(1, 4)), b=int(rng.choice([256, 512])), d=64, p=4,
             r=32 if seed % 2 else 64, per_head=bool((seed // 2) % 2), learned=True, local=psf.LOCAL_EXACT)
    c["n"] = c["b"] * int(rng.integers(2, 5))       # at least two blocks: the sketches carry a gradient
    q, k, v, G, desc = draw_inputs(c, seed)
    assert psf.bwd_kernel_path(desc) == 3, c
    dO = inputs.make_dout(c["batch"], c["heads"], c["n"], c["d"], seed=seed, dtype="bf16")
    dev = torch.device("cuda:0")
    dQ, dK, dV, dG = psf.psf_causal_attn_bwd_learned(desc, *[t.to(dev) for t in (q, k, v, G, dO)])
    torch.cuda.synchronize()
    wQ, wK, wV = (np.empty(tuple(t.shape)) for t in (q, k, v))
    wG = np.zeros(tuple(G.shape))
    for bi in range(c["batch"]):
        for h in range(c["heads"]):
            s = h if G.shape[0] > 1 else 0
            wQ[bi, h], wK[bi, h], wV[bi, h], dp = oracle.attn_bwd_learned(
                as_f64(q[bi, h]), as_f64(k[bi, h]), as_f64(v[bi, h]), as_f64(G[s]), as_f64(dO[bi, h]), c["p"], c["r"],
                c["b"], local=oracle.LOCAL_EXACT)
            wG[s] += dp
    for name, got, want in (("dQ", dQ, wQ), ("dK", dK, wK), ("dV", dV, wV)):
        assert_close_scaled(got.float().cpu().numpy(), want, "bf16", "%s %s" % (name, c))
    for s in range(G.shape[0]):
        assert_close_scaled(dG[s].cpu().numpy(), wG[s], "bf16", "dG set %d %s" % (s, c))
    print(c)
