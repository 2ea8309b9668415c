"""GPU parity on seeded random descriptors (through the C ABI, against the float64 oracle).

The hand-picked cases of the other files cover the shapes the kernels are tiled for; these draw
the descriptor itself -- batch, heads, block size and count, widths, sketch size, degree, storage
type, in-block rule, shared or per-head matrices, Gaussian or learned sketches -- from a seeded
generator, so that no combination of tails (a width that is no multiple of a lane group, a block
of one token, more value columns than key columns, ...) is left to chance.  All shapes are
small: the oracle evaluates every row of every unit.  Same tolerances as everywhere: 1e-4 (fp32
storage) / 2e-2 (bf16 storage)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2310_01655_amd import binding as psf
from paper_2310_01655_amd import inputs
from parity import as_f64, assert_close, assert_close_scaled

pytestmark = pytest.mark.gpu


def draw_desc(seed, max_width=40, max_r=24, degrees=(2, 4, 8), max_blocks=6, max_b=40, learned_too=True):
    rng = np.random.default_rng(seed)
    b = int(rng.integers(1, max_b + 1))
    c = dict(batch=int(rng.integers(1, 3)), heads=int(rng.integers(1, 4)), b=b,
             n=b * int(rng.integers(1, max_blocks + 1)),
             d=int(rng.integers(1, max_width + 1)), dv=int(rng.integers(1, max_width + 1)),
             r=int(rng.integers(1, max_r + 1)), p=int(rng.choice(degrees)),
             dtype=str(rng.choice(["f32", "bf16"])),
             local=int(rng.choice([psf.LOCAL_EXACT, psf.LOCAL_SKETCH])),
             per_head=bool(rng.integers(0, 2)))
    # one case in four with learned sketches (Algorithm 2); p = 2 has no sketch to learn
    c["learned"] = bool(learned_too and 2 < c["p"] <= 8 and rng.integers(0, 4) == 0)
    if c["learned"]:
        c["r"] = min(c["r"], 12)                 # hidden width 8 r: keeps the oracle's network loops short
    return c


def draw_inputs(c, seed):
    q, k, v = inputs.make_qkv(c["batch"], c["heads"], c["n"], c["d"], dv=c["dv"], seed=seed, dtype=c["dtype"])
    G = None
    if c["learned"]:
        G = inputs.make_learned_params(c["heads"], c["d"], c["r"], c["p"], per_head=c["per_head"], seed=seed + 1,
                                       dtype=c["dtype"])
    elif c["p"] > 2:
        G = inputs.make_sketch_matrices(c["heads"], c["d"], c["r"], c["p"], per_head=c["per_head"], seed=seed + 1,
                                        dtype=c["dtype"])
    desc = psf.make_desc(c["batch"], c["heads"], c["n"], c["d"], c["p"], c["r"], c["b"], c["dtype"], dv=c["dv"],
                         local=c["local"], per_head=c["per_head"], learned=c["learned"])
    return q, k, v, G, desc


def oracle_rows(c, q, k, v, G, rows=None):
    """The definition, unit by unit (every row, or the listed ones)."""
    nrows = c["n"] if rows is None else len(rows)
    want = np.empty((c["batch"], c["heads"], nrows, c["dv"]))
    for bi in range(c["batch"]):
        for h in range(c["heads"]):
            g = None if G is None else as_f64(G[h if G.shape[0] > 1 else 0])
            want[bi, h] = oracle.attn_def(as_f64(q[bi, h]), as_f64(k[bi, h]), as_f64(v[bi, h]), g, c["p"], c["r"],
                                          c["b"], local=oracle_local(c), rows=rows, learned=c["learned"])
    return want


def oracle_local(c):
    return oracle.LOCAL_EXACT if c["local"] == psf.LOCAL_EXACT else oracle.LOCAL_SKETCH


def on_gpu(*tensors):
    dev = torch.device("cuda:0")
    return [t.to(dev) if t is not None else None for t in tensors]


@pytest.mark.parametrize("seed", range(1000, 1048))
def test_forward_random_descriptor(seed):
    c = draw_desc(seed)
    q, k, v, G, desc = draw_inputs(c, seed)
    O = psf.psf_causal_attn_fwd(desc, *on_gpu(q, k, v, G))
    torch.cuda.synchronize()
    want = oracle_rows(c, q, k, v, G)
    print(c, assert_close(O.float().cpu().numpy(), want, c["dtype"], "forward %s" % c))


@pytest.mark.parametrize("seed", range(2000, 2024))
def test_noncausal_random_descriptor(seed):
    c = draw_desc(seed)
    q, k, v, G, desc = draw_inputs(c, seed)
    O = psf.psf_noncausal_attn_fwd(desc, *on_gpu(q, k, v, G))
    torch.cuda.synchronize()
    want = np.empty(tuple(v.shape))
    for bi in range(c["batch"]):
        for h in range(c["heads"]):
            g = None if G is None else as_f64(G[h if G.shape[0] > 1 else 0])
            want[bi, h] = oracle.attn_noncausal(as_f64(q[bi, h]), as_f64(k[bi, h]), as_f64(v[bi, h]), g,
                                                c["p"], c["r"], learned=c["learned"])
    print(c, assert_close(O.float().cpu().numpy(), want, c["dtype"], "noncausal %s" % c))


@pytest.mark.parametrize("seed", range(3000, 3032))
def test_backward_random_descriptor(seed):
    c = draw_desc(seed, max_width=32, max_r=16, max_blocks=4, max_b=32, learned_too=False)
    q, k, v, G, desc = draw_inputs(c, seed)
    dO = inputs.make_dout(c["batch"], c["heads"], c["n"], c["dv"], seed=seed, dtype=c["dtype"])
    dQ, dK, dV = psf.psf_causal_attn_bwd(desc, *on_gpu(q, k, v, G, dO))
    torch.cuda.synchronize()
    wQ, wK, wV, _ = oracle.attn_bwd_batch(as_f64(q), as_f64(k), as_f64(v), as_f64(G) if G is not None else None,
                                          as_f64(dO), c["p"], c["r"], c["b"], local=oracle_local(c))
    for name, got, want in (("dQ", dQ, wQ), ("dK", dK, wK), ("dV", dV, wV)):
        assert_close_scaled(got.float().cpu().numpy(), want, c["dtype"], "%s %s" % (name, c))
    print(c)


@pytest.mark.parametrize("seed", range(3500, 3516))
def test_learned_backward_random_descriptor(seed):
    """Learned sketches (Algorithm 2): gradients with respect to Q, K, V and to the networks'
    parameters; the oracle works unit by unit, the parameter gradient of a set is the sum over the
    units that use it."""
    c = draw_desc(seed, max_width=24, max_r=12, degrees=(4, 8), max_blocks=3, max_b=24)
    c["learned"] = True
    q, k, v, G, desc = draw_inputs(c, seed)
    dO = inputs.make_dout(c["batch"], c["heads"], c["n"], c["dv"], seed=seed, dtype=c["dtype"])
    dQ, dK, dV, dG = psf.psf_causal_attn_bwd_learned(desc, *on_gpu(q, k, v, G, dO))
    torch.cuda.synchronize()
    wQ, wK, wV = (np.empty(tuple(t.shape)) for t in (q, k, v))
    wG = np.zeros(tuple(G.shape))
    for bi in range(c["batch"]):
        for h in range(c["heads"]):
            s = h if G.shape[0] > 1 else 0
            wQ[bi, h], wK[bi, h], wV[bi, h], dp = oracle.attn_bwd_learned(
                as_f64(q[bi, h]), as_f64(k[bi, h]), as_f64(v[bi, h]), as_f64(G[s]), as_f64(dO[bi, h]), c["p"],
                c["r"], c["b"], local=oracle_local(c))
            wG[s] += dp
    for name, got, want in (("dQ", dQ, wQ), ("dK", dK, wK), ("dV", dV, wV)):
        assert_close_scaled(got.float().cpu().numpy(), want, c["dtype"], "%s %s" % (name, c))
    for s in range(G.shape[0]):
        assert_close_scaled(dG[s].cpu().numpy(), wG[s], "f32", "dG set %d %s" % (s, c))
    print(c)


@pytest.mark.parametrize("seed", range(4000, 4024))
def test_decode_random_descriptor(seed):
    """Prompt of a random length through psf_decode_prefill, the rest token by token: every
    output row equals the forward definition's."""
    c = draw_desc(seed, max_blocks=4, max_b=24)
    q, k, v, G, desc = draw_inputs(c, seed)
    rng = np.random.default_rng(seed + 7)
    n_prompt = int(rng.integers(0, c["n"] + 1))
    dev = torch.device("cuda:0")
    qd, kd, vd, Gd = on_gpu(q, k, v, G)
    state = psf.decode_new_state(desc, dev)
    ws = psf.psf_decode_prefill(desc, kd[:, :, :n_prompt].contiguous(), vd[:, :, :n_prompt].contiguous(), Gd, state)
    rows = list(range(n_prompt, c["n"]))
    out = torch.empty(c["batch"], c["heads"], len(rows), c["dv"], dtype=q.dtype, device=dev)
    for i, pos in enumerate(rows):
        o = psf.psf_decode_step(desc, qd[:, :, pos:pos + 1].contiguous(), kd[:, :, pos:pos + 1].contiguous(),
                                vd[:, :, pos:pos + 1].contiguous(), Gd, pos, state)
        out[:, :, i] = o[:, :, 0]
    torch.cuda.synchronize()
    del ws
    if rows:
        want = oracle_rows(c, q, k, v, G, rows=rows)
        print(c, n_prompt, assert_close(out.float().cpu().numpy(), want, c["dtype"], "decode %s" % c))


@pytest.mark.parametrize("seed", range(5000, 5024))
def test_sketch_entry_point_random_descriptor(seed):
    """psf_sketch on a random descriptor: m(x) of Algorithm 1 (or Algorithm 2) and its self tensor
    product phi'(x) = m(x) (x) m(x), row by row."""
    c = draw_desc(seed, degrees=(2, 4, 8, 16), max_blocks=3)
    q, _, _, G, desc = draw_inputs(c, seed)
    dev = torch.device("cuda:0")
    M, Phi = psf.psf_sketch(desc, q.to(dev), G.to(dev) if G is not None else None, want_m=True, want_phi=True)
    torch.cuda.synchronize()
    for bi in range(c["batch"]):
        for h in range(c["heads"]):
            g = None if G is None else as_f64(G[h if G.shape[0] > 1 else 0])
            x = as_f64(q[bi, h])
            m = oracle.sketch_learned(x, g, c["r"], c["p"]) if c["learned"] else oracle.sketch(x, g, c["r"], c["p"])
            assert_close_scaled(M[bi, h].float().cpu().numpy(), m, c["dtype"], "m %s" % c)
            assert_close_scaled(Phi[bi, h].float().cpu().numpy(), oracle.self_tensor(m), c["dtype"], "phi' %s" % c)
    print(c)
