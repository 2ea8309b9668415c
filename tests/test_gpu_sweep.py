"""The block-size / sketch-size sweep (2^20 tokens per step, 12 heads, d = 64, p = 4) at the batch
the benchmark times (2^20 / n sequences), every (n, r, b) point against the float64 oracle.

Exact in-block weights (the headline mode) depend on b by definition, so each point is compared
with the oracle evaluated with that b: probe rows of two units plus one whole block of each.
Invariance to b holds where every weight comes from the sketches (Section 3.1's in-block rule):
there the three block sizes are compared with each other over the whole batch and with the
oracle on probe rows, for every (n, r).

The 12 * 2^20 rows of Q, K, V are drawn once; each n views the same buffer as [2^20 / n, 12, n, 64]
(rows are iid, so every view is a draw of the workload's distribution).
"""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

import oracle
from paper_2310_01655_amd import binding as psf
from paper_2310_01655_amd import inputs
from parity import TOL, as_f64, assert_close, probe_rows

pytestmark = pytest.mark.gpu

TOKENS, HEADS, D, P = 1 << 20, 12, 64, 4
NS, RS, BS = (8192, 16384, 32768, 65536), (32, 64), (256, 512, 1024)
ROW_EPS = 1e-5


@pytest.fixture(scope="module")
def pool():
    q, k, v = inputs.make_qkv(1, 1, HEADS * TOKENS, D, seed=1004, dtype="bf16")
    dev = torch.device("cuda:0")
    host = dict(q=q.view(-1, D), k=k.view(-1, D), v=v.view(-1, D))
    devt = {nm: t.to(dev) for nm, t in host.items()}
    G = {r: inputs.make_sketch_matrices(HEADS, D, r, P, per_head=False, seed=0, dtype="bf16") for r in RS}
    yield dict(host=host, dev=devt, G=G, Gd={r: g.to(dev) for r, g in G.items()})
    devt.clear()
    torch.cuda.empty_cache()


@pytest.fixture(autouse=True)
def release_workspaces():
    yield
    torch.cuda.empty_cache()       # workspaces of up to ~35 GB, a different size at every point


def view(t, n):
    return t.view(TOKENS // n, HEADS, n, D)


def run_gpu(pool, n, r, b, local):
    desc = psf.make_desc(TOKENS // n, HEADS, n, D, P, r, b, "bf16", local=local)
    assert psf.kernel_path(desc) == 1
    O = psf.psf_causal_attn_fwd(desc, view(pool["dev"]["q"], n), view(pool["dev"]["k"], n),
                                view(pool["dev"]["v"], n), pool["Gd"][r])
    torch.cuda.synchronize()
    return O


def whole_batch_properties(O, vd):
    """Finite, and inside the convex hull of the values seen so far (weights are non-negative and
    the denominator exceeds their sum): checked on the device over all 2^20 x 12 rows."""
    assert bool(torch.isfinite(O).all())
    vmax = torch.cummax(vd.float().abs().amax(-1), dim=-1).values
    assert bool((O.float().abs().amax(-1) <= vmax * 1.01 + 1e-3).all())


def oracle_rows(pool, n, r, b, local, units, rows_of):
    """{unit: oracle rows rows_of[unit]} with one thread per unit."""
    hq, hk, hv = (view(pool["host"][nm], n) for nm in ("q", "k", "v"))
    g = as_f64(pool["G"][r][0])

    def one(u):
        bi, h = u
        return oracle.attn_def(as_f64(hq[bi, h]), as_f64(hk[bi, h]), as_f64(hv[bi, h]), g, P, r, b,
                               local=local, rows=rows_of[u])

    with ThreadPoolExecutor(len(units)) as ex:
        return dict(zip(units, ex.map(one, units)))


def check_rows(got, want, what):
    res = assert_close(got, want, "bf16", what)
    err = np.linalg.norm(got - want, axis=-1)
    ref = np.linalg.norm(want, axis=-1)
    assert (err <= TOL["bf16"] * ref + ROW_EPS).all(), "%s: row %d rel %.3e" % (
        what, int(np.argmax(err - TOL["bf16"] * ref)), float((err / np.maximum(ref, 1e-30)).max()))
    return res


@pytest.mark.parametrize("b", BS)
@pytest.mark.parametrize("r", RS)
@pytest.mark.parametrize("n", NS)
def test_sweep_point_exact_in_block_weights(pool, n, r, b):
    batch, t = TOKENS // n, n // b
    O = run_gpu(pool, n, r, b, psf.LOCAL_EXACT)
    whole_batch_properties(O, view(pool["dev"]["v"], n))
    # two units far apart in the grid; probe rows plus one whole block each (the last block, which
    # carries the longest prefix, and one in the middle)
    units = [(0, 0), (batch - 1, HEADS - 1)]
    blocks = {units[0]: t - 1, units[1]: t // 2}
    rows_of = {u: sorted(set(probe_rows(n, b, seed=n + r + b)) | set(range(blocks[u] * b, (blocks[u] + 1) * b)))
               for u in units}
    want = oracle_rows(pool, n, r, b, oracle.LOCAL_EXACT, units, rows_of)
    for u in units:
        got = O[u[0], u[1]].float().cpu().numpy().astype(np.float64)[rows_of[u]]
        print("sweep n=%d r=%d b=%d unit %s:" % (n, r, b, u),
              check_rows(got, want[u], "n=%d r=%d b=%d unit %s" % (n, r, b, u)))


@pytest.mark.parametrize("r", RS)
@pytest.mark.parametrize("n", NS)
def test_block_size_invariance_with_sketched_in_block_weights(pool, n, r):
    batch = TOKENS // n
    outs = {b: run_gpu(pool, n, r, b, psf.LOCAL_SKETCH) for b in BS}
    ref = outs[BS[0]].float()
    ref_norm = float(ref.double().norm())
    for b in BS[1:]:
        diff = outs[b].float() - ref
        max_abs, rel = float(diff.abs().max()), float(diff.double().norm()) / ref_norm
        print("b-invariance n=%d r=%d: b=%d against b=%d: max_abs %.3e rel_fro %.3e" % (n, r, b, BS[0], max_abs, rel))
        assert max_abs <= TOL["bf16"] and rel <= TOL["bf16"]
    units = [(0, 0), (batch - 1, HEADS - 1)]
    rows = probe_rows(n, 1024, seed=n + r)
    want = oracle_rows(pool, n, r, 1024, oracle.LOCAL_SKETCH, units, {u: rows for u in units})
    for b in BS:
        for u in units:
            got = outs[b][u[0], u[1]].float().cpu().numpy().astype(np.float64)[rows]
            check_rows(got, want[u], "sketched in-block n=%d r=%d b=%d unit %s" % (n, r, b, u))
