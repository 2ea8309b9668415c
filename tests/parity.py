"""Helpers for the GPU-vs-oracle parity tests (test infrastructure)."""
import numpy as np
import torch

import oracle
from paper_2310_01655_amd import binding as psf

TOL = {"f32": 1e-4, "bf16": 2e-2}     # max-abs and relative-Frobenius bound, per storage dtype


def errors(got, want):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    max_abs = float(np.abs(got - want).max()) if got.size else 0.0
    denom = float(np.linalg.norm(want))
    rel = float(np.linalg.norm(got - want) / denom) if denom > 0 else max_abs
    return max_abs, rel


def assert_close(got, want, dtype, what=""):
    max_abs, rel = errors(got, want)
    tol = TOL[dtype]
    assert np.isfinite(np.asarray(got, dtype=np.float64)).all(), what
    assert max_abs <= tol and rel <= tol, "%s: max_abs %.3e rel_fro %.3e (tol %.0e)" % (
        what, max_abs, rel, tol)
    return max_abs, rel


def assert_close_scaled(got, want, dtype, what=""):
    """For gradients, whose entries have no fixed scale (a bf16 result of magnitude 8 is already
    1.6e-2 away from its float64 value): max-abs error relative to the largest entry (at least
    1) and relative Frobenius error, both within the storage type's tolerance."""
    max_abs, rel = errors(got, want)
    scale = max(1.0, float(np.abs(np.asarray(want, dtype=np.float64)).max()))
    tol = TOL[dtype]
    assert np.isfinite(np.asarray(got, dtype=np.float64)).all(), what
    assert max_abs <= tol * scale and rel <= tol, "%s: max_abs %.3e (scale %.2e) rel_fro %.3e (tol %.0e)" % (
        what, max_abs, scale, rel, tol)
    return max_abs, rel


def as_f64(t):
    return t.to(torch.float64).numpy()


def gpu_attn(cfg, q, k, v, G, feat=psf.FEAT_SKETCH, local=psf.LOCAL_EXACT, b=None, timed=False):
    desc = psf.make_desc(cfg["batch"], cfg["heads"], cfg["n"], cfg["d"], cfg["p"], cfg["r"],
                         cfg["b"] if b is None else b, cfg["dtype"], feat=feat, local=local,
                         per_head=cfg.get("per_head", False))
    dev = torch.device("cuda:0")
    args = [x.to(dev) if x is not None else None for x in (q, k, v, G)]
    if timed:
        O, stages = psf.psf_causal_attn_fwd_timed(desc, *args)
    else:
        O, stages = psf.psf_causal_attn_fwd(desc, *args), None
    torch.cuda.synchronize()
    out = O.float().cpu()
    return (out, stages, desc) if timed else (out, desc)


def oracle_attn(cfg, q, k, v, G, feat=oracle.FEAT_SKETCH, local=oracle.LOCAL_EXACT, b=None,
                rows=None):
    O, _ = oracle.attn_def_batch(as_f64(q), as_f64(k), as_f64(v),
                                 as_f64(G) if G is not None else None,
                                 cfg["p"], cfg["r"], cfg["b"] if b is None else b,
                                 feat=feat, local=local, rows=rows)
    return O


def oracle_units_rows(cfg, q, k, v, G, units, rows, local=oracle.LOCAL_EXACT, b=None):
    """Oracle rows `rows` of the listed (batch, head) units -> {(bi, h): [len(rows), dv]}."""
    out = {}
    for bi, h in units:
        g = G[h if G.shape[0] > 1 else 0]
        out[(bi, h)] = oracle.attn_def(as_f64(q[bi, h]), as_f64(k[bi, h]), as_f64(v[bi, h]), as_f64(g),
                                       cfg["p"], cfg["r"], cfg["b"] if b is None else b,
                                       local=local, rows=rows)
    return out


def probe_rows(n, b, extra=24, seed=0):
    """Rows that exercise every regime: first/last of the sequence and of blocks, tile edges,
    plus a seeded random sample."""
    rng = np.random.default_rng(seed)
    fixed = {0, 1, 31, 32, 63, 64, 255, 256, b - 1, n - 1, n - b, n - b - 1, n // 2, n // 2 - 1}
    if n > b:
        fixed |= {b, b + 1, 2 * b - 1}
    fixed |= set(int(x) for x in rng.integers(0, n, size=extra))
    return sorted(x for x in fixed if 0 <= x < n)
