"""Every row of every unit of the numbered workloads against the float64 definition.

The probe-row tests of test_gpu_mfma.py look at ~40 rows per unit; here the oracle evaluates
the whole output (all host cores, one unit per thread) and the comparison is element by element:
max-abs and relative Frobenius error pooled and per unit, and a per-row relative bound
|got_i - want_i|_2 <= tol |want_i|_2 + eps, which a single wrong low-norm row or tile cannot
hide behind the pooled norms (most outputs are far smaller than the absolute bound).
"""
import os
import time

import numpy as np
import pytest

from paper_2310_01655_amd import binding as psf
from paper_2310_01655_amd import inputs
from parity import TOL, as_f64, gpu_attn
import oracle

pytestmark = pytest.mark.gpu

ROW_EPS = 1e-5      # absolute slack of the per-row bound (L2 over the dv columns of a row)


def assert_rows_close(got, want, dtype, what):
    """got, want: [batch, heads, n, dv].  Returns the figures it checked."""
    tol = TOL[dtype]
    got = np.asarray(got, dtype=np.float64)
    assert np.isfinite(got).all(), what
    diff = got - want
    max_abs = float(np.abs(diff).max())
    rel = float(np.linalg.norm(diff) / np.linalg.norm(want))
    unit_rel = np.linalg.norm(diff, axis=(2, 3)) / np.linalg.norm(want, axis=(2, 3))
    row_err = np.linalg.norm(diff, axis=-1)
    row_ref = np.linalg.norm(want, axis=-1)
    excess = row_err - (tol * row_ref + ROW_EPS)
    worst = np.unravel_index(int(np.argmax(excess)), excess.shape)
    row_rel_max = float((row_err / np.maximum(row_ref, 1e-30)).max())
    msg = ("%s: max_abs %.3e rel_fro %.3e worst unit rel_fro %.3e worst row rel %.3e at %s "
           "(|want| %.3e |diff| %.3e)" % (what, max_abs, rel, unit_rel.max(), row_rel_max, worst,
                                          row_ref[worst], row_err[worst]))
    print(msg)
    assert max_abs <= tol and rel <= tol, msg
    assert unit_rel.max() <= tol, msg
    assert excess.max() <= 0.0, msg
    return max_abs, rel


def full_parity(cfg, q, k, v, G, what):
    got, desc = gpu_attn(cfg, q, k, v, G)
    assert psf.kernel_path(desc) == 1
    t0 = time.perf_counter()
    want, threads = oracle.attn_def_batch(as_f64(q), as_f64(k), as_f64(v), as_f64(G), cfg["p"], cfg["r"],
                                          cfg["b"], max_threads=min(os.cpu_count() or 1, 16))
    print("%s: oracle %d units x %d rows in %.1f s on %d threads" % (
        what, cfg["batch"] * cfg["heads"], cfg["n"], time.perf_counter() - t0, threads))
    return assert_rows_close(got.numpy(), want, cfg["dtype"], what)


def test_config2_every_row_of_every_unit():
    cfg, q, k, v, G = inputs.make_config(2)
    full_parity(cfg, q, k, v, G, "config 2, 96 units in full")


def test_config3_every_row_of_every_unit():
    cfg, q, k, v, G = inputs.make_config(3)
    full_parity(cfg, q, k, v, G, "config 3, 24 units in full")


@pytest.mark.parametrize("variant", [None, "heavy"])
def test_config5_every_row_of_every_unit(variant):
    cfg, q, k, v, G = inputs.make_config(5, variant=variant)
    full_parity(cfg, q, k, v, G, "config 5 (%s), 16 units in full" % (variant or "normal"))
