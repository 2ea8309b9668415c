"""The float64 oracle under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only).

psf_oracle.c is rebuilt with -fsanitize=address,undefined and the pin suites that need nothing
but numpy run against that build in a child process (the sanitizer runtime has to be loaded
before the interpreter starts); the gradient and learned-sketch functions, whose pin suites also
import torch, are driven directly on small cases, edge cases included (one block, blocks of one
token, listed rows, every degree).  Any out-of-bounds access, use after free, signed overflow or
misaligned access in the oracle aborts the child."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

DIRECT = r"""
import numpy as np
import oracle
rng = np.random.default_rng(5)
for p in (2, 4, 8, 16):
    for n, b in ((12, 1), (12, 4), (12, 12)):
        d, dv, r = 6, 5, 4
        Q, K, V, dO = rng.standard_normal((n, d)), rng.standard_normal((n, d)), rng.standard_normal((n, dv)), rng.standard_normal((n, dv))
        G = rng.standard_normal(max(oracle.g_len(d, r, p), 1))
        for local in (oracle.LOCAL_EXACT, oracle.LOCAL_SKETCH):
            O = oracle.attn_def(Q, K, V, G, p, r, b, local=local)
            O2 = oracle.attn_block(Q, K, V, G, p, r, b, local=local)
            assert np.allclose(O, O2, rtol=1e-9, atol=1e-12)
            rows = [0, n - 1, n // 2]
            assert np.allclose(oracle.attn_def(Q, K, V, G, p, r, b, local=local, rows=rows), O[rows])
            g = oracle.attn_bwd(Q, K, V, G, dO, p, r, b, local=local)
            gr = oracle.attn_bwd_rows(Q, K, V, G, dO, p, r, b, list(range(n)), local=local)
            assert all(np.allclose(x, y) for x, y in zip(g, gr))
        oracle.attn_noncausal(Q[:5], K, V, G, p, r)
        oracle.sketch_bwd(Q, G, r, p, rng.standard_normal((n, d if p == 2 else r)))
        if p in (4, 8):
            P = 0.3 * rng.standard_normal(oracle.learned_len(d, r, p))
            M = oracle.sketch_learned(Q, P, r, p)
            assert np.isfinite(M).all() and np.abs(M).max() <= np.sqrt(r) + 1e-12
            oracle.attn_def(Q, K, V, P, p, r, b, learned=True)
            oracle.sketch_learned_bwd(Q, P, r, p, rng.standard_normal((n, r)))
            oracle.attn_bwd_learned(Q, K, V, P, dO, p, r, b)
Qb, Kb, Vb = rng.standard_normal((2, 3, 8, 4)), rng.standard_normal((2, 3, 8, 4)), rng.standard_normal((2, 3, 8, 3))
Gb = rng.standard_normal((3, oracle.g_len(4, 4, 4)))
O, _ = oracle.attn_def_batch(Qb, Kb, Vb, Gb, 4, 4, 2, max_threads=3)
oracle.attn_bwd_batch(Qb, Kb, Vb, Gb, rng.standard_normal(Vb.shape), 4, 4, 2, max_threads=3)
oracle.power_tensor(Qb[0, 0], 4)
print("direct cases ok")
"""


def _env(san_lib):
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], check=True, capture_output=True,
                          text=True).stdout.strip()
    env = dict(os.environ)
    env["LD_PRELOAD"] = asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"     # the interpreter itself leaks by design
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["PSF_ORACLE_LIB"] = san_lib
    env["OMP_NUM_THREADS"] = "4"
    env["PYTHONPATH"] = ROOT + (os.pathsep + env["PYTHONPATH"] if env.get("PYTHONPATH") else "")
    return env


@pytest.fixture(scope="module")
def san_lib():
    from oracle import build as oracle_build
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(asan) or not os.path.exists(asan):
        pytest.skip("no AddressSanitizer runtime for gcc on this machine")
    return oracle_build.build_sanitized()


def test_pin_suites_pass_on_the_sanitized_build(san_lib):
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py"),
                        os.path.join(ROOT, "tests", "test_oracle_noncausal_pins.py")],
                       cwd=ROOT, env=_env(san_lib), capture_output=True, text=True, timeout=900)
    assert r.returncode == 0, r.stdout[-3000:] + r.stderr[-3000:]
    assert "passed" in r.stdout
    assert "AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr, r.stderr[-3000:]


def test_gradient_learned_and_batch_functions_on_the_sanitized_build(san_lib):
    r = subprocess.run([sys.executable, "-c", DIRECT], cwd=ROOT, env=_env(san_lib), capture_output=True,
                       text=True, timeout=900)
    assert r.returncode == 0, r.stdout[-3000:] + r.stderr[-3000:]
    assert "direct cases ok" in r.stdout
    assert "AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr, r.stderr[-3000:]
