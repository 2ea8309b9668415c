"""float64 CPU oracle for causal polynomial-sketch attention (ctypes over psf_oracle.c).

TEST INFRASTRUCTURE ONLY.  Importers: tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py.  The GPU library never imports this package and this
package never imports the GPU library; they share no arithmetic.

All arrays are numpy float64, row-major.  A "unit" is one (batch, head) slice.
Sketch matrices travel as one flat vector per set: the p/2 matrices of shape d x r
first, then the p/2 - 2 matrices of shape r x r, each list in the order Algorithm 1
reaches its sampling line (left subtree, right subtree, node).
"""
import ctypes
import os

import numpy as np

from . import build as _build

FEAT_SKETCH, FEAT_EXACT = 0, 1
LOCAL_EXACT, LOCAL_SKETCH = 0, 1

_lib = None
_dp = ctypes.POINTER(ctypes.c_double)
_lp = ctypes.POINTER(ctypes.c_long)


def lib():
    global _lib
    if _lib is None:
        path = os.environ.get("PSF_ORACLE_LIB")      # another build of the same source (sanitizers)
        if not path:
            path = _build.LIB
            if (not os.path.exists(path)
                    or os.path.getmtime(path) < os.path.getmtime(_build.SRC)):
                _build.build()
        L = ctypes.CDLL(path)
        L.psf_oracle_num_g_first.restype = ctypes.c_long
        L.psf_oracle_num_g_first.argtypes = [ctypes.c_long]
        L.psf_oracle_num_g_inner.restype = ctypes.c_long
        L.psf_oracle_num_g_inner.argtypes = [ctypes.c_long]
        L.psf_oracle_sketch.restype = ctypes.c_int
        L.psf_oracle_sketch.argtypes = [_dp] + [ctypes.c_long] * 4 + [_dp, _dp]
        L.psf_oracle_self_tensor.restype = None
        L.psf_oracle_self_tensor.argtypes = [_dp, ctypes.c_long, ctypes.c_long, _dp]
        L.psf_oracle_power_tensor.restype = ctypes.c_int
        L.psf_oracle_power_tensor.argtypes = [_dp] + [ctypes.c_long] * 3 + [_dp]
        L.psf_oracle_attn_def.restype = ctypes.c_int
        L.psf_oracle_attn_def.argtypes = ([_dp] * 5 + [ctypes.c_long] * 6 + [ctypes.c_int] * 3
                                          + [_lp, ctypes.c_long, _dp, _dp])
        L.psf_oracle_attn_block.restype = ctypes.c_int
        L.psf_oracle_attn_block.argtypes = ([_dp] * 5 + [ctypes.c_long] * 6
                                            + [ctypes.c_int, _dp])
        L.psf_oracle_attn_def_batch.restype = ctypes.c_int
        L.psf_oracle_attn_def_batch.argtypes = ([_dp] * 4 + [ctypes.c_long] * 9
                                                + [ctypes.c_int] * 2
                                                + [_lp, ctypes.c_long, _dp, ctypes.c_int])
        L.psf_oracle_learned_len.restype = ctypes.c_long
        L.psf_oracle_learned_len.argtypes = [ctypes.c_long] * 3
        L.psf_oracle_sketch_learned.restype = ctypes.c_int
        L.psf_oracle_sketch_learned.argtypes = [_dp] + [ctypes.c_long] * 4 + [_dp, _dp]
        L.psf_oracle_attn_noncausal.restype = ctypes.c_int
        L.psf_oracle_attn_noncausal.argtypes = ([_dp] * 5 + [ctypes.c_long] * 6 + [ctypes.c_int] * 2 + [_dp])
        L.psf_oracle_sketch_bwd.restype = ctypes.c_int
        L.psf_oracle_sketch_bwd.argtypes = [_dp] + [ctypes.c_long] * 4 + [_dp, _dp, _dp]
        L.psf_oracle_attn_bwd.restype = ctypes.c_int
        L.psf_oracle_attn_bwd.argtypes = ([_dp] * 5 + [ctypes.c_long] * 6 + [ctypes.c_int] * 2
                                          + [_dp] * 3)
        L.psf_oracle_attn_bwd_rows.restype = ctypes.c_int
        L.psf_oracle_attn_bwd_rows.argtypes = ([_dp] * 5 + [ctypes.c_long] * 6 + [ctypes.c_int] * 2
                                               + [_lp, ctypes.c_long] + [_dp] * 3)
        L.psf_oracle_sketch_learned_bwd.restype = ctypes.c_int
        L.psf_oracle_sketch_learned_bwd.argtypes = [_dp] + [ctypes.c_long] * 4 + [_dp] * 4
        L.psf_oracle_attn_bwd_learned.restype = ctypes.c_int
        L.psf_oracle_attn_bwd_learned.argtypes = ([_dp] * 5 + [ctypes.c_long] * 6 + [ctypes.c_int] + [_dp] * 4)
        L.psf_oracle_attn_bwd_batch.restype = ctypes.c_int
        L.psf_oracle_attn_bwd_batch.argtypes = ([_dp] * 4 + [ctypes.c_long] * 2 + [_dp]
                                                + [ctypes.c_long] * 7 + [ctypes.c_int] * 2
                                                + [_dp] * 3 + [ctypes.c_int])
        _lib = L
    return _lib


def _f64(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _ptr(a):
    return a.ctypes.data_as(_dp) if a is not None else None


def g_len(d, r, p):
    L = lib()
    return L.psf_oracle_num_g_first(p) * d * r + L.psf_oracle_num_g_inner(p) * r * r


def sketch(X, G, r, p):
    """m(x) = PolySketchWithNegativity(x, r, p/2) for every row of X (Algorithm 1)."""
    X = _f64(X)
    k, d = X.shape
    G = _f64(G).reshape(-1) if p > 2 else np.zeros(1)
    if p > 2 and G.size != g_len(d, r, p):
        raise ValueError("G has %d entries, expected %d" % (G.size, g_len(d, r, p)))
    M = np.empty((k, d if p == 2 else r))
    rc = lib().psf_oracle_sketch(_ptr(X), k, d, r, p, _ptr(G), _ptr(M))
    if rc:
        raise ValueError("psf_oracle_sketch failed: %d" % rc)
    return M


def self_tensor(M):
    """phi'(x) = m (x) m, index a*r + b (Algorithm 1, PolySketchNonNegative)."""
    M = _f64(M)
    k, m = M.shape
    Phi = np.empty((k, m * m))
    lib().psf_oracle_self_tensor(_ptr(M), k, m, _ptr(Phi))
    return Phi


def power_tensor(X, p):
    """x^{(x)p} (Section 2.2), d^p columns."""
    X = _f64(X)
    k, d = X.shape
    Phi = np.empty((k, d ** p))
    rc = lib().psf_oracle_power_tensor(_ptr(X), k, d, p, _ptr(Phi))
    if rc:
        raise MemoryError("psf_oracle_power_tensor failed: %d" % rc)
    return Phi


def learned_len(d, r, p):
    """Number of parameters of the learned degree-p sketch (Appendix D): p - 2 networks."""
    return lib().psf_oracle_learned_len(d, r, p)


def sketch_learned(X, params, r, p):
    """m(x) = LearnablePolysketchWithNegativity(x, r, p/2) for every row of X (Algorithm 2)."""
    X = _f64(X)
    k, d = X.shape
    P = _f64(params).reshape(-1) if p > 2 else np.zeros(1)
    if p > 2 and P.size != learned_len(d, r, p):
        raise ValueError("params has %d entries, expected %d" % (P.size, learned_len(d, r, p)))
    M = np.empty((k, d if p == 2 else r))
    rc = lib().psf_oracle_sketch_learned(_ptr(X), k, d, r, p, _ptr(P), _ptr(M))
    if rc:
        raise ValueError("psf_oracle_sketch_learned failed: %d" % rc)
    return M


def attn_def(Q, K, V, G, p, r, b, feat=FEAT_SKETCH, local=LOCAL_EXACT, rows=None,
             explicit_features=False, return_weights=False, learned=False):
    """Rows of causal Polysketch attention straight from its definition (Section 3,
    with Section 3.2's exact in-block weights when local == LOCAL_EXACT).  learned=True: G holds
    the parameters of the learned sketch (Algorithm 2) instead of Gaussian matrices."""
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    n, d = Q.shape
    dv = V.shape[1]
    MQ = MK = None
    mcols = d if p == 2 else r
    if feat == FEAT_SKETCH and learned:
        MQ, MK = sketch_learned(Q, G, r, p), sketch_learned(K, G, r, p)
    elif feat == FEAT_SKETCH:
        MQ, MK = sketch(Q, G, r, p), sketch(K, G, r, p)
    rows_a = None if rows is None else np.ascontiguousarray(np.asarray(rows, dtype=np.int64))
    nrows = n if rows_a is None else rows_a.size
    O = np.empty((nrows, dv))
    W = np.empty((nrows, n)) if return_weights else None
    rc = lib().psf_oracle_attn_def(
        _ptr(Q), _ptr(K), _ptr(V), _ptr(MQ), _ptr(MK), n, d, dv, mcols, p, b,
        feat, local, int(bool(explicit_features)),
        rows_a.ctypes.data_as(_lp) if rows_a is not None else None, nrows, _ptr(O), _ptr(W))
    if rc:
        raise ValueError("psf_oracle_attn_def failed: %d" % rc)
    return (O, W) if return_weights else O


def attn_block(Q, K, V, G, p, r, b, feat=FEAT_SKETCH, local=LOCAL_EXACT):
    """The paper's block lower-triangular algorithm with explicit features
    (Section 3.1; Section 3.2 for the in-block term when local == LOCAL_EXACT)."""
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    n, d = Q.shape
    dv = V.shape[1]
    if feat == FEAT_EXACT:
        PhiQ, PhiK = power_tensor(Q, p), power_tensor(K, p)
    else:
        PhiQ, PhiK = self_tensor(sketch(Q, G, r, p)), self_tensor(sketch(K, G, r, p))
    F = PhiQ.shape[1]
    O = np.empty((n, dv))
    local_exact = int(local == LOCAL_EXACT and feat == FEAT_SKETCH)
    rc = lib().psf_oracle_attn_block(_ptr(Q), _ptr(K), _ptr(V), _ptr(PhiQ), _ptr(PhiK),
                                     n, d, dv, F, p, b, local_exact, _ptr(O))
    if rc:
        raise ValueError("psf_oracle_attn_block failed: %d" % rc)
    return O


def attn_def_batch(Q, K, V, G, p, r, b, feat=FEAT_SKETCH, local=LOCAL_EXACT, rows=None,
                   max_threads=0):
    """attn_def over [batch, heads, n, *] inputs; G is [1 or heads, g_len].
    Returns (O [batch, heads, nrows, dv], threads_used).  OpenMP over units only."""
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    B, H, n, d = Q.shape
    dv = V.shape[-1]
    if feat == FEAT_SKETCH and p > 2:
        G = _f64(G).reshape(-1, g_len(d, r, p))
        if G.shape[0] not in (1, H):
            raise ValueError("G must have 1 or `heads` sets")
    else:
        G = np.zeros((1, 1))
    rows_a = None if rows is None else np.ascontiguousarray(np.asarray(rows, dtype=np.int64))
    nrows = n if rows_a is None else rows_a.size
    O = np.empty((B, H, nrows, dv))
    rc = lib().psf_oracle_attn_def_batch(
        _ptr(Q), _ptr(K), _ptr(V), _ptr(G), G.shape[0], H, B * H, n, d, dv, p, r, b,
        feat, local, rows_a.ctypes.data_as(_lp) if rows_a is not None else None, nrows,
        _ptr(O), int(max_threads))
    if rc < 0:
        raise ValueError("psf_oracle_attn_def_batch failed: %d" % rc)
    return O, rc


def sketch_bwd(X, G, r, p, dM):
    """(d m(x) / d x)^T dM for every row of X, m as in `sketch` (gradient of Algorithm 1)."""
    X, dM = _f64(X), _f64(dM)
    k, d = X.shape
    G = _f64(G).reshape(-1) if p > 2 else np.zeros(1)
    dX = np.empty((k, d))
    rc = lib().psf_oracle_sketch_bwd(_ptr(X), k, d, r, p, _ptr(G), _ptr(dM), _ptr(dX))
    if rc:
        raise ValueError("psf_oracle_sketch_bwd failed: %d" % rc)
    return dX


def sketch_learned_bwd(X, params, r, p, dM):
    """((d m / d x)^T dM, (d m / d params)^T dM) for the learned sketch m of `sketch_learned`
    (gradient of Algorithm 2 with respect to the input rows and to the networks' parameters)."""
    X, dM = _f64(X), _f64(dM)
    k, d = X.shape
    P = _f64(params).reshape(-1) if p > 2 else np.zeros(1)
    dX = np.empty((k, d))
    dP = np.zeros(max(learned_len(d, r, p), 1))
    rc = lib().psf_oracle_sketch_learned_bwd(_ptr(X), k, d, r, p, _ptr(P), _ptr(dM), _ptr(dX), _ptr(dP))
    if rc:
        raise ValueError("psf_oracle_sketch_learned_bwd failed: %d" % rc)
    return dX, dP[:learned_len(d, r, p)]


def attn_bwd_learned(Q, K, V, params, dO, p, r, b, local=LOCAL_EXACT):
    """Gradient of `attn_def(..., learned=True)` (all rows) with respect to Q, K, V and the
    parameters of the learned sketch, for dL/dO = dO; one unit."""
    Q, K, V, dO = _f64(Q), _f64(K), _f64(V), _f64(dO)
    n, d = Q.shape
    dv = V.shape[1]
    P = _f64(params).reshape(-1) if p > 2 else np.zeros(1)
    dQ, dK, dV = np.empty((n, d)), np.empty((n, d)), np.empty((n, dv))
    dP = np.zeros(max(learned_len(d, r, p), 1))
    rc = lib().psf_oracle_attn_bwd_learned(_ptr(Q), _ptr(K), _ptr(V), _ptr(P), _ptr(dO), n, d, dv, r, p, b,
                                           local, _ptr(dQ), _ptr(dK), _ptr(dV), _ptr(dP))
    if rc:
        raise ValueError("psf_oracle_attn_bwd_learned failed: %d" % rc)
    return dQ, dK, dV, dP[:learned_len(d, r, p)]


def attn_noncausal(Q, K, V, G, p, r, feat=FEAT_SKETCH, explicit_features=False, learned=False):
    """Non-causal Polysketch attention (Section 2.2): every query row sees every key row.
    Q is [nq, d]; K, V are [nk, d], [nk, dv]."""
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    nq, d = Q.shape
    nk, dv = V.shape
    MQ = MK = None
    mcols = d if p == 2 else r
    if feat == FEAT_SKETCH and learned:
        MQ, MK = sketch_learned(Q, G, r, p), sketch_learned(K, G, r, p)
    elif feat == FEAT_SKETCH:
        MQ, MK = sketch(Q, G, r, p), sketch(K, G, r, p)
    O = np.empty((nq, dv))
    rc = lib().psf_oracle_attn_noncausal(_ptr(Q), _ptr(K), _ptr(V), _ptr(MQ), _ptr(MK), nq, nk, d, dv, mcols, p,
                                         feat, int(bool(explicit_features)), _ptr(O))
    if rc:
        raise ValueError("psf_oracle_attn_noncausal failed: %d" % rc)
    return O


def attn_bwd(Q, K, V, G, dO, p, r, b, feat=FEAT_SKETCH, local=LOCAL_EXACT):
    """Gradient of `attn_def` (all rows) with respect to Q, K, V for dL/dO = dO; one unit."""
    Q, K, V, dO = _f64(Q), _f64(K), _f64(V), _f64(dO)
    n, d = Q.shape
    dv = V.shape[1]
    G = _f64(G).reshape(-1) if (feat == FEAT_SKETCH and p > 2) else np.zeros(1)
    dQ, dK, dV = np.empty((n, d)), np.empty((n, d)), np.empty((n, dv))
    rc = lib().psf_oracle_attn_bwd(_ptr(Q), _ptr(K), _ptr(V), _ptr(G), _ptr(dO), n, d, dv, r, p, b,
                                   feat, local, _ptr(dQ), _ptr(dK), _ptr(dV))
    if rc:
        raise ValueError("psf_oracle_attn_bwd failed: %d" % rc)
    return dQ, dK, dV


def attn_bwd_rows(Q, K, V, G, dO, p, r, b, rows, feat=FEAT_SKETCH, local=LOCAL_EXACT):
    """The sums of `attn_bwd` over the listed query rows only: dQ[i] is complete for listed i,
    dK[j] and dV[j] are complete when every i >= j is listed; other rows are partial."""
    Q, K, V, dO = _f64(Q), _f64(K), _f64(V), _f64(dO)
    n, d = Q.shape
    dv = V.shape[1]
    G = _f64(G).reshape(-1) if (feat == FEAT_SKETCH and p > 2) else np.zeros(1)
    rows_a = np.ascontiguousarray(np.asarray(rows, dtype=np.int64))
    dQ, dK, dV = np.empty((n, d)), np.empty((n, d)), np.empty((n, dv))
    rc = lib().psf_oracle_attn_bwd_rows(_ptr(Q), _ptr(K), _ptr(V), _ptr(G), _ptr(dO), n, d, dv, r, p, b,
                                        feat, local, rows_a.ctypes.data_as(_lp), rows_a.size,
                                        _ptr(dQ), _ptr(dK), _ptr(dV))
    if rc:
        raise ValueError("psf_oracle_attn_bwd_rows failed: %d" % rc)
    return dQ, dK, dV


def attn_bwd_batch(Q, K, V, G, dO, p, r, b, feat=FEAT_SKETCH, local=LOCAL_EXACT, max_threads=0):
    """attn_bwd over [batch, heads, n, *] inputs; returns (dQ, dK, dV, threads_used)."""
    Q, K, V, dO = _f64(Q), _f64(K), _f64(V), _f64(dO)
    B, H, n, d = Q.shape
    dv = V.shape[-1]
    if feat == FEAT_SKETCH and p > 2:
        G = _f64(G).reshape(-1, g_len(d, r, p))
        if G.shape[0] not in (1, H):
            raise ValueError("G must have 1 or `heads` sets")
    else:
        G = np.zeros((1, 1))
    dQ, dK, dV = np.empty_like(Q), np.empty_like(K), np.empty_like(V)
    rc = lib().psf_oracle_attn_bwd_batch(
        _ptr(Q), _ptr(K), _ptr(V), _ptr(G), G.shape[0], H, _ptr(dO), B * H, n, d, dv, p, r, b,
        feat, local, _ptr(dQ), _ptr(dK), _ptr(dV), int(max_threads))
    if rc < 0:
        raise ValueError("psf_oracle_attn_bwd_batch failed: %d" % rc)
    return dQ, dK, dV, rc
