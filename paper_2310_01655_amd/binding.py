"""ctypes binding of libpsf (include/psf.h): argument marshalling only.

torch supplies device memory and the stream; every step of the path runs inside the
library's HIP kernels.  There is no CPU fallback: a missing library or a CPU tensor
raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpsf.so")

PSF_OK = 0
F32, BF16 = 0, 1
FEAT_SKETCH, FEAT_EXACT = 0, 1
LOCAL_EXACT, LOCAL_SKETCH = 0, 1

EXPORTS = ("psf_check_desc", "psf_kernel_path", "psf_fwd_beside_states", "psf_workspace_bytes", "psf_g_len", "psf_learned_len",
           "psf_sketch",
           "psf_causal_attn_fwd", "psf_causal_attn_fwd_static", "psf_causal_attn_fwd_timed", "psf_stage_name",
           "psf_status_string", "psf_noncausal_workspace_bytes", "psf_noncausal_attn_fwd",
           "psf_noncausal_attn_fwd_timed", "psf_fwd_save_bytes", "psf_causal_attn_fwd_save",
           "psf_causal_attn_bwd_saved", "psf_causal_attn_bwd_saved_learned", "psf_bwd_kernel_path", "psf_bwd_workspace_bytes", "psf_causal_attn_bwd",
           "psf_causal_attn_bwd_learned",
           "psf_causal_attn_bwd_timed", "psf_decode_state_bytes", "psf_decode_reset",
           "psf_decode_step", "psf_decode_prefill_workspace_bytes", "psf_decode_prefill", "psf_probe_mfma_loop")


class PsfDesc(ctypes.Structure):
    _fields_ = [(name, ctypes.c_int32) for name in
                ("batch", "heads", "n", "d", "dv", "p", "r", "b", "dtype", "feat", "local",
                 "sketch_per_head", "learned")]


class PsfError(RuntimeError):
    def __init__(self, code, where):
        self.code = int(code)
        super().__init__("%s: %s (status %d)" % (where, status_string(code), code))


_lib = None


def lib():
    """Load libpsf.so (built in-tree by build.py).  Raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                "%s not found: build it first (python -m paper_2310_01655_amd.build or "
                "__graft_entry__.build())" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        dp = ctypes.POINTER(PsfDesc)
        vp = ctypes.c_void_p
        L.psf_check_desc.restype = ctypes.c_int
        L.psf_check_desc.argtypes = [dp]
        L.psf_kernel_path.restype = ctypes.c_int
        L.psf_kernel_path.argtypes = [dp]
        L.psf_fwd_beside_states.restype = ctypes.c_int
        L.psf_fwd_beside_states.argtypes = [dp]
        L.psf_workspace_bytes.restype = ctypes.c_size_t
        L.psf_workspace_bytes.argtypes = [dp]
        L.psf_g_len.restype = ctypes.c_size_t
        L.psf_g_len.argtypes = [ctypes.c_int32] * 3
        L.psf_learned_len.restype = ctypes.c_size_t
        L.psf_learned_len.argtypes = [ctypes.c_int32] * 3
        L.psf_sketch.restype = ctypes.c_int
        L.psf_sketch.argtypes = [dp, vp, vp, vp, vp, vp]
        L.psf_causal_attn_fwd.restype = ctypes.c_int
        L.psf_causal_attn_fwd.argtypes = [dp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        L.psf_causal_attn_fwd_static.restype = ctypes.c_int
        L.psf_causal_attn_fwd_static.argtypes = [dp, vp, vp, vp, vp, vp, vp]
        L.psf_causal_attn_fwd_timed.restype = ctypes.c_int
        L.psf_causal_attn_fwd_timed.argtypes = [dp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp,
                                                ctypes.POINTER(ctypes.c_float), ctypes.c_int32,
                                                ctypes.POINTER(ctypes.c_int32)]
        L.psf_noncausal_workspace_bytes.restype = ctypes.c_size_t
        L.psf_noncausal_workspace_bytes.argtypes = [dp]
        L.psf_noncausal_attn_fwd.restype = ctypes.c_int
        L.psf_noncausal_attn_fwd.argtypes = L.psf_causal_attn_fwd.argtypes
        L.psf_noncausal_attn_fwd_timed.restype = ctypes.c_int
        L.psf_noncausal_attn_fwd_timed.argtypes = L.psf_causal_attn_fwd_timed.argtypes
        L.psf_fwd_save_bytes.restype = ctypes.c_size_t
        L.psf_fwd_save_bytes.argtypes = [dp]
        L.psf_causal_attn_fwd_save.restype = ctypes.c_int
        L.psf_causal_attn_fwd_save.argtypes = [dp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        L.psf_causal_attn_bwd_saved.restype = ctypes.c_int
        L.psf_causal_attn_bwd_saved.argtypes = [dp] + [vp] * 9 + [vp, ctypes.c_size_t, vp, ctypes.c_size_t, vp]
        L.psf_causal_attn_bwd_saved_learned.restype = ctypes.c_int
        L.psf_causal_attn_bwd_saved_learned.argtypes = [dp] + [vp] * 10 + [vp, ctypes.c_size_t, vp, ctypes.c_size_t, vp]
        L.psf_bwd_kernel_path.restype = ctypes.c_int
        L.psf_bwd_kernel_path.argtypes = [dp]
        L.psf_bwd_workspace_bytes.restype = ctypes.c_size_t
        L.psf_bwd_workspace_bytes.argtypes = [dp]
        L.psf_causal_attn_bwd.restype = ctypes.c_int
        L.psf_causal_attn_bwd.argtypes = [dp] + [vp] * 9 + [ctypes.c_size_t, vp]
        L.psf_causal_attn_bwd_learned.restype = ctypes.c_int
        L.psf_causal_attn_bwd_learned.argtypes = [dp] + [vp] * 10 + [ctypes.c_size_t, vp]
        L.psf_causal_attn_bwd_timed.restype = ctypes.c_int
        L.psf_causal_attn_bwd_timed.argtypes = [dp] + [vp] * 9 + [ctypes.c_size_t, vp,
                                                                  ctypes.POINTER(ctypes.c_float),
                                                                  ctypes.c_int32,
                                                                  ctypes.POINTER(ctypes.c_int32)]
        L.psf_decode_state_bytes.restype = ctypes.c_size_t
        L.psf_decode_state_bytes.argtypes = [dp]
        L.psf_decode_reset.restype = ctypes.c_int
        L.psf_decode_reset.argtypes = [dp, vp, ctypes.c_size_t, vp]
        L.psf_decode_step.restype = ctypes.c_int
        L.psf_decode_step.argtypes = [dp, vp, vp, vp, vp, ctypes.c_int32, vp, ctypes.c_size_t, vp, vp]
        L.psf_decode_prefill_workspace_bytes.restype = ctypes.c_size_t
        L.psf_decode_prefill_workspace_bytes.argtypes = [dp, ctypes.c_int32]
        L.psf_decode_prefill.restype = ctypes.c_int
        L.psf_decode_prefill.argtypes = [dp, vp, vp, vp, ctypes.c_int32, vp, ctypes.c_size_t, vp, ctypes.c_size_t, vp]
        L.psf_probe_mfma_loop.restype = ctypes.c_int
        L.psf_probe_mfma_loop.argtypes = [ctypes.c_int32, ctypes.c_int32, vp, vp]
        L.psf_stage_name.restype = ctypes.c_char_p
        L.psf_stage_name.argtypes = [ctypes.c_int, ctypes.c_int32]
        L.psf_status_string.restype = ctypes.c_char_p
        L.psf_status_string.argtypes = [ctypes.c_int]
        _lib = L
    return _lib


def status_string(code):
    return lib().psf_status_string(int(code)).decode()


def make_desc(batch, heads, n, d, p, r, b, dtype="bf16", dv=None, feat=FEAT_SKETCH,
              local=LOCAL_EXACT, per_head=False, learned=False):
    code = {"f32": F32, "bf16": BF16}[dtype] if isinstance(dtype, str) else int(dtype)
    return PsfDesc(batch, heads, n, d, d if dv is None else dv, p, r, b, code, int(feat),
                   int(local), int(bool(per_head)), int(bool(learned)))


def check_desc(desc):
    return lib().psf_check_desc(ctypes.byref(desc))


def kernel_path(desc):
    return lib().psf_kernel_path(ctypes.byref(desc))


def fwd_beside_states(desc):
    """Bit 0: in-block part + denominator scan run in the state kernel's launch; bit 1: the query sketch too."""
    return lib().psf_fwd_beside_states(ctypes.byref(desc))


def workspace_bytes(desc):
    return lib().psf_workspace_bytes(ctypes.byref(desc))


def g_len(d, r, p):
    return lib().psf_g_len(d, r, p)


def _torch_dtype(desc):
    return torch.bfloat16 if desc.dtype == BF16 else torch.float32


def _dev_ptr(t, desc, shape, name):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("%s must live on the GPU (no CPU path exists)" % name)
    if t.dtype != _torch_dtype(desc):
        raise ValueError("%s has dtype %s, descriptor says %s" % (name, t.dtype, _torch_dtype(desc)))
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError("%s has shape %s, expected %s" % (name, tuple(t.shape), tuple(shape)))
    return ctypes.c_void_p(t.data_ptr())


def _stream_ptr(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def learned_len(d, r, p):
    return lib().psf_learned_len(d, r, p)


def _g_shape(desc):
    if desc.feat == FEAT_EXACT or desc.p == 2:
        return None
    per_set = learned_len(desc.d, desc.r, desc.p) if desc.learned else g_len(desc.d, desc.r, desc.p)
    return (desc.heads if desc.sketch_per_head else 1, per_set)


def alloc_workspace(desc, device="cuda"):
    nbytes = workspace_bytes(desc)
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)


def psf_sketch(desc, X, G, want_m=True, want_phi=False, stream=None):
    """Algorithm 1 on every row of X.  Returns (M or None, Phi or None)."""
    st = check_desc(desc)
    if st != PSF_OK:
        raise PsfError(st, "psf_sketch")
    B, H, n, d = desc.batch, desc.heads, desc.n, desc.d
    exact = desc.feat == FEAT_EXACT
    mcols = d if desc.p == 2 else desc.r
    F = d ** desc.p if exact else mcols * mcols
    x_ptr = _dev_ptr(X, desc, (B, H, n, d), "X")
    g_ptr = _dev_ptr(G, desc, _g_shape(desc), "G") if _g_shape(desc) else None
    M = torch.empty(B, H, n, mcols, dtype=X.dtype, device=X.device) if (want_m and not exact) else None
    Phi = torch.empty(B, H, n, F, dtype=X.dtype, device=X.device) if want_phi else None
    st = lib().psf_sketch(ctypes.byref(desc), x_ptr, g_ptr,
                          ctypes.c_void_p(M.data_ptr()) if M is not None else None,
                          ctypes.c_void_p(Phi.data_ptr()) if Phi is not None else None,
                          _stream_ptr(stream))
    if st != PSF_OK:
        raise PsfError(st, "psf_sketch")
    return M, Phi


def _attn_args(desc, Q, K, V, G, O, workspace, noncausal=False):
    B, H, n, d, dv = desc.batch, desc.heads, desc.n, desc.d, desc.dv
    if O is None:
        O = torch.empty(B, H, n, dv, dtype=Q.dtype, device=Q.device)
    if workspace is None:
        workspace = alloc_noncausal_workspace(desc, Q.device) if noncausal else alloc_workspace(desc, Q.device)
    if not workspace.is_cuda or workspace.dtype != torch.uint8:
        raise ValueError("workspace must be a uint8 GPU tensor")
    gs = _g_shape(desc)
    ptrs = [_dev_ptr(Q, desc, (B, H, n, d), "Q"), _dev_ptr(K, desc, (B, H, n, d), "K"),
            _dev_ptr(V, desc, (B, H, n, dv), "V"),
            _dev_ptr(G, desc, gs, "G") if gs else None,
            _dev_ptr(O, desc, (B, H, n, dv), "O"),
            ctypes.c_void_p(workspace.data_ptr()), ctypes.c_size_t(workspace.numel())]
    return O, workspace, ptrs


def psf_causal_attn_fwd(desc, Q, K, V, G, O=None, workspace=None, stream=None):
    """Causal Polysketch attention forward; returns O [batch, heads, n, dv] (device)."""
    st = check_desc(desc)
    if st != PSF_OK:
        raise PsfError(st, "psf_causal_attn_fwd")
    O, workspace, ptrs = _attn_args(desc, Q, K, V, G, O, workspace)
    st = lib().psf_causal_attn_fwd(ctypes.byref(desc), *ptrs, _stream_ptr(stream))
    if st != PSF_OK:
        raise PsfError(st, "psf_causal_attn_fwd")
    return O


STATIC_SCRATCH_BYTES = 32 << 20      # PSF_STATIC_SCRATCH_BYTES of include/psf.h


def psf_causal_attn_fwd_static(desc, Q, K, V, G, O, stream=None):
    """The forward call on the library's own static device scratch: no workspace argument and
    no allocation anywhere (O is the caller's, so this wrapper allocates nothing either)."""
    B, H, n, d, dv = desc.batch, desc.heads, desc.n, desc.d, desc.dv
    gs = _g_shape(desc)
    st = lib().psf_causal_attn_fwd_static(
        ctypes.byref(desc), _dev_ptr(Q, desc, (B, H, n, d), "Q"), _dev_ptr(K, desc, (B, H, n, d), "K"),
        _dev_ptr(V, desc, (B, H, n, dv), "V"), _dev_ptr(G, desc, gs, "G") if gs else None,
        _dev_ptr(O, desc, (B, H, n, dv), "O"), _stream_ptr(stream))
    if st != PSF_OK:
        raise PsfError(st, "psf_causal_attn_fwd_static")
    return O


def psf_causal_attn_fwd_timed(desc, Q, K, V, G, O=None, workspace=None, stream=None):
    """Same call with per-kernel HIP-event timing; returns (O, {stage_name: ms})."""
    st = check_desc(desc)
    if st != PSF_OK:
        raise PsfError(st, "psf_causal_attn_fwd_timed")
    O, workspace, ptrs = _attn_args(desc, Q, K, V, G, O, workspace)
    ms = (ctypes.c_float * 16)()
    written = ctypes.c_int32(0)
    st = lib().psf_causal_attn_fwd_timed(ctypes.byref(desc), *ptrs, _stream_ptr(stream), ms, 16,
                                         ctypes.byref(written))
    if st != PSF_OK:
        raise PsfError(st, "psf_causal_attn_fwd_timed")
    path = kernel_path(desc)
    names = [lib().psf_stage_name(path, i).decode() for i in range(written.value)]
    return O, {nm: float(ms[i]) for i, nm in enumerate(names)}


def noncausal_workspace_bytes(desc):
    return lib().psf_noncausal_workspace_bytes(ctypes.byref(desc))


def alloc_noncausal_workspace(desc, device="cuda"):
    return torch.empty(max(noncausal_workspace_bytes(desc), 256), dtype=torch.uint8, device=device)


def psf_noncausal_attn_fwd(desc, Q, K, V, G, O=None, workspace=None, stream=None):
    """Polysketch attention without a mask (every query sees every key); returns O."""
    st = check_desc(desc)
    if st != PSF_OK:
        raise PsfError(st, "psf_noncausal_attn_fwd")
    O, workspace, ptrs = _attn_args(desc, Q, K, V, G, O, workspace, noncausal=True)
    st = lib().psf_noncausal_attn_fwd(ctypes.byref(desc), *ptrs, _stream_ptr(stream))
    if st != PSF_OK:
        raise PsfError(st, "psf_noncausal_attn_fwd")
    return O


def psf_noncausal_attn_fwd_timed(desc, Q, K, V, G, O=None, workspace=None, stream=None):
    """Same call with per-kernel HIP-event timing; returns (O, {stage_name: ms})."""
    st = check_desc(desc)
    if st != PSF_OK:
        raise PsfError(st, "psf_noncausal_attn_fwd_timed")
    O, workspace, ptrs = _attn_args(desc, Q, K, V, G, O, workspace, noncausal=True)
    ms = (ctypes.c_float * 16)()
    written = ctypes.c_int32(0)
    st = lib().psf_noncausal_attn_fwd_timed(ctypes.byref(desc), *ptrs, _stream_ptr(stream), ms, 16,
                                            ctypes.byref(written))
    if st != PSF_OK:
        raise PsfError(st, "psf_noncausal_attn_fwd_timed")
    path = kernel_path(desc)
    names = [lib().psf_stage_name(path, i).decode() for i in range(written.value)]
    return O, {nm: float(ms[i]) for i, nm in enumerate(names)}


def fwd_save_bytes(desc):
    """Bytes of the buffer psf_causal_attn_fwd_save fills for psf_causal_attn_bwd_saved (0: not available)."""
    return lib().psf_fwd_save_bytes(ctypes.byref(desc))


def psf_causal_attn_fwd_save(desc, Q, K, V, G, O=None, save=None, stream=None):
    """Forward pass that keeps what the backward pass needs; returns (O, save)."""
    st = check_desc(desc)
    if st != PSF_OK:
        raise PsfError(st, "psf_causal_attn_fwd_save")
    if save is None:
        save = torch.empty(max(fwd_save_bytes(desc), 256), dtype=torch.uint8, device=Q.device)
    O, _, ptrs = _attn_args(desc, Q, K, V, G, O, save)
    st = lib().psf_causal_attn_fwd_save(ctypes.byref(desc), *ptrs, _stream_ptr(stream))
    if st != PSF_OK:
        raise PsfError(st, "psf_causal_attn_fwd_save")
    return O, save


def _bwd_saved(desc, Q, K, V, G, O, dO, save, workspace, stream, out, learned):
    B, H, n, d, dv = desc.batch, desc.heads, desc.n, desc.d, desc.dv
    if workspace is None:
        workspace = alloc_bwd_workspace(desc, Q.device)
    dQ, dK, dV = out if out is not None else (torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V))
    gs = _g_shape(desc)
    ptrs = [_dev_ptr(Q, desc, (B, H, n, d), "Q"), _dev_ptr(K, desc, (B, H, n, d), "K"),
            _dev_ptr(V, desc, (B, H, n, dv), "V"), _dev_ptr(G, desc, gs, "G") if gs else None,
            _dev_ptr(O, desc, (B, H, n, dv), "O"), _dev_ptr(dO, desc, (B, H, n, dv), "dO"),
            _dev_ptr(dQ, desc, (B, H, n, d), "dQ"), _dev_ptr(dK, desc, (B, H, n, d), "dK"),
            _dev_ptr(dV, desc, (B, H, n, dv), "dV")]
    tail = [ctypes.c_void_p(save.data_ptr()), ctypes.c_size_t(save.numel()),
            ctypes.c_void_p(workspace.data_ptr()), ctypes.c_size_t(workspace.numel()), _stream_ptr(stream)]
    if not learned:
        st = lib().psf_causal_attn_bwd_saved(ctypes.byref(desc), *ptrs, *tail)
        if st != PSF_OK:
            raise PsfError(st, "psf_causal_attn_bwd_saved")
        return dQ, dK, dV
    dG = torch.empty(gs if gs else (1,), dtype=torch.float32, device=Q.device)
    st = lib().psf_causal_attn_bwd_saved_learned(ctypes.byref(desc), *ptrs, ctypes.c_void_p(dG.data_ptr()), *tail)
    if st != PSF_OK:
        raise PsfError(st, "psf_causal_attn_bwd_saved_learned")
    return dQ, dK, dV, dG


def psf_causal_attn_bwd_saved(desc, Q, K, V, G, O, dO, save, workspace=None, stream=None, out=None):
    """Backward pass from the buffer psf_causal_attn_fwd_save left; returns (dQ, dK, dV)."""
    return _bwd_saved(desc, Q, K, V, G, O, dO, save, workspace, stream, out, False)


def psf_causal_attn_bwd_saved_learned(desc, Q, K, V, G, O, dO, save, workspace=None, stream=None, out=None):
    """The same with learned sketches and the gradient of the networks' parameters; returns
    (dQ, dK, dV, dG) with dG fp32 of G's shape."""
    return _bwd_saved(desc, Q, K, V, G, O, dO, save, workspace, stream, out, True)


def bwd_kernel_path(desc):
    """2 = general fp32 kernels, 3 = MFMA kernels, -1 = invalid or unsupported."""
    return lib().psf_bwd_kernel_path(ctypes.byref(desc))


def bwd_workspace_bytes(desc):
    return lib().psf_bwd_workspace_bytes(ctypes.byref(desc))


def alloc_bwd_workspace(desc, device="cuda"):
    return torch.empty(max(bwd_workspace_bytes(desc), 256), dtype=torch.uint8, device=device)


def _bwd_args(desc, Q, K, V, G, dO, workspace):
    B, H, n, d, dv = desc.batch, desc.heads, desc.n, desc.d, desc.dv
    if workspace is None:
        workspace = alloc_bwd_workspace(desc, Q.device)
    if not workspace.is_cuda or workspace.dtype != torch.uint8:
        raise ValueError("workspace must be a uint8 GPU tensor")
    dQ, dK, dV = torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V)
    gs = _g_shape(desc)
    ptrs = [_dev_ptr(Q, desc, (B, H, n, d), "Q"), _dev_ptr(K, desc, (B, H, n, d), "K"),
            _dev_ptr(V, desc, (B, H, n, dv), "V"),
            _dev_ptr(G, desc, gs, "G") if gs else None,
            _dev_ptr(dO, desc, (B, H, n, dv), "dO"),
            ctypes.c_void_p(dQ.data_ptr()), ctypes.c_void_p(dK.data_ptr()),
            ctypes.c_void_p(dV.data_ptr()),
            ctypes.c_void_p(workspace.data_ptr()), ctypes.c_size_t(workspace.numel())]
    # the workspace is handed back so that the caller holds it until the call is enqueued: a
    # tensor allocated in between must not be given the same memory
    return (dQ, dK, dV), ptrs, workspace


def psf_causal_attn_bwd(desc, Q, K, V, G, dO, workspace=None, stream=None):
    """Gradient of the forward output with respect to Q, K, V; returns (dQ, dK, dV)."""
    st = check_desc(desc)
    if st != PSF_OK:
        raise PsfError(st, "psf_causal_attn_bwd")
    grads, ptrs, workspace = _bwd_args(desc, Q, K, V, G, dO, workspace)
    st = lib().psf_causal_attn_bwd(ctypes.byref(desc), *ptrs, _stream_ptr(stream))
    if st != PSF_OK:
        raise PsfError(st, "psf_causal_attn_bwd")
    return grads


def psf_causal_attn_bwd_learned(desc, Q, K, V, G, dO, workspace=None, stream=None):
    """Learned sketches: gradient with respect to Q, K, V and to the networks' parameters;
    returns (dQ, dK, dV, dG) with dG fp32 of G's shape."""
    st = check_desc(desc)
    if st != PSF_OK:
        raise PsfError(st, "psf_causal_attn_bwd_learned")
    grads, ptrs, workspace = _bwd_args(desc, Q, K, V, G, dO, workspace)
    gs = _g_shape(desc)
    dG = torch.empty(gs if gs else (1,), dtype=torch.float32, device=Q.device)
    ptrs = ptrs[:8] + [ctypes.c_void_p(dG.data_ptr())] + ptrs[8:]
    st = lib().psf_causal_attn_bwd_learned(ctypes.byref(desc), *ptrs, _stream_ptr(stream))
    if st != PSF_OK:
        raise PsfError(st, "psf_causal_attn_bwd_learned")
    return grads + (dG,)


def psf_causal_attn_bwd_timed(desc, Q, K, V, G, dO, workspace=None, stream=None):
    """Same call with per-stage HIP-event timing; returns ((dQ, dK, dV), {stage_name: ms})."""
    st = check_desc(desc)
    if st != PSF_OK:
        raise PsfError(st, "psf_causal_attn_bwd_timed")
    grads, ptrs, workspace = _bwd_args(desc, Q, K, V, G, dO, workspace)
    ms = (ctypes.c_float * 16)()
    written = ctypes.c_int32(0)
    st = lib().psf_causal_attn_bwd_timed(ctypes.byref(desc), *ptrs, _stream_ptr(stream), ms, 16,
                                         ctypes.byref(written))
    if st != PSF_OK:
        raise PsfError(st, "psf_causal_attn_bwd_timed")
    path = lib().psf_bwd_kernel_path(ctypes.byref(desc))
    names = [lib().psf_stage_name(path, i).decode() for i in range(written.value)]
    return grads, {nm: float(ms[i]) for i, nm in enumerate(names)}


def decode_state_bytes(desc):
    return lib().psf_decode_state_bytes(ctypes.byref(desc))


def decode_new_state(desc, device="cuda", stream=None):
    """Allocate (torch) and reset the state of token-by-token evaluation."""
    nbytes = decode_state_bytes(desc)
    if nbytes == 0:
        raise PsfError(lib().psf_check_desc(ctypes.byref(desc)) or 3, "psf_decode_state_bytes")
    state = torch.empty(nbytes, dtype=torch.uint8, device=device)
    st = lib().psf_decode_reset(ctypes.byref(desc), ctypes.c_void_p(state.data_ptr()),
                                ctypes.c_size_t(state.numel()), _stream_ptr(stream))
    if st != PSF_OK:
        raise PsfError(st, "psf_decode_reset")
    return state


def psf_decode_prefill(desc, K, V, G, state, stream=None):
    """State after the prompt K, V ([batch, heads, n_prompt, d | dv]); next: psf_decode_step at pos = n_prompt."""
    B, H, d, dv = desc.batch, desc.heads, desc.d, desc.dv
    n_prompt = int(K.shape[2])
    need = lib().psf_decode_prefill_workspace_bytes(ctypes.byref(desc), n_prompt)
    ws = torch.empty(max(need, 1), dtype=torch.uint8, device=K.device)
    gs = _g_shape(desc)
    st = lib().psf_decode_prefill(
        ctypes.byref(desc), _dev_ptr(K, desc, (B, H, n_prompt, d), "K"), _dev_ptr(V, desc, (B, H, n_prompt, dv), "V"),
        _dev_ptr(G, desc, gs, "G") if gs else None, n_prompt, ctypes.c_void_p(state.data_ptr()),
        ctypes.c_size_t(state.numel()), ctypes.c_void_p(ws.data_ptr()) if need else None, ctypes.c_size_t(need),
        _stream_ptr(stream))
    if st != PSF_OK:
        raise PsfError(st, "psf_decode_prefill")
    return ws      # alive until the caller has synchronised


def psf_decode_step(desc, q, k, v, G, pos, state, o=None, stream=None):
    """Row `pos` of the attention for the sequence fed so far; q, k, v are [batch, heads, 1, d|dv]."""
    B, H, d, dv = desc.batch, desc.heads, desc.d, desc.dv
    if o is None:
        o = torch.empty(B, H, 1, dv, dtype=q.dtype, device=q.device)
    gs = _g_shape(desc)
    st = lib().psf_decode_step(
        ctypes.byref(desc), _dev_ptr(q, desc, (B, H, 1, d), "q"), _dev_ptr(k, desc, (B, H, 1, d), "k"),
        _dev_ptr(v, desc, (B, H, 1, dv), "v"), _dev_ptr(G, desc, gs, "G") if gs else None, int(pos),
        ctypes.c_void_p(state.data_ptr()), ctypes.c_size_t(state.numel()),
        _dev_ptr(o, desc, (B, H, 1, dv), "o"), _stream_ptr(stream))
    if st != PSF_OK:
        raise PsfError(st, "psf_decode_step")
    return o


def psf_probe_mfma_loop(workgroups, iters, sink, stream=None):
    """Pure MFMA loop (measurement aid): workgroups x 4 waves x iters x 8 MFMAs of 32768 flops.
    Returns the flop count of the launch."""
    if not sink.is_cuda or sink.dtype != torch.float32 or sink.numel() < workgroups * 256:
        raise ValueError("sink must be a float32 GPU tensor of at least workgroups * 256 entries")
    st = lib().psf_probe_mfma_loop(int(workgroups), int(iters), ctypes.c_void_p(sink.data_ptr()), _stream_ptr(stream))
    if st != PSF_OK:
        raise PsfError(st, "psf_probe_mfma_loop")
    return workgroups * 4 * iters * 8 * 32768
