"""Host-only checks of the C ABI: the library loads, exports every symbol the header declares,
and validates descriptors and pointers before anything is launched (no GPU needed)."""
import ctypes
import os
import re

import pytest

from paper_2310_01655_amd import binding as psf

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_symbols():
    text = open(os.path.join(ROOT, "include", "psf.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(psf_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = psf.lib()
    names = header_symbols()
    assert set(names) == set(psf.EXPORTS), names
    for nm in names:
        assert getattr(L, nm) is not None


def good():
    return psf.make_desc(2, 12, 32768, 64, 4, 64, 1024, "bf16")


def test_descriptor_validation_codes():
    assert psf.check_desc(good()) == 0
    assert psf.lib().psf_check_desc(None) == 1
    for field, val, code in [("n", 0, 2), ("batch", -1, 2), ("b", 1000, 2), ("r", 0, 2),
                             ("p", 6, 3), ("p", 32, 3), ("dtype", 7, 3), ("feat", 2, 3),
                             ("local", -1, 3), ("d", 512, 3), ("r", 300, 3)]:
        d = good()
        setattr(d, field, val)
        assert psf.check_desc(d) == code, (field, val)
        assert psf.workspace_bytes(d) == 0 and psf.kernel_path(d) == -1
    # exact features: d^p must stay within the stated cap
    assert psf.check_desc(psf.make_desc(1, 1, 64, 8, 4, 1, 8, "f32", feat=psf.FEAT_EXACT)) == 0
    assert psf.check_desc(psf.make_desc(1, 1, 64, 16, 4, 1, 8, "f32", feat=psf.FEAT_EXACT)) == 0
    assert psf.check_desc(psf.make_desc(1, 1, 64, 64, 4, 1, 8, "f32", feat=psf.FEAT_EXACT)) == 3
    # r is ignored for p = 2 (Algorithm 1's base case returns the input)
    assert psf.check_desc(psf.make_desc(1, 1, 64, 64, 2, 0, 8, "f32")) == 0


def test_path_selection_and_workspace():
    assert psf.kernel_path(psf.make_desc(1, 1, 1024, 64, 4, 16, 128, "f32")) == 0
    assert psf.kernel_path(psf.make_desc(1, 1, 1024, 64, 4, 64, 128, "f32")) == 0
    d1 = psf.make_desc(1, 1, 1024, 64, 4, 16, 128, "f32")
    # general path: m(Q), m(K) in fp32 and t states of r^2 x (dv+1) fp32
    assert psf.workspace_bytes(d1) >= 2 * 1024 * 16 * 4 + 8 * 256 * 65 * 4
    assert psf.g_len(64, 64, 4) == 2 * 64 * 64
    assert psf.g_len(128, 64, 8) == 4 * 128 * 64 + 2 * 64 * 64
    assert psf.g_len(64, 8, 16) == 8 * 64 * 8 + 6 * 8 * 8
    assert psf.g_len(64, 8, 2) == 0


def test_null_pointers_are_rejected_before_any_launch():
    L = psf.lib()
    d = psf.make_desc(1, 1, 1024, 64, 4, 16, 128, "f32")
    ref = ctypes.byref(d)
    one = ctypes.c_void_p(256)   # never dereferenced: the calls must fail on the NULL first
    assert L.psf_sketch(ref, None, one, one, None, None) == 1
    assert L.psf_sketch(ref, one, None, one, None, None) == 1
    assert L.psf_sketch(ref, one, one, None, None, None) == 1
    assert L.psf_causal_attn_fwd(ref, None, one, one, one, one, one, 1 << 40, None) == 1
    assert L.psf_causal_attn_fwd(ref, one, one, one, one, None, one, 1 << 40, None) == 1
    assert L.psf_causal_attn_fwd(ref, one, one, one, None, one, one, 1 << 40, None) == 1
    assert L.psf_causal_attn_fwd(ref, one, one, one, one, one, one, 16, None) == 4
    assert L.psf_causal_attn_fwd(ref, one, one, one, one, one, ctypes.c_void_p(264), 1 << 40, None) == 4
    d.p = 5
    assert L.psf_causal_attn_fwd(ref, one, one, one, one, one, one, 1 << 40, None) == 3
    assert L.psf_causal_attn_fwd_timed(ref, one, one, one, one, one, one, 1 << 40, None, None, 0, None) == 1


def test_backward_entry_point_validates_on_the_host():
    L = psf.lib()
    d = psf.make_desc(1, 1, 1024, 64, 4, 16, 128, "f32")
    ref = ctypes.byref(d)
    one = ctypes.c_void_p(256)   # never dereferenced: every call below fails validation first
    need = psf.bwd_workspace_bytes(d)
    # m(Q), m(K) and their gradients, [V|1] and G_i rows, both state arrays, direct dQ / dK terms
    rows, kc = 1024, 65
    assert need >= 4 * rows * 16 * 4 + 2 * rows * kc * 4 + 2 * 8 * 256 * kc * 4 + 2 * rows * 64 * 4
    big = 1 << 40
    args = [one] * 8
    for hole in (0, 1, 2, 3, 4, 5, 6, 7):                                    # each required pointer
        a = list(args)
        a[hole] = None
        assert L.psf_causal_attn_bwd(ref, *a, one, big, None) == 1, hole
    assert L.psf_causal_attn_bwd(ref, *args, None, big, None) == 1
    assert L.psf_causal_attn_bwd(ref, *args, one, need - 1, None) == 4
    assert L.psf_causal_attn_bwd(ref, *args, ctypes.c_void_p(264), big, None) == 4
    exact = psf.make_desc(1, 1, 64, 8, 4, 1, 8, "f32", feat=psf.FEAT_EXACT)
    assert psf.bwd_workspace_bytes(exact) == 0
    assert L.psf_causal_attn_bwd(ctypes.byref(exact), *args, one, big, None) == 3
    assert L.psf_causal_attn_bwd_timed(ref, *args, one, big, None, None, 0, None) == 1
    assert psf.lib().psf_stage_name(2, 0) == b"sketches"
    assert psf.lib().psf_stage_name(2, 5) == b"sketch_gradient"


def test_backward_kernel_path_and_mfma_workspace():
    mf = psf.make_desc(2, 12, 32768, 64, 4, 64, 1024, "bf16")                 # config 3
    assert psf.bwd_kernel_path(mf) == 3
    rows = 2 * 12 * 32768
    snaps = 2 * 12 * 31
    # forward workspace + two more sets of state snapshots + the fp32 gradient accumulators
    assert psf.bwd_workspace_bytes(mf) >= psf.workspace_bytes(mf) + 2 * snaps * 64 * 64 * 64 * 2 + 5 * rows * 64 * 4
    assert psf.bwd_kernel_path(psf.make_desc(1, 1, 1024, 64, 4, 16, 128, "f32")) == 2
    assert psf.bwd_kernel_path(psf.make_desc(1, 2, 1024, 128, 4, 64, 256, "bf16")) == 3     # d = 128
    assert psf.bwd_kernel_path(psf.make_desc(1, 2, 1024, 64, 8, 64, 256, "bf16")) == 3      # p = 8
    assert psf.bwd_kernel_path(psf.make_desc(1, 16, 16384, 128, 8, 64, 512, "bf16")) == 3   # config 5
    assert psf.bwd_kernel_path(psf.make_desc(1, 2, 1024, 128, 8, 64, 256, "bf16", local=psf.LOCAL_SKETCH)) == 2
    assert psf.bwd_kernel_path(psf.make_desc(1, 2, 1024, 64, 16, 64, 256, "bf16")) == 2     # p = 16
    # learned sketches of degree 4 with exact in-block weights: the MFMA kernels; other degrees,
    # the in-block rule of Section 3.1 and fp32 storage: the general ones
    learned = psf.make_desc(1, 2, 1024, 64, 4, 64, 256, "bf16", learned=True)
    plain = psf.make_desc(1, 2, 1024, 64, 4, 64, 256, "bf16")
    assert psf.bwd_kernel_path(learned) == 3
    rows = 2 * 1024
    # the Gaussian-sketch workspace + staged r-wide vectors of both networks (rows and tiles) + the
    # per-unit parameter sums of both sides
    assert psf.bwd_workspace_bytes(learned) >= (psf.bwd_workspace_bytes(plain) + 2 * rows * 64 * 2 + 12 * rows * 64 * 2
                                                + 2 * 2 * psf.lib().psf_learned_len(64, 64, 4) * 4)
    assert psf.fwd_save_bytes(learned) > psf.workspace_bytes(learned)                      # the saving forward covers it
    assert psf.bwd_kernel_path(psf.make_desc(1, 2, 1024, 64, 8, 64, 256, "bf16", learned=True)) == 2
    assert psf.bwd_kernel_path(psf.make_desc(1, 2, 1024, 64, 4, 64, 256, "bf16", learned=True,
                                             local=psf.LOCAL_SKETCH)) == 2
    learned_general = psf.make_desc(1, 2, 1024, 64, 4, 64, 256, "f32", learned=True)
    plain_general = psf.make_desc(1, 2, 1024, 64, 4, 64, 256, "f32")
    assert psf.bwd_kernel_path(learned_general) == 2
    # the general workspace plus the staging the parameter sums read (here 2048 rows of 2 networks)
    assert psf.bwd_workspace_bytes(learned_general) >= psf.bwd_workspace_bytes(plain_general) + 2048 * 2 * (3 * 64 + 6 * 512 + 3 * 64) * 4
    assert psf.bwd_kernel_path(plain) == 3
    assert psf.lib().psf_stage_name(3, 0) == b"forward_again"
    assert psf.lib().psf_stage_name(3, 4) == b"cross_block_and_sketch_gradient"


def test_noncausal_entry_point_validates_on_the_host():
    L = psf.lib()
    d = psf.make_desc(1, 1, 1024, 64, 4, 16, 128, "f32")
    ref = ctypes.byref(d)
    one = ctypes.c_void_p(256)   # never dereferenced: every call below fails validation first
    need = psf.noncausal_workspace_bytes(d)
    assert need >= 2 * 1024 * 16 * 4 + 8 * 256 * 65 * 4          # sketches + one state per block, fp32
    assert L.psf_noncausal_attn_fwd(ref, None, one, one, one, one, one, 1 << 40, None) == 1
    assert L.psf_noncausal_attn_fwd(ref, one, one, one, None, one, one, 1 << 40, None) == 1
    assert L.psf_noncausal_attn_fwd(ref, one, one, one, one, None, one, 1 << 40, None) == 1
    assert L.psf_noncausal_attn_fwd(ref, one, one, one, one, one, None, 1 << 40, None) == 1
    assert L.psf_noncausal_attn_fwd(ref, one, one, one, one, one, one, need - 1, None) == 4
    assert L.psf_noncausal_attn_fwd(ref, one, one, one, one, one, ctypes.c_void_p(264), 1 << 40, None) == 4
    assert L.psf_noncausal_attn_fwd_timed(ref, one, one, one, one, one, one, 1 << 40, None, None, 0, None) == 1
    # MFMA path: one snapshot per unit however many blocks the descriptor names
    a = psf.make_desc(2, 12, 32768, 64, 4, 64, 1024, "bf16")
    b = psf.make_desc(2, 12, 32768, 64, 4, 64, 256, "bf16")
    assert psf.noncausal_workspace_bytes(a) == psf.noncausal_workspace_bytes(b) < psf.workspace_bytes(a)
    d.p = 5
    assert L.psf_noncausal_attn_fwd(ref, one, one, one, one, one, one, 1 << 40, None) == 3
    assert psf.noncausal_workspace_bytes(d) == 0


def test_decode_entry_points_validate_on_the_host():
    L = psf.lib()
    d = psf.make_desc(2, 3, 4096, 64, 4, 32, 256, "bf16")
    ref = ctypes.byref(d)
    one = ctypes.c_void_p(256)   # never dereferenced: every call below fails validation first
    need = psf.decode_state_bytes(d)
    # per unit: r (r + 1) / 2 x (dv + 1) fp32 state (the pairs a <= b' of the symmetric r x r
    # feature grid), for bf16 storage its value columns once more in bf16, and the block cache
    # (keys and values in the storage type, sketches in fp32); no n in it
    pairs = 32 * 33 // 2
    per_unit = (pairs * 65 + 256 * 32) * 4 + pairs * 64 * 2 + 256 * (64 + 64) * 2
    assert need >= 6 * per_unit
    assert need < 6 * per_unit + (1 << 16)
    f32 = psf.make_desc(2, 3, 4096, 64, 4, 32, 256, "f32")
    per_unit_f32 = (pairs * 65 + 256 * (32 + 64 + 64)) * 4
    assert 6 * per_unit_f32 <= psf.decode_state_bytes(f32) < 6 * per_unit_f32 + (1 << 16)
    d2 = psf.make_desc(2, 3, 65536, 64, 4, 32, 256, "bf16")
    assert psf.decode_state_bytes(d2) == need
    assert L.psf_decode_reset(ref, None, need, None) == 1
    assert L.psf_decode_reset(ref, one, need - 1, None) == 4
    assert L.psf_decode_reset(ref, ctypes.c_void_p(264), need, None) == 4
    args = [one, one, one, one]
    for hole in (0, 1, 2, 3):
        a = list(args)
        a[hole] = None
        assert L.psf_decode_step(ref, *a, 0, one, need, one, None) == 1, hole
    assert L.psf_decode_step(ref, *args, 0, one, need, None, None) == 1
    assert L.psf_decode_step(ref, *args, 0, None, need, one, None) == 1
    assert L.psf_decode_step(ref, *args, -1, one, need, one, None) == 2
    assert L.psf_decode_step(ref, *args, 4096, one, need, one, None) == 2
    assert L.psf_decode_step(ref, *args, 0, one, need - 1, one, None) == 4
    exact = psf.make_desc(1, 1, 64, 8, 4, 1, 8, "f32", feat=psf.FEAT_EXACT)
    assert psf.decode_state_bytes(exact) == 0
    assert L.psf_decode_step(ctypes.byref(exact), *args, 0, one, 1 << 40, one, None) == 3
    # hand-over from a prompt: no workspace while the prompt is shorter than a block; with complete
    # blocks on the MFMA shapes the forward kernels' buffers (sketches, value octets, one state,
    # the prefix of K and V when a tail follows); the fp32 sketches of every prompt key for
    # learned sketches; every failure below is found before any launch
    assert L.psf_decode_prefill_workspace_bytes(ref, 200) == 0
    units, n_full = 6, 768
    fast = L.psf_decode_prefill_workspace_bytes(ref, 1000)
    assert fast >= units * n_full * (32 * 4 + 64 * 2 + 2 * 64 * 2) + units * 32 * 32 * 64 * 2
    assert fast < units * n_full * (32 * 4 + 64 * 2 + 2 * 64 * 2) + units * 32 * 32 * 64 * 2 + (1 << 20)
    assert L.psf_decode_prefill_workspace_bytes(ref, 768) < fast      # no tail: K and V are used in place
    assert L.psf_decode_prefill(ref, one, one, one, 1000, one, need, None, fast, None) == 1
    assert L.psf_decode_prefill(ref, one, one, one, 1000, one, need, one, fast - 1, None) == 4
    f32d = psf.make_desc(2, 3, 4096, 64, 4, 32, 256, "f32")
    assert L.psf_decode_prefill_workspace_bytes(ctypes.byref(f32d), 1000) == 0    # general kernels only
    assert L.psf_decode_prefill_workspace_bytes(ref, 4097) == 0
    assert L.psf_decode_prefill(ref, one, one, one, -1, one, need, None, 0, None) == 2
    assert L.psf_decode_prefill(ref, one, one, one, 4097, one, need, None, 0, None) == 2
    assert L.psf_decode_prefill(ref, None, one, one, 5, one, need, None, 0, None) == 1
    assert L.psf_decode_prefill(ref, one, None, one, 5, one, need, None, 0, None) == 1
    assert L.psf_decode_prefill(ref, one, one, None, 5, one, need, None, 0, None) == 1
    assert L.psf_decode_prefill(ref, one, one, one, 5, None, need, None, 0, None) == 1
    assert L.psf_decode_prefill(ref, one, one, one, 5, one, need - 1, None, 0, None) == 4
    lrn = psf.make_desc(2, 3, 4096, 64, 4, 32, 256, "f32", learned=True)
    lref, lneed = ctypes.byref(lrn), psf.decode_state_bytes(lrn)
    want_ws = 6 * 1000 * 32 * 4
    # (bf16 on the MFMA shapes: only the 232 rows after the last block boundary are sketched this
    # way, the complete blocks take the forward kernels' buffers)
    lbf = psf.make_desc(2, 3, 4096, 64, 4, 32, 256, "bf16", learned=True)
    assert L.psf_decode_prefill_workspace_bytes(ctypes.byref(lbf), 1000) > fast + 6 * 232 * (32 * 4 + 64 * 2)
    assert L.psf_decode_prefill_workspace_bytes(lref, 1000) == want_ws
    assert L.psf_decode_prefill(lref, one, one, one, 1000, one, lneed, None, want_ws, None) == 1
    assert L.psf_decode_prefill(lref, one, one, one, 1000, one, lneed, one, want_ws - 1, None) == 4
    assert L.psf_decode_prefill(lref, one, one, one, 1000, one, lneed, ctypes.c_void_p(264), want_ws, None) == 4
    assert L.psf_decode_prefill(ctypes.byref(exact), one, one, one, 5, one, 1 << 40, None, 0, None) == 3


def test_misaligned_tensors_are_rejected_on_the_mfma_paths_before_any_launch():
    """The bf16 MFMA kernels move 16-byte pieces: a tensor that is not 16-byte aligned gives
    PSF_ERR_ALIGNMENT (6).  Every call below has exactly one misaligned tensor, so each returns
    from validation; none reaches a launch."""
    L = psf.lib()
    d = psf.make_desc(1, 2, 1024, 64, 4, 64, 256, "bf16")
    assert psf.kernel_path(d) == 1 and psf.bwd_kernel_path(d) == 3
    ref = ctypes.byref(d)
    ok, odd, big = ctypes.c_void_p(256), ctypes.c_void_p(258), 1 << 40
    for hole in range(5):                                                    # Q, K, V, G, O
        a = [ok] * 5
        a[hole] = odd
        assert L.psf_causal_attn_fwd(ref, *a, ok, big, None) == 6, hole
        assert L.psf_noncausal_attn_fwd(ref, *a, ok, big, None) == 6, hole
        assert L.psf_causal_attn_fwd_save(ref, *a, ok, big, None) == 6, hole
    for hole in range(8):                                                    # Q, K, V, G, dO, dQ, dK, dV
        a = [ok] * 8
        a[hole] = odd
        assert L.psf_causal_attn_bwd(ref, *a, ok, big, None) == 6, hole
    for hole in range(3):                                                    # K, V, G of a prompt
        a = [ok] * 3
        a[hole] = odd
        assert L.psf_decode_prefill(ref, *a, 512, ok, big, ok, big, None) == 6, hole
    # the hand-over takes the MFMA kernels for complete blocks whatever b % 256 and the in-block
    # rule are, i.e. also where the forward call itself runs the general kernels
    for dd in (psf.make_desc(1, 2, 1024, 64, 4, 64, 128, "bf16"),
               psf.make_desc(1, 2, 1024, 128, 4, 32, 256, "bf16", local=psf.LOCAL_SKETCH)):
        assert psf.kernel_path(dd) == 0
        for hole in range(3):
            a = [ok] * 3
            a[hole] = odd
            assert L.psf_decode_prefill(ctypes.byref(dd), *a, 512, ok, big, ok, big, None) == 6, hole
    # the general fp32 kernels read element by element: no such requirement (NULL check comes first)
    g = psf.make_desc(1, 1, 64, 16, 4, 8, 16, "f32")
    assert psf.kernel_path(g) == 0
    assert L.psf_causal_attn_fwd(ctypes.byref(g), odd, odd, odd, odd, None, ok, big, None) == 1
    assert psf.status_string(6)


def test_status_strings_and_stage_names():
    assert psf.status_string(0) == "ok"
    assert all(psf.status_string(c) for c in range(7))
    assert psf.lib().psf_stage_name(0, 0) == b"sketch_q"
    assert psf.lib().psf_stage_name(1, 3) == b"output"


def test_binding_refuses_cpu_tensors():
    import torch
    d = psf.make_desc(1, 1, 64, 8, 4, 4, 8, "f32")
    x = torch.zeros(1, 1, 64, 8)
    with pytest.raises(ValueError):
        psf.psf_sketch(d, x, torch.zeros(1, 64), want_m=True)
