"""GPU parity of token-by-token evaluation (psf_decode_step through the C ABI): feeding a
sequence one position at a time must reproduce, row by row, the float64 oracle's rows of the
full causal attention with the same block size (tolerance 1e-4 fp32 / 2e-2 bf16 storage)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2310_01655_amd import binding as psf
from paper_2310_01655_amd import inputs
from parity import as_f64, assert_close

pytestmark = pytest.mark.gpu


def decode_all(batch, heads, n, d, dv, p, r, b, dtype, local=psf.LOCAL_EXACT, per_head=True, seed=51, steps=None):
    q, k, v = inputs.make_qkv(batch, heads, n, d, dv=dv, seed=seed, dtype=dtype)
    G = inputs.make_sketch_matrices(heads, d, r, p, per_head=per_head, seed=0, dtype=dtype) if p > 2 else None
    desc = psf.make_desc(batch, heads, n, d, p, r, b, dtype, dv=dv, local=local, per_head=per_head)
    dev = torch.device("cuda:0")
    qd, kd, vd = q.to(dev), k.to(dev), v.to(dev)
    Gd = G.to(dev) if G is not None else None
    state = psf.decode_new_state(desc, dev)
    steps = n if steps is None else steps
    out = torch.empty(batch, heads, steps, dv, dtype=q.dtype, device=dev)
    for pos in range(steps):
        o = psf.psf_decode_step(desc, qd[:, :, pos:pos + 1].contiguous(), kd[:, :, pos:pos + 1].contiguous(),
                                vd[:, :, pos:pos + 1].contiguous(), Gd, pos, state)
        out[:, :, pos] = o[:, :, 0]
    torch.cuda.synchronize()
    want, _ = oracle.attn_def_batch(as_f64(q), as_f64(k), as_f64(v), as_f64(G) if G is not None else None,
                                    p, r, b, local=oracle.LOCAL_EXACT if local == psf.LOCAL_EXACT else oracle.LOCAL_SKETCH,
                                    rows=list(range(steps)))
    res = assert_close(out.float().cpu().numpy(), want, dtype, "decode n=%d d=%d p=%d r=%d b=%d" % (n, d, p, r, b))
    print((n, d, dv, p, r, b, dtype), res)
    return out


@pytest.mark.parametrize("n,d,dv,p,r,b", [
    (192, 32, 32, 4, 16, 64),      # three blocks: two folds
    (96, 24, 40, 4, 12, 32),       # dv != d, sizes that are no powers of two
    (64, 16, 16, 2, 8, 16),        # p = 2: m(x) = x
    (64, 16, 16, 8, 8, 16),        # one inner level
    (48, 16, 16, 4, 8, 1),         # every token its own block: pure recurrence
    (64, 32, 32, 4, 16, 64),       # single block: only the cache is used
])
def test_decode_fp32_matches_forward_rows(n, d, dv, p, r, b):
    decode_all(1, 2, n, d, dv, p, r, b, "f32")


def test_decode_largest_admitted_dimensions():
    decode_all(1, 1, 32, 256, 256, 4, 256, 16, "f32", per_head=False)


def test_decode_sketched_local_weights():
    decode_all(2, 2, 96, 32, 32, 4, 16, 32, "f32", local=psf.LOCAL_SKETCH)


def test_decode_bf16_storage_headline_shape_per_unit():
    # d = 64, r = 64, b = 256: the per-unit state of the headline configuration, shorter context
    decode_all(1, 3, 768, 64, 64, 4, 64, 256, "bf16")


@pytest.mark.parametrize("n,d,r,b", [(384, 128, 32, 128), (288, 64, 64, 96), (512, 64, 32, 256)])
def test_decode_bf16_block_fold_on_mfma(n, d, r, b):
    # bf16 storage with r, dv multiples of 32: completed blocks are folded into the state by the
    # MFMA kernel (one 32 x 32 tile per wave and more; b = 96 leaves a padded token chunk)
    decode_all(1, 2, n, d, d, 4, r, b, "bf16")


@pytest.mark.parametrize("r,dv", [(64, 32), (64, 96), (64, 128), (32, 32), (32, 96)])
def test_decode_bf16_block_fold_every_tile_shape(r, dv):
    # the MFMA fold is instantiated per (sketch size, value width): one, two, three or four
    # 32-wide value tiles per fragment, one or two 32-wide ranges of sketch columns
    decode_all(1, 2, 192, 64, dv, 4, r, 64, "bf16", steps=150)


@pytest.mark.parametrize("dtype,n,d,r,b", [("bf16", 48, 64, 32, 16), ("f32", 40, 16, 8, 8)])
def test_decode_many_units_one_workgroup_per_unit(dtype, n, d, r, b):
    # 768 units: the state product of a unit is not split into slices, and the same workgroup
    # finishes the row (own pair, division, cache append): two launches per step
    decode_all(64, 12, n, d, d, 4, r, b, dtype, per_head=False)


def test_decode_many_units_large_sketch_keeps_slices_within_lds():
    # 384 units and r = 128 (8256 pairs): more pairs than one workgroup holds in LDS, so the
    # unit count alone must not decide the number of slices
    decode_all(32, 12, 24, 16, 16, 4, 128, 8, "f32", per_head=False)


def prefill_then_decode(batch, heads, n, n_prompt, d, dv, p, r, b, dtype, local=psf.LOCAL_EXACT, learned=False,
                        per_head=True, seed=57):
    """psf_decode_prefill on the first n_prompt tokens, then steps n_prompt .. n - 1: every
    decoded row against the float64 oracle's row of the whole sequence."""
    q, k, v = inputs.make_qkv(batch, heads, n, d, dv=dv, seed=seed, dtype=dtype)
    if learned:
        G = inputs.make_learned_params(heads, d, r, p, per_head=per_head, seed=3, dtype=dtype)
    else:
        G = inputs.make_sketch_matrices(heads, d, r, p, per_head=per_head, seed=0, dtype=dtype) if p > 2 else None
    desc = psf.make_desc(batch, heads, n, d, p, r, b, dtype, dv=dv, local=local, per_head=per_head, learned=learned)
    dev = torch.device("cuda:0")
    qd, kd, vd = q.to(dev), k.to(dev), v.to(dev)
    Gd = G.to(dev) if G is not None else None
    state = psf.decode_new_state(desc, dev)
    state.fill_(0x7f)                                       # prefill must not rely on an earlier reset
    ws = psf.psf_decode_prefill(desc, kd[:, :, :n_prompt].contiguous(), vd[:, :, :n_prompt].contiguous(), Gd, state)
    out = torch.empty(batch, heads, n - n_prompt, dv, dtype=q.dtype, device=dev)
    for pos in range(n_prompt, n):
        o = psf.psf_decode_step(desc, qd[:, :, pos:pos + 1].contiguous(), kd[:, :, pos:pos + 1].contiguous(),
                                vd[:, :, pos:pos + 1].contiguous(), Gd, pos, state)
        out[:, :, pos - n_prompt] = o[:, :, 0]
    torch.cuda.synchronize()
    del ws
    rows = list(range(n_prompt, n))
    want = np.empty((batch, heads, len(rows), dv))
    olocal = oracle.LOCAL_EXACT if local == psf.LOCAL_EXACT else oracle.LOCAL_SKETCH
    for bi in range(batch):
        for h in range(heads):
            Gh = None if G is None else as_f64(G[h if G.shape[0] > 1 else 0])
            want[bi, h] = oracle.attn_def(as_f64(q[bi, h]), as_f64(k[bi, h]), as_f64(v[bi, h]), Gh, p, r, b,
                                          local=olocal, rows=rows, learned=learned)
    res = assert_close(out.float().cpu().numpy(), want, dtype, "prefill %d of %d, b=%d" % (n_prompt, n, b))
    print("prefill", (n, n_prompt, d, dv, p, r, b, dtype, learned), res)


@pytest.mark.parametrize("n,n_prompt,b", [
    (96, 0, 32),        # empty prompt: the same as a reset
    (96, 20, 32),       # inside the first block: cache only
    (96, 64, 32),       # exactly two blocks: two folds, empty cache
    (96, 75, 32),       # two folds and a tail in the cache
    (40, 39, 8),        # almost everything, odd tail
])
def test_decode_prefill_then_steps_fp32(n, n_prompt, b):
    prefill_then_decode(1, 2, n, n_prompt, 24, 40, 4, 12, b, "f32")


@pytest.mark.parametrize("p,local", [(2, psf.LOCAL_EXACT), (8, psf.LOCAL_EXACT), (4, psf.LOCAL_SKETCH)])
def test_decode_prefill_other_degrees_and_in_block_rule(p, local):
    prefill_then_decode(1, 2, 64, 37, 16, 16, p, 8, 16, "f32", local=local)


def test_decode_prefill_bf16_mfma_fold_many_units():
    # 768 units (the step kernel's one-workgroup mode), blocks folded by the MFMA kernel
    prefill_then_decode(64, 12, 64, 50, 64, 64, 4, 32, 16, "bf16", per_head=False)


def test_decode_prefill_headline_unit_shape_bf16():
    prefill_then_decode(1, 3, 768, 600, 64, 64, 4, 64, 256, "bf16")


@pytest.mark.parametrize("heads,n,n_prompt,d,p,r,b,per_head", [
    (2, 768, 512, 64, 4, 32, 256, True),      # complete blocks only: K and V used in place
    (3, 1024, 700, 64, 4, 32, 256, False),    # two blocks through the forward kernels, a tail through the cache
    (2, 768, 600, 128, 8, 64, 256, True),     # d = 128, two-level sketch
    (2, 1024, 1023, 64, 4, 64, 512, False),   # one block, then all but one token of the next
])
def test_decode_prefill_through_the_forward_state_kernel(heads, n, n_prompt, d, p, r, b, per_head):
    # bf16 on the MFMA shapes: the state of the prompt's complete blocks is the forward path's
    # total state (bf16, as the forward pass stores its prefix states), imported into the packed
    # fp32 / bf16 decode state; the rows decoded afterwards against the oracle
    prefill_then_decode(1, heads, n, n_prompt, d, d, p, r, b, "bf16", per_head=per_head)


def test_decode_prefill_learned_sketches():
    prefill_then_decode(1, 2, 48, 29, 16, 16, 4, 8, 16, "f32", learned=True)


@pytest.mark.parametrize("n,n_prompt,r,b,per_head", [(768, 600, 64, 256, True), (768, 512, 32, 256, False)])
def test_decode_prefill_learned_sketches_through_the_forward_kernels(n, n_prompt, r, b, per_head):
    # bf16, d = 64, degree 4: the complete blocks through the MFMA learned-sketch kernel and the
    # state kernel, the tail through the general sketch kernel and the cache
    prefill_then_decode(1, 2, n, n_prompt, 64, 64, 4, r, b, "bf16", learned=True, per_head=per_head)


@pytest.mark.parametrize("batch,heads,n,d,r,b,dtype,local,learned", [
    # the step kernel's variants: storage type x bf16 copy of the state x in-block rule x
    # (slices + finish kernel | one workgroup | one workgroup that also sketches)
    (1, 2, 128, 64, 64, 32, "bf16", psf.LOCAL_SKETCH, False),      # slices, weights from the sketches, bf16 copy
    (64, 12, 48, 64, 32, 16, "bf16", psf.LOCAL_SKETCH, False),     # 768 units: one launch, weights from the sketches
    (1, 2, 128, 64, 64, 32, "f32", psf.LOCAL_SKETCH, False),       # slices, fp32 state only
    (1, 2, 96, 64, 64, 32, "bf16", psf.LOCAL_EXACT, True),         # learned sketches, slices + finish kernel
    (1, 2, 96, 64, 64, 32, "f32", psf.LOCAL_EXACT, True),
    (32, 24, 32, 16, 8, 8, "f32", psf.LOCAL_EXACT, True),          # learned sketches, 768 units: finish inside
    # (fp32 storage: with 4 x 10^5 bf16 outputs of magnitude up to 4 the largest rounding error
    # alone reaches the 2e-2 bound)
])
def test_decode_step_kernel_variants(batch, heads, n, d, r, b, dtype, local, learned):
    prefill_then_decode(batch, heads, n, 0, d, d, 4, r, b, dtype, local=local, learned=learned, per_head=False)


def test_decode_equals_the_forward_entry_point():
    batch, heads, n, d, p, r, b = 1, 2, 128, 32, 4, 16, 32
    out = decode_all(batch, heads, n, d, d, p, r, b, "f32", seed=53)
    q, k, v = inputs.make_qkv(batch, heads, n, d, seed=53, dtype="f32")
    G = inputs.make_sketch_matrices(heads, d, r, p, per_head=True, seed=0, dtype="f32")
    desc = psf.make_desc(batch, heads, n, d, p, r, b, "f32", per_head=True)
    O = psf.psf_causal_attn_fwd(desc, q.cuda(), k.cuda(), v.cuda(), G.cuda())
    torch.cuda.synchronize()
    assert (out - O).abs().max().item() <= 2e-5


def test_decode_rejects_bad_positions_and_exact_features():
    desc = psf.make_desc(1, 1, 64, 8, 4, 4, 16, "f32")
    state = psf.decode_new_state(desc)
    x = torch.zeros(1, 1, 1, 8, device="cuda")
    G = torch.zeros(1, psf.g_len(8, 4, 4), device="cuda")
    for pos in (-1, 64):
        with pytest.raises(psf.PsfError) as e:
            psf.psf_decode_step(desc, x, x, x, G, pos, state)
        assert e.value.code == 2
    exact = psf.make_desc(1, 1, 64, 4, 4, 4, 16, "f32", feat=psf.FEAT_EXACT)
    assert psf.decode_state_bytes(exact) == 0
