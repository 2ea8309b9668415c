"""GPU parity of the backward pass through learned sketches (Algorithm 2, Appendix D) against the
float64 gradient oracle, through the C ABI: gradients with respect to Q, K, V and to the
networks' parameters (psf_causal_attn_bwd_learned), and the row gradients alone
(psf_causal_attn_bwd with desc.learned).  The oracle takes the storage-rounded inputs and
parameters upcast to float64 and works one unit at a time; the parameter gradient of a set is the
sum over the units that share it.  Tolerances as for the other gradients: relative Frobenius
error and max-abs error relative to the largest entry, 1e-4 (fp32 storage) / 2e-2 (bf16)."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

import oracle
from paper_2310_01655_amd import binding as psf
from paper_2310_01655_amd import inputs
from parity import as_f64, assert_close_scaled

pytestmark = pytest.mark.gpu


def oracle_grads(q, k, v, P, dO, p, r, b, local):
    B, H = q.shape[:2]
    units = [(bi, h) for bi in range(B) for h in range(H)]

    def one(u):
        bi, h = u
        return oracle.attn_bwd_learned(as_f64(q[bi, h]), as_f64(k[bi, h]), as_f64(v[bi, h]),
                                       as_f64(P[h if P.shape[0] > 1 else 0]), as_f64(dO[bi, h]), p, r, b, local=local)

    with ThreadPoolExecutor(min(len(units), 8)) as ex:
        parts = list(ex.map(one, units))
    wQ, wK, wV = (np.empty(tuple(t.shape)) for t in (q, k, v))
    wP = np.zeros(tuple(P.shape))
    for (bi, h), (dq, dk, dv, dp) in zip(units, parts):
        wQ[bi, h], wK[bi, h], wV[bi, h] = dq, dk, dv
        wP[h if P.shape[0] > 1 else 0] += dp
    return wQ, wK, wV, wP


def run_case(batch, heads, n, d, dv, p, r, b, dtype, local=psf.LOCAL_EXACT, per_head=True, seed=71, path=2):
    q, k, v = inputs.make_qkv(batch, heads, n, d, dv=dv, seed=seed, dtype=dtype)
    dO = inputs.make_dout(batch, heads, n, dv, seed=seed, dtype=dtype)
    P = inputs.make_learned_params(heads, d, r, p, per_head=per_head, seed=3, dtype=dtype)
    desc = psf.make_desc(batch, heads, n, d, p, r, b, dtype, dv=dv, local=local, per_head=per_head, learned=True)
    assert psf.bwd_kernel_path(desc) == path
    dev = torch.device("cuda:0")
    args = [x.to(dev) for x in (q, k, v, P, dO)]
    dQ, dK, dV, dG = psf.psf_causal_attn_bwd_learned(desc, *args)
    torch.cuda.synchronize()
    assert dG.dtype == torch.float32 and tuple(dG.shape) == tuple(P.shape)
    wQ, wK, wV, wP = oracle_grads(q, k, v, P, dO, p, r, b,
                                  oracle.LOCAL_EXACT if local == psf.LOCAL_EXACT else oracle.LOCAL_SKETCH)
    what = "n=%d d=%d p=%d r=%d b=%d %s" % (n, d, p, r, b, dtype)
    res = {}
    for name, got, want in (("dQ", dQ, wQ), ("dK", dK, wK), ("dV", dV, wV)):
        res[name] = assert_close_scaled(got.float().cpu().numpy(), want, dtype, name + " " + what)
    # the parameter gradient is accumulated and returned in fp32 whatever the storage type: on the
    # general path what separates it from the oracle is the fp32 arithmetic of the row kernels; the
    # MFMA kernels (path 3) form it from bf16 operands like every other product of that path
    for s in range(P.shape[0]):
        res["dG%d" % s] = assert_close_scaled(dG[s].cpu().numpy(), wP[s], "f32" if path == 2 else "bf16",
                                              "dG set %d %s" % (s, what))
    print(what, {k2: ("%.2e" % v2[0], "%.2e" % v2[1]) for k2, v2 in res.items()})
    return desc, args, (dQ, dK, dV, dG)


@pytest.mark.parametrize("n,d,dv,p,r,b,per_head", [
    (96, 24, 16, 4, 8, 32, True),      # three blocks, dv != d, a set per head
    (96, 24, 24, 4, 8, 32, False),     # one shared set: its gradient sums over all units
    (64, 16, 16, 8, 8, 16, True),      # degree 8: six networks, two of them on sketches
    (64, 20, 12, 4, 12, 64, True),     # single block, sizes that are no powers of two
])
def test_learned_backward_fp32(n, d, dv, p, r, b, per_head):
    run_case(2, 2, n, d, dv, p, r, b, "f32", per_head=per_head)


@pytest.mark.parametrize("p", [4, 8])
def test_learned_backward_in_block_weights_from_the_sketches(p):
    run_case(1, 2, 64, 16, 16, p, 8, 16, "f32", local=psf.LOCAL_SKETCH)


def test_learned_backward_bf16_storage():
    run_case(1, 2, 128, 32, 32, 4, 16, 32, "bf16")


def test_learned_backward_widest_networks():
    # d = r = 256: 2048 hidden units, the largest the row kernel's workgroup memory is sized for
    run_case(1, 1, 32, 256, 64, 4, 256, 16, "f32")


def test_learned_backward_several_chunks_of_rows():
    # 6144 rows share one parameter set: the staging holds 4096 rows, so the sums over rows run
    # in two chunks that do not end on unit boundaries
    run_case(2, 3, 1024, 16, 16, 4, 8, 256, "f32", per_head=False)


@pytest.mark.parametrize("batch,heads,n,r,b,per_head", [
    (1, 2, 512, 32, 256, True),        # two blocks, a set per head, 16 hidden chunks of 32 per network
    (2, 2, 512, 64, 256, False),       # one shared set: sums over four units; r = d = 64
    (1, 1, 256, 64, 256, True),        # a single block: no cross-block term at all
    (1, 3, 768, 32, 256, True),        # three blocks, a unit count the XCD-aware order does not apply to
])
def test_learned_backward_mfma(batch, heads, n, r, b, per_head):
    run_case(batch, heads, n, 64, 64, 4, r, b, "bf16", per_head=per_head, path=3)


def test_learned_backward_mfma_several_slices_per_unit():
    # 2048 rows per unit: the parameter kernel works on four slices of 512 rows per unit, every
    # one with its own part of the sums (all rows carry a gradient here)
    run_case(1, 2, 2048, 64, 64, 4, 64, 512, "bf16", per_head=True, path=3)


def test_learned_backward_mfma_eight_units():
    # eight units: the parameter kernel's XCD-aware workgroup order
    run_case(4, 2, 256, 64, 64, 4, 32, 256, "bf16", per_head=True, path=3)


def test_learned_backward_mfma_from_the_saved_forward():
    """psf_causal_attn_fwd_save + psf_causal_attn_bwd_saved_learned: the same bits as the recomputing
    call (the saving forward runs the launches the recomputation runs); psf_causal_attn_bwd_saved
    treats the parameters as constants."""
    desc, args, (dQ, dK, dV, dG) = run_case(2, 2, 512, 64, 64, 4, 32, 256, "bf16", path=3)
    q, k, v, P, dO = args
    assert psf.fwd_save_bytes(desc) > 0
    O, save = psf.psf_causal_attn_fwd_save(desc, q, k, v, P)
    got = psf.psf_causal_attn_bwd_saved_learned(desc, q, k, v, P, O, dO, save)
    rows = psf.psf_causal_attn_bwd_saved(desc, q, k, v, P, O, dO, save)
    O_plain = psf.psf_causal_attn_fwd(desc, q, k, v, P)
    torch.cuda.synchronize()
    for a, c in zip(got, (dQ, dK, dV, dG)):
        assert torch.equal(a, c)
    for a, c in zip(rows, (dQ, dK, dV)):
        assert torch.equal(a, c)
    from parity import assert_close
    assert_close(O.float().cpu().numpy(), O_plain.float().cpu().numpy(), "bf16", "saving forward against plain forward")


def test_learned_backward_mfma_rows_only_and_repeat():
    desc, args, (dQ, dK, dV, dG) = run_case(1, 2, 512, 64, 64, 4, 64, 256, "bf16", path=3)
    rQ, rK, rV = psf.psf_causal_attn_bwd(desc, *args)
    again = psf.psf_causal_attn_bwd_learned(desc, *args)
    torch.cuda.synchronize()
    for a, c in ((rQ, dQ), (rK, dK), (rV, dV)):
        assert torch.equal(a, c)
    for a, c in zip(again, (dQ, dK, dV, dG)):
        assert torch.equal(a, c)               # fixed summation order: no atomics


def test_learned_backward_mfma_config3_size_against_the_oracle_on_a_prefix():
    """The launch configuration `bench.py --pass bwd --learned` times (config 3's shapes: 2 x 12
    units of 32768 tokens, a parameter set per head).  dL/dO is zero from row T = 2048 on, so by
    causality the gradient is that of the T-token prefix problem: rows below T of dQ, dK, dV and
    the parameter gradient equal the oracle's on the prefix (two parameter sets = four units are
    checked), every row from T on is exactly zero.  A second call with 2 dL/dO returns twice the
    first (every step of the reverse pass is linear in dL/dO), and <dV, V> = <dO, O> per unit
    (the output is linear in V)."""
    cfg, q, k, v, _ = inputs.make_config(3)
    B, H, n, d, r, b = cfg["batch"], cfg["heads"], cfg["n"], cfg["d"], cfg["r"], cfg["b"]
    T = 2 * b
    P = inputs.make_learned_params(H, d, r, 4, per_head=True, seed=3, dtype="bf16")
    dO = inputs.make_dout(B, H, n, d, seed=1003, dtype="bf16")
    dO[:, :, T:] = 0
    desc = psf.make_desc(B, H, n, d, 4, r, b, "bf16", per_head=True, learned=True)
    assert psf.bwd_kernel_path(desc) == 3
    dev = torch.device("cuda:0")
    qd, kd, vd, Pd, dOd = (x.to(dev) for x in (q, k, v, P, dO))
    ws = psf.alloc_bwd_workspace(desc, dev)
    dQ, dK, dV, dG = psf.psf_causal_attn_bwd_learned(desc, qd, kd, vd, Pd, dOd, workspace=ws)
    dQ2, dK2, dV2, dG2 = psf.psf_causal_attn_bwd_learned(desc, qd, kd, vd, Pd, 2 * dOd, workspace=ws)
    O = psf.psf_causal_attn_fwd(desc, qd, kd, vd, Pd)
    torch.cuda.synchronize()
    for a in (dQ, dK, dV):
        assert torch.isfinite(a.float()).all()
        assert not a[:, :, T:].any()
    for a, c in ((dQ, dQ2), (dK, dK2), (dV, dV2), (dG, dG2)):
        assert torch.allclose(2 * a.float(), c.float(), rtol=1e-5, atol=0)
    f = lambda t: t.float()
    lv, lo = (f(dV) * f(vd)).sum((-1, -2)), (f(dOd) * f(O)).sum((-1, -2))
    scale_v = (f(dOd) * f(O)).sum(-1).abs().sum(-1)
    assert ((lv - lo).abs() <= 2e-2 * scale_v).all(), ((lv - lo).abs() / scale_v).max()
    sets = [0, 7]
    units = [(bi, h) for h in sets for bi in range(B)]

    def one(u):
        bi, h = u
        return oracle.attn_bwd_learned(as_f64(q[bi, h, :T]), as_f64(k[bi, h, :T]), as_f64(v[bi, h, :T]), as_f64(P[h]),
                                       as_f64(dO[bi, h, :T]), 4, r, b, local=oracle.LOCAL_EXACT)

    with ThreadPoolExecutor(len(units)) as ex:
        parts = list(ex.map(one, units))
    wP = {h: 0.0 for h in sets}
    for (bi, h), (wq, wk, wv, wp) in zip(units, parts):
        wP[h] = wP[h] + wp
        print("config 3 learned bwd", (bi, h),
              assert_close_scaled(dQ[bi, h, :T].float().cpu().numpy(), wq, "bf16", "dQ"),
              assert_close_scaled(dK[bi, h, :T].float().cpu().numpy(), wk, "bf16", "dK"),
              assert_close_scaled(dV[bi, h, :T].float().cpu().numpy(), wv, "bf16", "dV"))
    for h in sets:
        print("set", h, assert_close_scaled(dG[h].cpu().numpy(), wP[h], "bf16", "dG set %d" % h))


def test_rows_only_call_gives_the_same_row_gradients_and_repeats_bit_for_bit():
    desc, args, (dQ, dK, dV, dG) = run_case(1, 2, 64, 16, 16, 4, 8, 16, "f32")
    rQ, rK, rV = psf.psf_causal_attn_bwd(desc, *args)
    again = psf.psf_causal_attn_bwd_learned(desc, *args)
    torch.cuda.synchronize()
    for a, c in ((rQ, dQ), (rK, dK), (rV, dV)):
        assert torch.equal(a, c)
    for a, c in zip(again, (dQ, dK, dV, dG)):
        assert torch.equal(a, c)               # fixed summation order: no atomics


@pytest.mark.parametrize("dtype,d,r,b,n", [("f32", 16, 8, 16, 64), ("bf16", 64, 32, 256, 512)])
def test_autograd_function_trains_the_learned_sketches(dtype, d, r, b, n):
    # torch.autograd glue (marshalling only): with parameters that require a gradient the
    # backward is psf_causal_attn_bwd_learned (general kernels / MFMA kernels), bit for bit
    from paper_2310_01655_amd.autograd import causal_polysketch_attention
    batch, heads, p = 1, 2, 4
    q, k, v = inputs.make_qkv(batch, heads, n, d, seed=61, dtype=dtype)
    P = inputs.make_learned_params(heads, d, r, p, per_head=True, seed=3, dtype=dtype)
    W = inputs.make_dout(batch, heads, n, d, seed=62, dtype=dtype)
    qd, kd, vd, Pd = (t.cuda().requires_grad_(True) for t in (q, k, v, P))
    O = causal_polysketch_attention(qd, kd, vd, Pd, p, r, b, per_head=True, learned=True)
    (O.float() * W.cuda().float()).sum().backward()
    desc = psf.make_desc(batch, heads, n, d, p, r, b, dtype, per_head=True, learned=True)
    dQ, dK, dV, dG = psf.psf_causal_attn_bwd_learned(desc, qd.detach(), kd.detach(), vd.detach(), Pd.detach(),
                                                     W.cuda())
    torch.cuda.synchronize()
    for got, want in ((qd.grad, dQ), (kd.grad, dK), (vd.grad, dV), (Pd.grad, dG.to(Pd.dtype))):
        assert torch.equal(got, want)
    # constants: no parameter gradient is asked for, the rows-only call runs
    q2, k2, v2 = (t.cuda().requires_grad_(True) for t in (q, k, v))
    O2 = causal_polysketch_attention(q2, k2, v2, P.cuda(), p, r, b, per_head=True, learned=True)
    (O2.float() * W.cuda().float()).sum().backward()
    torch.cuda.synchronize()
    assert torch.equal(q2.grad, dQ) and torch.equal(k2.grad, dK) and torch.equal(v2.grad, dV)


def test_parameter_gradient_is_refused_for_gaussian_sketches():
    desc = psf.make_desc(1, 1, 64, 16, 4, 8, 16, "f32")
    q, k, v = inputs.make_qkv(1, 1, 64, 16, seed=1, dtype="f32")
    dO = inputs.make_dout(1, 1, 64, 16, seed=1, dtype="f32")
    G = inputs.make_sketch_matrices(1, 16, 8, 4, per_head=False, seed=0, dtype="f32")
    with pytest.raises(psf.PsfError):
        psf.psf_causal_attn_bwd_learned(desc, *[x.cuda() for x in (q, k, v, G, dO)])
