"""GPU parity of psf_causal_attn_bwd (through the C ABI) against the float64 gradient oracle.
Same seeded inputs on both sides; the oracle consumes the storage-rounded values upcast to
float64.  Tolerance: 1e-4 (fp32 storage) / 2e-2 (bf16 storage) on relative Frobenius error and on
max-abs error relative to the largest entry (gradients have no fixed scale), for each of dQ,
dK, dV."""
import numpy as np
import pytest
import torch

import oracle
from paper_2310_01655_amd import binding as psf
from paper_2310_01655_amd import inputs
from parity import as_f64, assert_close, assert_close_scaled

pytestmark = pytest.mark.gpu


def run_case(batch, heads, n, d, dv, p, r, b, dtype, local=psf.LOCAL_EXACT, per_head=False, seed=41,
             dist="normal"):
    q, k, v = inputs.make_qkv(batch, heads, n, d, dv=dv, seed=seed, dist=dist, dtype=dtype)
    dO = inputs.make_dout(batch, heads, n, dv, seed=seed, dtype=dtype)
    G = inputs.make_sketch_matrices(heads, d, r, p, per_head=per_head, seed=0, dtype=dtype) if p > 2 else None
    desc = psf.make_desc(batch, heads, n, d, p, r, b, dtype, dv=dv, local=local, per_head=per_head)
    dev = torch.device("cuda:0")
    args = [x.to(dev) if x is not None else None for x in (q, k, v, G, dO)]
    dQ, dK, dV = psf.psf_causal_attn_bwd(desc, *args)
    torch.cuda.synchronize()
    wQ, wK, wV, _ = oracle.attn_bwd_batch(as_f64(q), as_f64(k), as_f64(v),
                                          as_f64(G) if G is not None else None, as_f64(dO), p, r, b,
                                          local=oracle.LOCAL_EXACT if local == psf.LOCAL_EXACT else oracle.LOCAL_SKETCH)
    res = {}
    for name, got, want in (("dQ", dQ, wQ), ("dK", dK, wK), ("dV", dV, wV)):
        res[name] = assert_close_scaled(got.float().cpu().numpy(), want, dtype, "%s n=%d d=%d p=%d r=%d b=%d" % (name, n, d, p, r, b))
    print((n, d, dv, p, r, b, dtype), {k2: ("%.2e" % v2[0], "%.2e" % v2[1]) for k2, v2 in res.items()})
    return dQ, dK, dV


@pytest.mark.parametrize("n,d,dv,p,r,b", [
    (256, 64, 64, 4, 16, 64),      # config-1 shape, shorter
    (128, 32, 48, 4, 16, 32),      # dv != d
    (128, 24, 24, 2, 16, 32),      # base case p = 2: m(x) = x
    (128, 32, 32, 8, 16, 32),      # one inner level
    (96, 16, 16, 16, 8, 32),       # two inner levels
    (128, 32, 32, 4, 16, 128),     # single block
    (64, 16, 16, 4, 8, 1),         # every token its own block
    (192, 40, 24, 4, 20, 64),      # sizes that are no powers of two
])
def test_backward_fp32_small_full_parity(n, d, dv, p, r, b):
    run_case(2, 2, n, d, dv, p, r, b, "f32", per_head=True)


@pytest.mark.parametrize("p", [4, 8])
def test_backward_fp32_sketched_local_weights(p):
    run_case(1, 3, 128, 32, 32, p, 16, 32, "f32", local=psf.LOCAL_SKETCH, per_head=True)


def test_backward_config1_full_size():
    run_case(1, 1, 1024, 64, 64, 4, 16, 128, "f32", seed=1001)


@pytest.mark.parametrize("n,d,p,r,b", [(256, 64, 4, 32, 64), (256, 64, 4, 64, 128), (128, 128, 8, 64, 64)])
def test_backward_bf16_storage(n, d, p, r, b):
    run_case(1, 2, n, d, d, p, r, b, "bf16", per_head=True)


def test_backward_largest_admitted_dimensions():
    # d = dv = r = 256 (r^2 = 65536 features): the run-time LDS carving beyond 64 KB per workgroup
    run_case(1, 1, 32, 256, 256, 4, 256, 16, "f32")
    run_case(1, 1, 64, 256, 256, 4, 64, 32, "f32", local=psf.LOCAL_SKETCH)


def test_backward_heavy_tailed_inputs():
    run_case(1, 2, 256, 64, 64, 4, 32, 64, "f32", dist="student_t3")


def test_backward_is_deterministic():
    a = run_case(1, 2, 256, 64, 64, 4, 32, 64, "f32")
    b2 = run_case(1, 2, 256, 64, 64, 4, 32, 64, "f32")
    for x, y in zip(a, b2):
        assert torch.equal(x, y)


def test_backward_exact_features_are_refused():
    desc = psf.make_desc(1, 1, 64, 4, 4, 4, 16, "f32", feat=psf.FEAT_EXACT)
    assert psf.bwd_workspace_bytes(desc) == 0
    x = torch.zeros(1, 1, 64, 4, device="cuda")
    with pytest.raises(psf.PsfError) as e:
        psf.psf_causal_attn_bwd(desc, x, x, x, None, x)
    assert e.value.code == 3


@pytest.mark.parametrize("heads,n,r,b,per_head", [
    (2, 1024, 64, 256, True),      # four blocks: cross-block terms on both sides
    (2, 1024, 32, 256, True),
    (1, 512, 64, 512, False),      # single block: in-block pairs only
    (3, 2048, 64, 512, False),     # several 256-token workgroups per block
    (2, 1536, 32, 768, True),      # block size that is no power of two
])
def test_backward_mfma_path_full_parity(heads, n, r, b, per_head):
    desc = psf.make_desc(1, heads, n, 64, 4, r, b, "bf16", per_head=per_head)
    assert psf.bwd_kernel_path(desc) == 3
    run_case(1, heads, n, 64, 64, 4, r, b, "bf16", per_head=per_head, seed=43)


@pytest.mark.parametrize("heads,n,d,p,r,b,per_head", [
    (2, 1024, 128, 8, 64, 256, True),    # config 5's head width and degree: four blocks
    (2, 1024, 128, 8, 32, 512, False),
    (1, 512, 128, 8, 64, 512, True),     # single block: in-block pairs only, s^7 slopes
    (2, 1024, 64, 8, 64, 256, True),     # degree 8 at d = 64
    (2, 768, 128, 4, 64, 256, False),    # d = 128 with degree 4
    (3, 1536, 128, 8, 64, 768, True),    # block size that is no power of two
])
def test_backward_mfma_path_wide_heads_and_degree_eight(heads, n, d, p, r, b, per_head):
    desc = psf.make_desc(1, heads, n, d, p, r, b, "bf16", per_head=per_head)
    assert psf.bwd_kernel_path(desc) == 3
    run_case(1, heads, n, d, d, p, r, b, "bf16", per_head=per_head, seed=49)


@pytest.mark.parametrize("heads,n,b,per_head", [(2, 1024, 256, True), (3, 1536, 512, False), (1, 512, 512, False)])
def test_backward_mfma_path_in_block_weights_from_the_sketches(heads, n, b, per_head):
    # Section 3.1's in-block rule on the MFMA kernels (r = d = 64): the in-block kernels work on
    # m(Q), m(K) and their result joins dm before the sketch gradient; r = 32 stays on the
    # general kernels
    desc = psf.make_desc(1, heads, n, 64, 4, 64, b, "bf16", per_head=per_head, local=psf.LOCAL_SKETCH)
    assert psf.bwd_kernel_path(desc) == 3
    assert psf.bwd_kernel_path(psf.make_desc(1, heads, n, 64, 4, 32, b, "bf16", local=psf.LOCAL_SKETCH)) == 2
    run_case(1, heads, n, 64, 64, 4, 64, b, "bf16", local=psf.LOCAL_SKETCH, per_head=per_head, seed=45)


def test_backward_mfma_path_is_deterministic_and_matches_general_kernels():
    """The MFMA kernels against the general fp32 kernels of the same library on a shape both
    accept (b % 256 != 0 sends the same problem down the general path)."""
    a = run_case(1, 2, 1024, 64, 64, 4, 64, 256, "bf16", per_head=True, seed=47)
    a2 = run_case(1, 2, 1024, 64, 64, 4, 64, 256, "bf16", per_head=True, seed=47)
    for x, y in zip(a, a2):
        assert torch.equal(x, y)


@pytest.mark.parametrize("idx,units", [(3, [(0, 0), (1, 7)]), (5, [(0, 0), (0, 9)])])
def test_backward_config3_full_size_sampled_rows_and_identities(idx, units):
    """The workloads `bench.py --pass bwd` times (config 3: 2 x 12 units of 32768 tokens; config 5:
    16 units of 16384 tokens with d = 128 and degree 8; MFMA kernels).  Element-wise against the oracle where it can afford the sums: dQ on probe rows
    spread over the sequence, dK and dV on the last block plus the end of the block before it
    (those rows see in-block pairs and one later block's cross-block pairs), for two units.
    Over all tokens of every unit, two identities that hold at any size: the weights are
    homogeneous of degree p in q_i and in k_j, so sum_i <q_i, dQ_i> = sum_j <k_j, dK_j>
    (= p sum w dw, Euler); the output is linear in V, so <dV, V> = <dO, O>."""
    from concurrent.futures import ThreadPoolExecutor
    from parity import probe_rows
    cfg, q, k, v, G = inputs.make_config(idx)
    n, b, r, p, heads = cfg["n"], cfg["b"], cfg["r"], cfg["p"], cfg["heads"]
    dO = inputs.make_dout(cfg["batch"], heads, n, cfg["d"], seed=1000 + idx, dtype="bf16")
    desc = psf.make_desc(cfg["batch"], heads, n, cfg["d"], p, r, b, "bf16", per_head=cfg["per_head"])
    assert psf.bwd_kernel_path(desc) == 3
    dev = torch.device("cuda:0")
    qd, kd, vd, Gd, dOd = (x.to(dev) for x in (q, k, v, G, dO))
    dQ, dK, dV = psf.psf_causal_attn_bwd(desc, qd, kd, vd, Gd, dOd)
    O = psf.psf_causal_attn_fwd(desc, qd, kd, vd, Gd)
    torch.cuda.synchronize()
    f = lambda t: t.float()
    # identities, per unit
    a = (f(qd) * f(dQ)).sum((-1, -2))
    c = (f(kd) * f(dK)).sum((-1, -2))
    scale = ((f(qd) * f(dQ)).sum(-1).abs().sum(-1) + (f(kd) * f(dK)).sum(-1).abs().sum(-1)) / 2
    assert ((a - c).abs() <= 2e-2 * scale).all(), ((a - c).abs() / scale).max()
    lv, lo = (f(dV) * f(vd)).sum((-1, -2)), (f(dOd) * f(O)).sum((-1, -2))
    scale_v = (f(dOd) * f(O)).sum(-1).abs().sum(-1)
    assert ((lv - lo).abs() <= 2e-2 * scale_v).all(), ((lv - lo).abs() / scale_v).max()
    # sampled rows against the oracle
    tail0 = n - b - 128
    probe = [x for x in probe_rows(n, b, extra=12) if x < tail0]
    rows = probe + list(range(tail0, n))

    def one(unit):
        bi, h = unit
        g = as_f64(G[h]) if G.shape[0] > 1 else as_f64(G[0])
        return oracle.attn_bwd_rows(as_f64(q[bi, h]), as_f64(k[bi, h]), as_f64(v[bi, h]), g, as_f64(dO[bi, h]),
                                    p, r, b, rows)

    with ThreadPoolExecutor(2) as ex:
        want = list(ex.map(one, units))
    for (bi, h), (wQ, wK, wV) in zip(units, want):
        gq, gk, gv = (x[bi, h].float().cpu().numpy() for x in (dQ, dK, dV))
        print("config %d bwd" % idx, (bi, h),
              assert_close_scaled(gq[rows], wQ[rows], "bf16", "dQ"),
              assert_close_scaled(gk[tail0:], wK[tail0:], "bf16", "dK"),
              assert_close_scaled(gv[tail0:], wV[tail0:], "bf16", "dV"))


@pytest.mark.parametrize("d,p,r,b,local", [(64, 4, 64, 256, psf.LOCAL_EXACT), (64, 4, 32, 512, psf.LOCAL_EXACT),
                                           (64, 4, 64, 256, psf.LOCAL_SKETCH), (128, 8, 64, 512, psf.LOCAL_EXACT)])
def test_saved_forward_gives_the_same_output_and_gradients(d, p, r, b, local):
    """psf_causal_attn_fwd_save + psf_causal_attn_bwd_saved against the plain forward and the
    plain (recomputing) backward of the same library.  The gradients are identical bits: the
    recomputing backward runs the very forward kernels the saving call runs, on the same data.
    The plain forward call may take other kernels for the prefix states (half-precision products
    where the in-block part runs beside them), so its output agrees within the rounding of the
    storage type, not bit for bit; the plain calls are the ones checked against the oracle above."""
    batch, heads, n = 1, 3, 1024
    q, k, v = inputs.make_qkv(batch, heads, n, d, seed=53, dtype="bf16")
    dO = inputs.make_dout(batch, heads, n, d, seed=53, dtype="bf16")
    G = inputs.make_sketch_matrices(heads, d, r, p, per_head=True, seed=0, dtype="bf16")
    desc = psf.make_desc(batch, heads, n, d, p, r, b, "bf16", per_head=True, local=local)
    assert psf.bwd_kernel_path(desc) == 3 and psf.fwd_save_bytes(desc) > psf.workspace_bytes(desc)
    dev = torch.device("cuda:0")
    qd, kd, vd, Gd, dOd = (x.to(dev) for x in (q, k, v, G, dO))
    O1 = psf.psf_causal_attn_fwd(desc, qd, kd, vd, Gd)
    O2, save = psf.psf_causal_attn_fwd_save(desc, qd, kd, vd, Gd)
    g1 = psf.psf_causal_attn_bwd(desc, qd, kd, vd, Gd, dOd)
    g2 = psf.psf_causal_attn_bwd_saved(desc, qd, kd, vd, Gd, O2, dOd, save)
    torch.cuda.synchronize()
    assert_close(O2.float().cpu().numpy(), O1.float().cpu().numpy(), "bf16", "saving forward against plain forward")
    for a, c in zip(g1, g2):
        assert torch.equal(a, c)


def test_saved_forward_is_refused_where_the_general_kernels_run():
    desc = psf.make_desc(1, 1, 256, 64, 4, 16, 64, "f32")
    assert psf.bwd_kernel_path(desc) == 2 and psf.fwd_save_bytes(desc) == 0
    q, k, v = inputs.make_qkv(1, 1, 256, 64, seed=1, dtype="f32")
    G = inputs.make_sketch_matrices(1, 64, 16, 4, seed=0, dtype="f32")
    with pytest.raises(psf.PsfError):
        psf.psf_causal_attn_fwd_save(desc, q.cuda(), k.cuda(), v.cuda(), G.cuda())


@pytest.mark.parametrize("dtype,d,r,b,n", [("f32", 16, 8, 16, 64), ("bf16", 64, 64, 256, 512)])
def test_autograd_function_matches_the_oracle_gradient(dtype, d, r, b, n):
    # torch.autograd glue over the two entry points (general fp32 path; MFMA path with the saved
    # forward state): loss = <O, W> with a fixed W, gradients against the float64 oracle
    from paper_2310_01655_amd.autograd import causal_polysketch_attention
    batch, heads, p = 1, 2, 4
    q, k, v = inputs.make_qkv(batch, heads, n, d, seed=61, dtype=dtype)
    G = inputs.make_sketch_matrices(heads, d, r, p, per_head=True, seed=0, dtype=dtype)
    W = inputs.make_dout(batch, heads, n, d, seed=62, dtype=dtype)
    qd, kd, vd = (t.cuda().requires_grad_(True) for t in (q, k, v))
    O = causal_polysketch_attention(qd, kd, vd, G.cuda(), p, r, b, per_head=True)
    (O.float() * W.cuda().float()).sum().backward()
    torch.cuda.synchronize()
    for h in range(heads):
        dq, dk, dvv = oracle.attn_bwd(as_f64(q[0, h]), as_f64(k[0, h]), as_f64(v[0, h]), as_f64(G[h]),
                                      as_f64(W[0, h]), p, r, b)
        for name, got, want in (("dQ", qd.grad, dq), ("dK", kd.grad, dk), ("dV", vd.grad, dvv)):
            assert_close_scaled(got[0, h].float().cpu().numpy(), want, dtype, "autograd %s head %d" % (name, h))
