"""GPU parity of the bf16 MFMA path against the float64 oracle (through the C ABI).
The oracle consumes the same bf16-rounded inputs upcast to float64; tolerance 2e-2 on both
max-abs and relative Frobenius error."""
import numpy as np
import pytest
import torch

import oracle
from paper_2310_01655_amd import binding as psf
from paper_2310_01655_amd import inputs
from parity import as_f64, assert_close, assert_close_scaled, errors, gpu_attn, oracle_attn, oracle_units_rows, probe_rows

pytestmark = pytest.mark.gpu


def mk(batch, heads, n, d, p, r, b, per_head=False, dist="normal"):
    return dict(batch=batch, heads=heads, n=n, d=d, p=p, r=r, b=b, dtype="bf16", per_head=per_head,
                dist=dist)


def draw(cfg, seed=17):
    q, k, v = inputs.make_qkv(cfg["batch"], cfg["heads"], cfg["n"], cfg["d"], seed=seed,
                              dist=cfg["dist"], dtype="bf16")
    G = inputs.make_sketch_matrices(cfg["heads"], cfg["d"], cfg["r"], cfg["p"],
                                    per_head=cfg["per_head"], seed=0, dtype="bf16")
    return q, k, v, G


@pytest.mark.parametrize("d,p,r,b", [(64, 4, 64, 256), (64, 4, 32, 256), (64, 4, 64, 512),
                                     (128, 8, 64, 256), (128, 4, 32, 256), (64, 8, 32, 512)])
def test_small_full_parity(d, p, r, b):
    cfg = mk(1, 2, 1024, d, p, r, b, per_head=True)
    q, k, v, G = draw(cfg)
    got, desc = gpu_attn(cfg, q, k, v, G)
    assert psf.kernel_path(desc) == 1
    want = oracle_attn(cfg, q, k, v, G)
    print("small", (d, p, r, b), assert_close(got.numpy(), want, "bf16", "d=%d p=%d r=%d b=%d" % (d, p, r, b)))


@pytest.mark.parametrize("d,p,r", [(64, 4, 64), (64, 4, 32), (128, 8, 64), (64, 8, 64)])
def test_sketch_entry_point(d, p, r):
    cfg = mk(2, 3, 512, d, p, r, 256, per_head=True)
    q, _, _, G = draw(cfg)
    desc = psf.make_desc(2, 3, 512, d, p, r, 256, "bf16", per_head=True)
    M, _ = psf.psf_sketch(desc, q.cuda(), G.cuda())
    torch.cuda.synchronize()
    for bi in range(2):
        for h in range(3):
            want = oracle.sketch(as_f64(q[bi, h]), as_f64(G[h]), r, p)
            assert_close(M[bi, h].float().cpu().numpy(), want, "bf16", "sketch d=%d p=%d r=%d" % (d, p, r))


def test_single_block_fast_path_is_exact_polynomial_attention():
    cfg = mk(1, 1, 512, 64, 4, 64, 512)
    q, k, v, G = draw(cfg)
    got, desc = gpu_attn(cfg, q, k, v, G)
    assert psf.kernel_path(desc) == 1
    Q, K, V = as_f64(q)[0, 0], as_f64(k)[0, 0], as_f64(v)[0, 0]
    W = np.tril((Q @ K.T) ** 4)
    assert_close(got.numpy()[0, 0], (W @ V) / (1.0 + W.sum(1, keepdims=True)), "bf16", "b = n")


def sampled_parity(cfg, q, k, v, G, units, what):
    got, desc = gpu_attn(cfg, q, k, v, G)
    assert psf.kernel_path(desc) == 1
    rows = probe_rows(cfg["n"], cfg["b"])
    want = oracle_units_rows(cfg, q, k, v, G, units, rows)
    g = np.stack([got[bi, h].numpy()[rows] for bi, h in units])
    w = np.stack([want[u] for u in units])
    res = assert_close(g, w, "bf16", what)
    # properties that hold at any size: finite, convex-hull bound (weights are non-negative)
    gn = got.numpy()
    assert np.isfinite(gn).all()
    vmax = np.maximum.accumulate(np.abs(v.float().numpy()).max(-1), axis=-1)
    assert (np.abs(gn).max(-1) <= vmax * 1.01 + 1e-3).all()
    print(what, res)
    return got


def test_config2_sampled_rows_all_heads():
    cfg, q, k, v, G = inputs.make_config(2)
    units = [(bi, h) for bi in (0, 7) for h in range(cfg["heads"])]
    sampled_parity(cfg, q, k, v, G, units, "config 2")


def test_config3_headline_sampled_rows():
    cfg, q, k, v, G = inputs.make_config(3)
    units = [(0, h) for h in range(0, cfg["heads"], 3)] + [(1, 11)]
    sampled_parity(cfg, q, k, v, G, units, "config 3")


@pytest.mark.parametrize("variant", [None, "heavy"])
def test_config5_sampled_rows(variant):
    cfg, q, k, v, G = inputs.make_config(5, variant=variant)
    units = [(0, 0), (0, 7), (0, 15)]
    sampled_parity(cfg, q, k, v, G, units, "config 5 %s" % variant)


@pytest.mark.parametrize("n,r,b", [(8192, 32, 256), (16384, 64, 512), (65536, 64, 1024), (65536, 32, 256)])
def test_config4_sweep_points_reduced_batch(n, r, b):
    # sweep shapes at 2 batch entries instead of 2^20/n (units are independent; the full batch
    # is what bench.py --workload sweep times)
    cfg = mk(2, 12, n, 64, 4, r, b)
    q, k, v, G = draw(cfg, seed=1004)
    sampled_parity(cfg, q, k, v, G, [(0, 0), (1, 11)], "config 4 n=%d r=%d b=%d" % (n, r, b))


def test_state_kernel_two_workgroups_per_cu_variant():
    # 36 units x 10 workgroups exceed one per CU: the state kernel runs its half-chunk variant
    cfg = mk(3, 12, 2048, 64, 4, 64, 512)
    q, k, v, G = draw(cfg, seed=23)
    sampled_parity(cfg, q, k, v, G, [(0, 0), (1, 5), (2, 11)], "r=64, 36 units")


def test_state_kernel_symmetric_variant_r32_large_grid():
    # 192 units x 3 workgroups: r = 32 switches to the symmetric 16-wide segments
    cfg = mk(16, 12, 1024, 64, 4, 32, 256)
    q, k, v, G = draw(cfg, seed=29)
    sampled_parity(cfg, q, k, v, G, [(0, 0), (7, 3), (15, 11)], "r=32, 192 units")


def test_single_block_several_units():
    # t = 1: no state kernel, no cross-block phase, every unit still gets its own tiles
    cfg = mk(2, 3, 512, 64, 4, 64, 512, per_head=True)
    q, k, v, G = draw(cfg, seed=31)
    got, desc = gpu_attn(cfg, q, k, v, G)
    assert psf.kernel_path(desc) == 1
    assert_close(got.numpy(), oracle_attn(cfg, q, k, v, G), "bf16", "t = 1, 6 units")


def test_deterministic_across_runs():
    cfg = mk(1, 2, 2048, 64, 4, 64, 512)
    q, k, v, G = draw(cfg)
    a, _ = gpu_attn(cfg, q, k, v, G)
    b2, _ = gpu_attn(cfg, q, k, v, G)
    assert torch.equal(a, b2)


@pytest.mark.parametrize("d,p,r,b", [(64, 4, 64, 256), (64, 4, 32, 256), (64, 4, 64, 512), (128, 8, 64, 256),
                                     (64, 8, 32, 512)])
def test_in_block_weights_from_the_sketches_full_parity(d, p, r, b):
    """Section 3.1's in-block rule (L R^T)^2 on the MFMA path: every weight is <m(q), m(k)>^2."""
    cfg = mk(1, 2, 1024, d, p, r, b, per_head=True)
    q, k, v, G = draw(cfg, seed=37)
    got, desc = gpu_attn(cfg, q, k, v, G, local=psf.LOCAL_SKETCH)
    assert psf.kernel_path(desc) == 1
    want = oracle_attn(cfg, q, k, v, G, local=oracle.LOCAL_SKETCH)
    print("local sketch", (d, p, r, b), assert_close(got.numpy(), want, "bf16", "local sketch d=%d p=%d r=%d b=%d" % (d, p, r, b)))


@pytest.mark.parametrize("n,r", [(8192, 64), (16384, 32)])
def test_block_size_invariance_at_sweep_shapes(n, r):
    """With every weight taken from the sketches the function does not depend on b (the block
    decomposition is exact): the three block sizes of the sweep agree with each other within
    the bf16 tolerance and with the oracle (evaluated once, b irrelevant) on sampled rows."""
    outs = {}
    for b in (256, 512, 1024):
        cfg = mk(2, 12, n, 64, 4, r, b)
        q, k, v, G = draw(cfg, seed=1004)
        got, desc = gpu_attn(cfg, q, k, v, G, local=psf.LOCAL_SKETCH)
        assert psf.kernel_path(desc) == 1
        outs[b] = got.numpy()
    for b in (512, 1024):
        assert_close(outs[b], outs[256], "bf16", "b=%d against b=256" % b)
    rows = probe_rows(n, 1024)
    units = [(0, 0), (1, 11)]
    want = oracle_units_rows(cfg, q, k, v, G, units, rows, local=oracle.LOCAL_SKETCH, b=1024)
    for b in (256, 512, 1024):
        g = np.stack([outs[b][bi, h][rows] for bi, h in units])
        print("b-invariance", (n, r, b), assert_close(g, np.stack([want[u] for u in units]), "bf16", "b=%d" % b))


def test_in_block_sketch_rule_path_selection():
    assert psf.kernel_path(psf.make_desc(1, 2, 1024, 128, 4, 32, 256, "bf16", local=psf.LOCAL_SKETCH)) == 0
    assert psf.kernel_path(psf.make_desc(1, 2, 1024, 64, 4, 32, 256, "bf16", local=psf.LOCAL_SKETCH, learned=True)) == 0
    assert psf.kernel_path(psf.make_desc(1, 2, 1024, 128, 4, 64, 256, "bf16", local=psf.LOCAL_SKETCH)) == 1


@pytest.mark.parametrize("b,local", [(256, psf.LOCAL_EXACT), (512, psf.LOCAL_SKETCH), (1024, psf.LOCAL_EXACT)])
def test_base_case_degree_two_on_the_mfma_path(b, local):
    # p = 2: m(x) = x (Algorithm 1's base case), 64^2 = 4096 features, no randomness; the two
    # in-block rules coincide.  Full parity against the definition, which is exact degree-2
    # polynomial attention.
    cfg = mk(1, 2, 1024, 64, 2, 64, b)
    q, k, v = inputs.make_qkv(1, 2, 1024, 64, seed=19, dtype="bf16")
    got, desc = gpu_attn(cfg, q, k, v, None, local=local)
    assert psf.kernel_path(desc) == 1
    want = oracle_attn(cfg, q, k, v, None)
    print("p=2", (b, local), assert_close(got.numpy(), want, "bf16", "p=2 b=%d" % b))
    desc_r = psf.make_desc(1, 2, 1024, 64, 2, 16, b, "bf16", local=local)      # r is ignored for p = 2
    O2 = psf.psf_causal_attn_fwd(desc_r, q.cuda(), k.cuda(), v.cuda(), None)
    torch.cuda.synchronize()
    assert torch.equal(O2.float().cpu(), got)
    # learned sketches of degree 2 are the same base case (no network is applied): bit-equal
    desc_l = psf.make_desc(1, 2, 1024, 64, 2, 64, b, "bf16", local=local, learned=True)
    assert psf.kernel_path(desc_l) == 1
    O3 = psf.psf_causal_attn_fwd(desc_l, q.cuda(), k.cuda(), v.cuda(), None)
    O4 = psf.psf_noncausal_attn_fwd(desc_l, q.cuda(), k.cuda(), v.cuda(), None)
    O5 = psf.psf_noncausal_attn_fwd(desc, q.cuda(), k.cuda(), v.cuda(), None)
    torch.cuda.synchronize()
    assert torch.equal(O3.float().cpu(), got)
    assert torch.equal(O4, O5)


def test_forward_replays_from_a_captured_graph():
    # The library only enqueues kernels on the caller's stream (no allocation, no memset, no
    # synchronisation), so a call can be captured into a HIP graph: several replays, with eager
    # work and synchronisations between them, must reproduce the eager result bit for bit.
    cfg = mk(1, 2, 1024, 64, 4, 64, 256)
    q, k, v, G = draw(cfg)
    dev = torch.device("cuda:0")
    qd, kd, vd, Gd = q.to(dev), k.to(dev), v.to(dev), G.to(dev)
    desc = psf.make_desc(cfg["batch"], cfg["heads"], cfg["n"], cfg["d"], cfg["p"], cfg["r"], cfg["b"], "bf16",
                         per_head=cfg["per_head"])
    ws = psf.alloc_workspace(desc, dev)
    eager = psf.psf_causal_attn_fwd(desc, qd, kd, vd, Gd, workspace=ws).clone()
    torch.cuda.synchronize()
    O = torch.empty_like(eager)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        psf.psf_causal_attn_fwd(desc, qd, kd, vd, Gd, O=O, workspace=ws)       # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        psf.psf_causal_attn_fwd(desc, qd, kd, vd, Gd, O=O, workspace=ws)
    for rep in range(4):
        O.fill_(float("nan"))
        ws.random_(0, 255)                                   # eager work that dirties everything the graph rewrites
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(O, eager), "replay %d differs from the eager call" % rep


@pytest.mark.parametrize("k_scales,v_scale", [((8.0, 8.0), 1.0), ((1 / 16, 1 / 16), 64.0), ((8.0, 0.25), 1.0),
                                               ((0.25, 1.0, 16.0, 0.5), 1 / 256)])
def test_rows_of_other_norms_through_the_half_precision_state_kernel(k_scales, v_scale):
    """The state kernel of the d = r = 64 path multiplies fp16 operands; what keeps key rows of
    any norm inside fp16's exponent range is a power-of-two scale per 256..1024-token part of the
    key sketches, divided out again exactly.  Key rows of norm 8 (what layer normalisation gives
    at d = 64), of norm 1/16, and norms that change from block to block (so that the running
    accumulators are rescaled on the way), with values far from unit scale, against the oracle."""
    cfg = mk(1, 2, 2048, 64, 4, 64, 512)
    q, k, v, G = draw(cfg, seed=43)
    seg = cfg["n"] // len(k_scales)
    k = k.float()
    for i, sc in enumerate(k_scales):
        k[:, :, i * seg:(i + 1) * seg] *= sc
    k = k.to(torch.bfloat16)
    v = (v.float() * v_scale).to(torch.bfloat16)
    got, desc = gpu_attn(cfg, q, k, v, G)
    assert psf.kernel_path(desc) == 1
    want = oracle_attn(cfg, q, k, v, G)
    print("norms", k_scales, v_scale, assert_close_scaled(got.numpy(), want, "bf16", "k x %s, v x %s" % (k_scales, v_scale)))


@pytest.mark.parametrize("k_scales,v_scale", [((8.0, 0.25), 1.0), ((0.25, 1.0, 16.0, 0.5), 1 / 256)])
def test_rows_of_other_norms_through_the_half_precision_state_launch(k_scales, v_scale):
    """The same with more units than the fused launch takes (27 units x 10 state workgroups > 256
    CUs): the half-precision state kernel then runs as a launch of its own, two workgroups per
    CU, and the output kernel is the one-launch form."""
    cfg = mk(3, 9, 1024, 64, 4, 64, 256)
    q, k, v, G = draw(cfg, seed=47)
    seg = cfg["n"] // len(k_scales)
    k = k.float()
    for i, sc in enumerate(k_scales):
        k[:, :, i * seg:(i + 1) * seg] *= sc
    k = k.to(torch.bfloat16)
    v = (v.float() * v_scale).to(torch.bfloat16)
    got, desc = gpu_attn(cfg, q, k, v, G)
    assert psf.kernel_path(desc) == 1 and psf.fwd_beside_states(desc) == 0
    want = oracle_attn(cfg, q, k, v, G)
    print("norms, own launch", k_scales, v_scale,
          assert_close_scaled(got.numpy(), want, "bf16", "k x %s, v x %s" % (k_scales, v_scale)))
