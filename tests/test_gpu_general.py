"""GPU parity of the general fp32 path against the float64 oracle (through the C ABI)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2310_01655_amd import binding as psf
from paper_2310_01655_amd import inputs
from parity import as_f64, assert_close, gpu_attn, oracle_attn

pytestmark = pytest.mark.gpu


def small_cfg(**kw):
    cfg = dict(batch=2, heads=3, n=192, d=16, p=4, r=8, b=32, dtype="f32", per_head=True,
               dist="normal")
    cfg.update(kw)
    return cfg


def draw(cfg, seed=7):
    q, k, v = inputs.make_qkv(cfg["batch"], cfg["heads"], cfg["n"], cfg["d"], seed=seed,
                              dist=cfg["dist"], dtype=cfg["dtype"])
    G = inputs.make_sketch_matrices(cfg["heads"], cfg["d"], cfg["r"], cfg["p"],
                                    per_head=cfg["per_head"], seed=0, dtype=cfg["dtype"])
    return q, k, v, G


def test_config1_fp32_full_parity():
    cfg, q, k, v, G = inputs.make_config(1)
    got, desc = gpu_attn(cfg, q, k, v, G)
    assert psf.kernel_path(desc) == 0
    want = oracle_attn(cfg, q, k, v, G)
    print("config1", assert_close(got.numpy(), want, "f32", "config 1"))


@pytest.mark.parametrize("d,p,n,b", [(4, 4, 1024, 128), (8, 4, 1024, 128), (64, 2, 1024, 128)])
def test_exact_feature_mode_vs_brute_force(d, p, n, b):
    # phi(x) = x^{(x)p}: the library must reproduce masked (QK^T)^p attention itself
    cfg = dict(batch=1, heads=2, n=n, d=d, p=p, r=1, b=b, dtype="f32", per_head=False, dist="normal")
    q, k, v = inputs.make_qkv(1, 2, n, d, dv=d, seed=11, dtype="f32")
    got, desc = gpu_attn(cfg, q, k, v, None, feat=psf.FEAT_EXACT)
    Q, K, V = as_f64(q), as_f64(k), as_f64(v)
    W = np.tril(np.einsum("bhid,bhjd->bhij", Q, K) ** p)
    want = (W @ V) / (1.0 + W.sum(-1, keepdims=True))
    assert_close(got.numpy(), want, "f32", "exact features d=%d p=%d" % (d, p))
    assert_close(got.numpy(), oracle_attn(cfg, q, k, v, None, feat=oracle.FEAT_EXACT), "f32", "oracle")


def test_single_block_is_plain_polynomial_attention_d64_p4():
    cfg, q, k, v, G = inputs.make_config(1)
    n = cfg["n"]
    got, _ = gpu_attn(cfg, q, k, v, G, b=n)
    Q, K, V = as_f64(q)[0, 0], as_f64(k)[0, 0], as_f64(v)[0, 0]
    W = np.tril((Q @ K.T) ** 4)
    assert_close(got.numpy()[0, 0], (W @ V) / (1.0 + W.sum(1, keepdims=True)), "f32", "b = n")


@pytest.mark.parametrize("p", [2, 4, 8, 16])
@pytest.mark.parametrize("local", [psf.LOCAL_EXACT, psf.LOCAL_SKETCH])
def test_all_degrees_and_local_rules(p, local):
    cfg = small_cfg(p=p)
    q, k, v, G = draw(cfg)
    got, _ = gpu_attn(cfg, q, k, v, G if p > 2 else None, local=local)
    want = oracle_attn(cfg, q, k, v, G, local=local)
    assert_close(got.numpy(), want, "f32", "p=%d local=%d" % (p, local))


def test_block_size_invariance_with_sketched_local_weights():
    cfg = small_cfg(n=256, heads=1, batch=1, per_head=False)
    q, k, v, G = draw(cfg)
    outs = [gpu_attn(cfg, q, k, v, G, local=psf.LOCAL_SKETCH, b=b)[0].numpy() for b in (1, 4, 32, 256)]
    want = oracle_attn(cfg, q, k, v, G, local=oracle.LOCAL_SKETCH, b=32)
    for o in outs:
        assert_close(o, want, "f32", "b-invariance")


def test_ragged_shapes_and_odd_sizes():
    # d, dv, r not multiples of anything; b = 1 and b = n; single row
    for cfg in (small_cfg(n=35, b=7, d=5, r=3, heads=1), small_cfg(n=9, b=1, d=3, r=2),
                small_cfg(n=1, b=1, d=7, r=5, batch=1, heads=1)):
        q, k, v = inputs.make_qkv(cfg["batch"], cfg["heads"], cfg["n"], cfg["d"], dv=11, seed=3)
        G = inputs.make_sketch_matrices(cfg["heads"], cfg["d"], cfg["r"], cfg["p"], per_head=True)
        desc = psf.make_desc(cfg["batch"], cfg["heads"], cfg["n"], cfg["d"], cfg["p"], cfg["r"],
                             cfg["b"], "f32", dv=11, per_head=True)
        O = psf.psf_causal_attn_fwd(desc, q.cuda(), k.cuda(), v.cuda(), G.cuda())
        torch.cuda.synchronize()
        want = oracle_attn(cfg, q, k, v, G)
        assert_close(O.cpu().numpy(), want, "f32", str(cfg))


def test_bf16_storage_on_general_path():
    cfg = small_cfg(dtype="bf16", r=8)
    q, k, v, G = draw(cfg)
    got, desc = gpu_attn(cfg, q, k, v, G)
    assert psf.kernel_path(desc) == 0
    assert_close(got.numpy(), oracle_attn(cfg, q, k, v, G), "bf16", "bf16 storage")


@pytest.mark.parametrize("p", [2, 4, 8, 16])
def test_psf_sketch_m_and_phi(p):
    cfg = small_cfg(p=p, n=64)
    q, _, _, G = draw(cfg)
    desc = psf.make_desc(cfg["batch"], cfg["heads"], cfg["n"], cfg["d"], p, cfg["r"], cfg["b"],
                         "f32", per_head=True)
    M, Phi = psf.psf_sketch(desc, q.cuda(), G.cuda() if p > 2 else None, want_m=True, want_phi=True)
    torch.cuda.synchronize()
    for bi in range(cfg["batch"]):
        for h in range(cfg["heads"]):
            m = oracle.sketch(as_f64(q[bi, h]), as_f64(G[h]), cfg["r"], p)
            assert_close(M[bi, h].cpu().numpy(), m, "f32", "M p=%d" % p)
            assert_close(Phi[bi, h].cpu().numpy(), oracle.self_tensor(m), "f32", "Phi p=%d" % p)


def test_psf_sketch_exact_features():
    desc = psf.make_desc(1, 1, 32, 5, 4, 1, 8, "f32", feat=psf.FEAT_EXACT)
    x, _, _ = inputs.make_qkv(1, 1, 32, 5, seed=2)
    _, Phi = psf.psf_sketch(desc, x.cuda(), None, want_m=False, want_phi=True)
    torch.cuda.synchronize()
    assert_close(Phi[0, 0].cpu().numpy(), oracle.power_tensor(as_f64(x[0, 0]), 4), "f32", "x^(x)4")


def test_timed_entry_point_reports_stages():
    cfg, q, k, v, G = inputs.make_config(1)
    got, stages, desc = gpu_attn(cfg, q, k, v, G, timed=True)
    assert list(stages) == ["sketch_q", "sketch_k", "block_states", "exclusive_scan", "output"]
    assert all(ms >= 0 for ms in stages.values())
    assert_close(got.numpy(), oracle_attn(cfg, q, k, v, G), "f32", "timed")


def test_largest_admitted_dimensions():
    # d = dv = r = 256: every per-token array at its stated maximum (r^2 = 65536 features)
    cfg = dict(batch=1, heads=1, n=32, d=256, p=4, r=256, b=16, dtype="f32", per_head=False, dist="normal")
    q, k, v = inputs.make_qkv(1, 1, 32, 256, seed=3, dtype="f32")
    G = inputs.make_sketch_matrices(1, 256, 256, 4, seed=0, dtype="f32")
    got, _ = gpu_attn(cfg, q, k, v, G)
    assert_close(got.numpy(), oracle_attn(cfg, q, k, v, G), "f32", "d = dv = r = 256")


@pytest.mark.parametrize("dtype,d,r,b,n", [("f32", 16, 8, 16, 64), ("bf16", 64, 64, 256, 512), ("bf16", 64, 32, 256, 512)])
def test_degenerate_all_zero_queries_and_keys(dtype, d, r, b, n):
    # q = k = 0: every weight is 0, so o = 0 / (1 + 0) = 0 and every gradient is 0 -- on the
    # general and on the MFMA kernels, forward, backward and token by token; nothing may turn
    # into a NaN on the way (the 1 + keeps the denominator away from 0)
    batch, heads, p = 1, 2, 4
    dev = torch.device("cuda:0")
    td = inputs.torch_dtype(dtype)
    z = torch.zeros(batch, heads, n, d, dtype=td, device=dev)
    _, _, v = inputs.make_qkv(batch, heads, n, d, seed=71, dtype=dtype)
    dO = inputs.make_dout(batch, heads, n, d, seed=72, dtype=dtype)
    G = inputs.make_sketch_matrices(heads, d, r, p, per_head=True, seed=0, dtype=dtype)
    desc = psf.make_desc(batch, heads, n, d, p, r, b, dtype, per_head=True)
    O = psf.psf_causal_attn_fwd(desc, z, z, v.to(dev), G.to(dev))
    dQ, dK, dV = psf.psf_causal_attn_bwd(desc, z, z, v.to(dev), G.to(dev), dO.to(dev))
    state = psf.decode_new_state(desc, dev)
    rows = []
    for pos in range(b + 3):
        rows.append(psf.psf_decode_step(desc, z[:, :, pos:pos + 1].contiguous(), z[:, :, pos:pos + 1].contiguous(),
                                        v.to(dev)[:, :, pos:pos + 1].contiguous(), G.to(dev), pos, state).clone())
    torch.cuda.synchronize()
    for name, t in (("O", O), ("dQ", dQ), ("dK", dK), ("dV", dV), ("decoded rows", torch.cat(rows, 2))):
        assert torch.count_nonzero(t).item() == 0 and torch.isfinite(t.float()).all(), name
