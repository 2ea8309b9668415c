"""GPU parity of the learned-sketch variant (Algorithm 2) against the float64 oracle, through
the C ABI: the sketch entry point, the general fp32 attention path and the bf16 MFMA path
(degree 4 with d = 64: the MFMA network kernel; otherwise sketches from the fp32 kernel; then the
MFMA state / output kernels)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2310_01655_amd import binding as psf
from paper_2310_01655_amd import inputs
from parity import as_f64, assert_close

pytestmark = pytest.mark.gpu


def case(batch, heads, n, d, p, r, b, dtype, per_head=True, seed=61):
    q, k, v = inputs.make_qkv(batch, heads, n, d, seed=seed, dtype=dtype)
    P = inputs.make_learned_params(heads, d, r, p, per_head=per_head, seed=3, dtype=dtype)
    desc = psf.make_desc(batch, heads, n, d, p, r, b, dtype, per_head=per_head, learned=True)
    return q, k, v, P, desc


def oracle_rows(q, k, v, P, p, r, b):
    out = np.empty(tuple(v.shape), dtype=np.float64)
    for bi in range(q.shape[0]):
        for h in range(q.shape[1]):
            out[bi, h] = oracle.attn_def(as_f64(q[bi, h]), as_f64(k[bi, h]), as_f64(v[bi, h]),
                                         as_f64(P[h if P.shape[0] > 1 else 0]), p, r, b, learned=True)
    return out


def test_lengths_agree_between_library_oracle_and_generator():
    for d, r, p in ((64, 64, 4), (64, 32, 8), (128, 64, 4), (24, 12, 4), (64, 64, 2)):
        assert psf.learned_len(d, r, p) == oracle.learned_len(d, r, p) == inputs.learned_len(d, r, p)


@pytest.mark.parametrize("d,p,r", [(64, 4, 16), (24, 4, 12), (32, 8, 16), (64, 4, 64)])
def test_sketch_entry_point_learned_fp32(d, p, r):
    q, _, _, P, desc = case(1, 2, 64, d, p, r, 32, "f32")
    M, Phi = psf.psf_sketch(desc, q.cuda(), P.cuda(), want_m=True, want_phi=True)
    torch.cuda.synchronize()
    for h in range(2):
        want = oracle.sketch_learned(as_f64(q[0, h]), as_f64(P[h]), r, p)
        assert_close(M[0, h].cpu().numpy(), want, "f32", "learned m d=%d p=%d r=%d" % (d, p, r))
        assert_close(Phi[0, h].cpu().numpy(), oracle.self_tensor(want), "f32", "learned phi")


@pytest.mark.parametrize("p,local", [(4, psf.LOCAL_EXACT), (8, psf.LOCAL_EXACT), (4, psf.LOCAL_SKETCH)])
def test_attention_general_path_learned_fp32(p, local):
    batch, heads, n, d, r, b = 1, 2, 128, 32, 16, 32
    q, k, v = inputs.make_qkv(batch, heads, n, d, seed=62, dtype="f32")
    P = inputs.make_learned_params(heads, d, r, p, per_head=True, seed=3, dtype="f32")
    desc = psf.make_desc(batch, heads, n, d, p, r, b, "f32", per_head=True, learned=True, local=local)
    assert psf.kernel_path(desc) == 0
    O = psf.psf_causal_attn_fwd(desc, q.cuda(), k.cuda(), v.cuda(), P.cuda())
    torch.cuda.synchronize()
    want = np.empty(tuple(v.shape))
    for h in range(heads):
        want[0, h] = oracle.attn_def(as_f64(q[0, h]), as_f64(k[0, h]), as_f64(v[0, h]), as_f64(P[h]), p, r, b,
                                     local=oracle.LOCAL_EXACT if local == psf.LOCAL_EXACT else oracle.LOCAL_SKETCH,
                                     learned=True)
    print("general learned", p, assert_close(O.cpu().numpy(), want, "f32", "general learned p=%d" % p))


@pytest.mark.parametrize("d,p,r,b", [(64, 4, 64, 256), (64, 4, 32, 256), (128, 4, 64, 256), (64, 8, 32, 512),
                                     (64, 8, 64, 256), (128, 8, 32, 256)])
def test_attention_mfma_path_learned_bf16(d, p, r, b):
    q, k, v, P, desc = case(1, 2, 1024, d, p, r, b, "bf16")
    assert psf.kernel_path(desc) == 1
    O = psf.psf_causal_attn_fwd(desc, q.cuda(), k.cuda(), v.cuda(), P.cuda())
    torch.cuda.synchronize()
    want = oracle_rows(q, k, v, P, p, r, b)
    print("mfma learned", (d, p, r, b), assert_close(O.float().cpu().numpy(), want, "bf16", "mfma learned"))


@pytest.mark.parametrize("per_head,heads,n,b,r", [(False, 3, 2048, 512, 64), (True, 3, 2048, 1024, 32),
                                                  (True, 2, 1536, 768, 64)])
def test_attention_mfma_learned_kernel_sets_and_blocks(per_head, heads, n, b, r):
    """Degree 4, d = 64: the MFMA network kernel with shared and per-head parameters, several
    256-token workgroups per block and several blocks."""
    q, k, v, P, desc = case(2, heads, n, 64, 4, r, b, "bf16", per_head=per_head, seed=67)
    assert psf.kernel_path(desc) == 1
    O = psf.psf_causal_attn_fwd(desc, q.cuda(), k.cuda(), v.cuda(), P.cuda())
    torch.cuda.synchronize()
    want = oracle_rows(q, k, v, P, 4, r, b)
    print("mfma learned sets", (per_head, heads, n, b, r),
          assert_close(O.float().cpu().numpy(), want, "bf16", "mfma learned sets"))


@pytest.mark.parametrize("per_head,heads,n,b,r", [(False, 3, 1024, 512, 64), (True, 3, 1536, 768, 32)])
def test_attention_mfma_learned_kernel_degree_8(per_head, heads, n, b, r):
    """Degree 8, d = 64: six networks per set on the MFMA network kernel (two of them take the
    first-level sketches as input), shared and per-head parameters, several workgroups per block."""
    q, k, v, P, desc = case(2, heads, n, 64, 8, r, b, "bf16", per_head=per_head, seed=69)
    assert psf.kernel_path(desc) == 1
    O = psf.psf_causal_attn_fwd(desc, q.cuda(), k.cuda(), v.cuda(), P.cuda())
    torch.cuda.synchronize()
    want = oracle_rows(q, k, v, P, 8, r, b)
    print("mfma learned degree 8", (per_head, heads, n, b, r),
          assert_close(O.float().cpu().numpy(), want, "bf16", "mfma learned degree 8"))


def test_config3_shape_learned_sampled_rows():
    """The workload `bench.py --learned` times (config 3 shapes, per-head parameters), on sampled
    rows of two units.  The oracle's network runs over all keys of the unit (in slices on a few
    threads: its C loops release the interpreter lock), the weights of the sampled rows are then
    the definition written out: exact degree-4 inside the row's block, squared inner product of
    the learned sketches before it, causal, `1 +` in the denominator."""
    from concurrent.futures import ThreadPoolExecutor
    from parity import probe_rows
    cfg = dict(inputs.CONFIGS[3])
    n, b, r, heads = cfg["n"], cfg["b"], cfg["r"], cfg["heads"]
    q, k, v, P, desc = case(cfg["batch"], heads, n, cfg["d"], 4, r, b, "bf16", per_head=True, seed=1003)
    assert psf.kernel_path(desc) == 1
    O = psf.psf_causal_attn_fwd(desc, q.cuda(), k.cuda(), v.cuda(), P.cuda())
    torch.cuda.synchronize()
    got = O.float().cpu().numpy()
    assert np.isfinite(got).all()
    rows = np.array(probe_rows(n, b))
    for bi, h in ((0, 0), (1, 7)):
        Q, K, V, Ph = as_f64(q[bi, h]), as_f64(k[bi, h]), as_f64(v[bi, h]), as_f64(P[h])
        with ThreadPoolExecutor(8) as ex:
            parts = list(ex.map(lambda lo: oracle.sketch_learned(K[lo:lo + 2048], Ph, r, 4), range(0, n, 2048)))
        MK = np.concatenate(parts)
        MQ = oracle.sketch_learned(Q[rows], Ph, r, 4)
        W = (MQ @ MK.T) ** 2
        same = (rows[:, None] // b) == (np.arange(n)[None, :] // b)
        W = np.where(same, (Q[rows] @ K.T) ** 4, W) * (np.arange(n)[None, :] <= rows[:, None])
        want = (W @ V) / (1.0 + W.sum(1, keepdims=True))
        print("config 3 learned", (bi, h), assert_close(got[bi, h][rows], want, "bf16", "config 3 learned"))


def test_decode_with_learned_sketches():
    batch, heads, n, d, p, r, b = 1, 2, 96, 32, 4, 16, 32
    q, k, v, P, desc = case(batch, heads, n, d, p, r, b, "f32")
    dev = torch.device("cuda:0")
    qd, kd, vd, Pd = q.to(dev), k.to(dev), v.to(dev), P.to(dev)
    state = psf.decode_new_state(desc, dev)
    out = torch.empty(batch, heads, n, d, device=dev)
    for pos in range(n):
        o = psf.psf_decode_step(desc, qd[:, :, pos:pos + 1].contiguous(), kd[:, :, pos:pos + 1].contiguous(),
                                vd[:, :, pos:pos + 1].contiguous(), Pd, pos, state)
        out[:, :, pos] = o[:, :, 0]
    torch.cuda.synchronize()
    assert_close(out.cpu().numpy(), oracle_rows(q, k, v, P, p, r, b), "f32", "decode learned")


def test_degree_16_and_exact_features_are_refused():
    assert psf.check_desc(psf.make_desc(1, 1, 64, 16, 16, 8, 16, "f32", learned=True)) == 3
    assert psf.check_desc(psf.make_desc(1, 1, 64, 4, 4, 8, 16, "f32", learned=True, feat=psf.FEAT_EXACT)) == 3
