"""GPU parity of psf_noncausal_attn_fwd (Polysketch attention without a mask, Section 2.2)
against the float64 oracle, through the C ABI, on both kernel paths."""
import numpy as np
import pytest
import torch

import oracle
from paper_2310_01655_amd import binding as psf
from paper_2310_01655_amd import inputs
from parity import as_f64, assert_close

pytestmark = pytest.mark.gpu


def run_case(batch, heads, n, d, dv, p, r, b, dtype, feat=None, per_head=True, learned=False, seed=71, path=None):
    feat = psf.FEAT_SKETCH if feat is None else feat
    q, k, v = inputs.make_qkv(batch, heads, n, d, dv=dv, seed=seed, dtype=dtype)
    if feat == psf.FEAT_EXACT or p == 2:
        G = None
    elif learned:
        G = inputs.make_learned_params(heads, d, r, p, per_head=per_head, seed=3, dtype=dtype)
    else:
        G = inputs.make_sketch_matrices(heads, d, r, p, per_head=per_head, seed=0, dtype=dtype)
    desc = psf.make_desc(batch, heads, n, d, p, r, b, dtype, dv=dv, feat=feat, per_head=per_head, learned=learned)
    if path is not None:
        assert psf.kernel_path(desc) == path
    dev = torch.device("cuda:0")
    O = psf.psf_noncausal_attn_fwd(desc, q.to(dev), k.to(dev), v.to(dev), G.to(dev) if G is not None else None)
    torch.cuda.synchronize()
    want = np.empty(tuple(v.shape))
    for bi in range(batch):
        for h in range(heads):
            g = None if G is None else as_f64(G[h if G.shape[0] > 1 else 0])
            want[bi, h] = oracle.attn_noncausal(as_f64(q[bi, h]), as_f64(k[bi, h]), as_f64(v[bi, h]), g, p, r,
                                                feat=oracle.FEAT_EXACT if feat == psf.FEAT_EXACT else oracle.FEAT_SKETCH,
                                                learned=learned)
    res = assert_close(O.float().cpu().numpy(), want, dtype, "noncausal n=%d d=%d p=%d r=%d b=%d" % (n, d, p, r, b))
    print("noncausal", (n, d, dv, p, r, b, dtype, learned), res)
    return O


@pytest.mark.parametrize("n,d,dv,p,r,b", [
    (96, 16, 12, 4, 8, 32),        # three blocks, dv != d
    (128, 24, 24, 2, 16, 32),      # p = 2: features are x (x) x
    (128, 32, 32, 8, 16, 32),
    (64, 16, 16, 4, 8, 64),        # one block
    (48, 16, 16, 4, 8, 1),         # every token its own block
    (100, 20, 12, 4, 10, 25),      # sizes that are no powers of two
])
def test_noncausal_general_fp32(n, d, dv, p, r, b):
    run_case(2, 2, n, d, dv, p, r, b, "f32", path=0)


def test_noncausal_general_exact_features_and_bf16_storage_and_learned():
    run_case(1, 2, 64, 4, 4, 4, 8, 16, "f32", feat=psf.FEAT_EXACT, path=0)
    run_case(1, 2, 128, 32, 32, 4, 16, 32, "bf16", path=0)
    run_case(1, 2, 96, 16, 16, 4, 8, 32, "f32", learned=True, path=0)


@pytest.mark.parametrize("n,d,p,r,b", [(1024, 64, 4, 64, 256), (1024, 64, 4, 32, 256), (768, 64, 4, 64, 256),
                                       (512, 128, 8, 64, 256), (1024, 64, 8, 32, 512), (512, 64, 4, 64, 512)])
def test_noncausal_mfma_bf16(n, d, p, r, b):
    run_case(1, 2, n, d, d, p, r, b, "bf16", path=1)


def test_noncausal_mfma_learned_and_shared_matrices():
    run_case(1, 2, 1024, 64, 64, 4, 64, 256, "bf16", learned=True, path=1)
    run_case(2, 3, 512, 64, 64, 4, 32, 256, "bf16", per_head=False, path=1)


def test_noncausal_does_not_depend_on_the_block_size_and_differs_from_causal():
    a = run_case(1, 2, 1024, 64, 64, 4, 64, 256, "bf16", path=1)
    b2 = run_case(1, 2, 1024, 64, 64, 4, 64, 1024, "bf16", path=1)
    assert torch.equal(a, b2)                        # b only partitions the work on this path: same kernels, same order
    c = run_case(1, 1, 96, 16, 16, 4, 8, 32, "f32", path=0)
    d2 = run_case(1, 1, 96, 16, 16, 4, 8, 96, "f32", path=0)
    np.testing.assert_allclose(c.cpu().numpy(), d2.cpu().numpy(), rtol=2e-5, atol=2e-6)
