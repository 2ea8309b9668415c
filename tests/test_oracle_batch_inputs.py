"""Host-side checks: the oracle's batch driver agrees with its single-unit function, and the
seeded input generators are deterministic and shaped as documented."""
import numpy as np
import torch

import oracle
from paper_2310_01655_amd import inputs


def test_batch_driver_matches_single_unit_and_head_indexing():
    q, k, v = inputs.make_qkv(2, 3, 32, 8, seed=5)
    G = inputs.make_sketch_matrices(3, 8, 4, 4, per_head=True, seed=0)
    rows = [0, 7, 8, 31]
    O, threads = oracle.attn_def_batch(q.numpy(), k.numpy(), v.numpy(), G.numpy(), 4, 4, 8, rows=rows)
    assert threads >= 1 and O.shape == (2, 3, 4, 8)
    for bi in range(2):
        for h in range(3):
            want = oracle.attn_def(q[bi, h].numpy(), k[bi, h].numpy(), v[bi, h].numpy(),
                                   G[h].numpy(), 4, 4, 8, rows=rows)
            np.testing.assert_array_equal(O[bi, h], want)
    Gs = inputs.make_sketch_matrices(3, 8, 4, 4, per_head=False, seed=0)
    O1, _ = oracle.attn_def_batch(q.numpy(), k.numpy(), v.numpy(), Gs.numpy(), 4, 4, 8)
    want = oracle.attn_def(q[1, 2].numpy(), k[1, 2].numpy(), v[1, 2].numpy(), Gs[0].numpy(), 4, 4, 8)
    np.testing.assert_array_equal(O1[1, 2], want)


def test_inputs_are_seeded_unit_norm_and_rounded():
    q, k, v = inputs.make_qkv(1, 2, 64, 16, seed=3, dtype="bf16")
    q2, _, _ = inputs.make_qkv(1, 2, 64, 16, seed=3, dtype="bf16")
    assert q.dtype == torch.bfloat16 and torch.equal(q, q2)
    assert torch.allclose(q.float().norm(dim=-1), torch.ones(1, 2, 64), atol=2e-2)
    assert abs(v.float().std().item() - 1.0) < 0.1
    qt, kt, _ = inputs.make_qkv(1, 1, 4096, 8, seed=4, dist="student_t3")
    assert torch.allclose(qt.norm(dim=-1), torch.ones(1, 1, 4096), atol=1e-5)
    # heavy tails concentrate a unit row's mass on few coordinates far more often than Gaussians do
    qn, _, _ = inputs.make_qkv(1, 1, 4096, 8, seed=4)
    assert (qt.abs().max(-1).values > 0.95).float().mean() > 3 * (qn.abs().max(-1).values > 0.95).float().mean()
    assert inputs.g_len(64, 64, 8) == 4 * 64 * 64 + 2 * 64 * 64 == oracle.g_len(64, 64, 8)
    assert inputs.g_len(64, 16, 4) == oracle.g_len(64, 16, 4)
    G = inputs.make_sketch_matrices(12, 64, 32, 4, per_head=True)
    assert G.shape == (12, 2 * 64 * 32) and not torch.equal(G[0], G[1])
    assert len(inputs.sweep_configs()) == 24 and all(c["batch"] * c["n"] == 1 << 20 for c in inputs.sweep_configs())
