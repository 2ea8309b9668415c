"""Benchmark of causal polysketch attention on one MI355X.

Default: the forward hot path; a step = one full pass (sketch of Q and K, block prefix states,
fused output) over one synthetic batch.  `--pass bwd` times the backward entry point instead
(a step = gradients with respect to Q, K, V, forward quantities recomputed inside);
`--pass train` the forward that keeps its state plus the backward that uses it; `--pass decode`
the token-by-token entry point at a serving shape.  Prints ONE JSON line: metric, value, unit,
the step time, the workload, and two objects -- `roofline` (the dominant kernel's algorithmic
flops or bytes over its HIP-event time against the MI355X peak) and `cpu_baseline` (the float64
oracle timed on the host cores on a bounded sample of the same workload).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0      # MI355X dense bf16 MFMA, published
FP32_VALU_PEAK_TFLOPS = 157.3       # MI355X fp32 vector, published (256 CUs x 128 FMA lanes x 2.4 GHz)
HBM_PEAK_GBS = 8000.0

# HBM bytes per launch of the dominant kernel, from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# runs summarised in profiles/ (scaled by the copy calibration described there).  bench.py
# cannot collect counters itself; workloads without a committed counter run report null.
MEASURED_TRAFFIC_BYTES = {
    ("config3", "output"): 0.802e9,                 # k_out, cross-block part: 631 MB read + 171 MB written
    ("config3", "block_states_scan"): 1.529e9,      # k_state_and_in_block: 965 MB read + 564 MB written
}


def workloads():
    from paper_2310_01655_amd import inputs
    w = {"config%d" % i: dict(c) for i, c in inputs.CONFIGS.items()}
    for c in inputs.sweep_configs():
        w["sweep_n%d_r%d_b%d" % (c["n"], c["r"], c["b"])] = c
    return w


def stage_flops(cfg, learned=False, noncausal=False, local_sketch=False):
    """Algorithmic flops per step (multiply-add = 2), split by kernel stage.  Causal lower
    triangle only; the first block has no prefix and the last block's state is never needed.
    noncausal: one state over all n keys, applied to all n queries, no in-block pairs."""
    U = cfg["batch"] * cfg["heads"]
    n, d, r, b, p = cfg["n"], cfg["d"], cfg["r"], cfg["b"], cfg["p"]
    # Algorithm 1 on both sides: p/2 projections of 2 d r flops per row for Q and for K (8 n d r
    # at p = 4), plus the two r x r projections per side of the second level at p = 8
    sketch = 8 * n * d * r if p == 4 else 16 * n * d * r + 8 * n * r * r
    if learned:          # p - 2 networks per row: four dense layers each (Appendix D)
        net = lambda win: 2 * (win * 8 * r + 24 * r * r)
        sketch = 2 * n * ((p // 2) * net(d) + max(p // 2 - 2, 0) * net(r))
    if noncausal:
        f = {"sketch_and_layouts": U * (sketch + 2 * n * r * r), "block_states_scan": U * 2 * n * r * r * d,
             "output": U * 2 * n * r * r * (d + 1)}
        f["total"] = sum(f.values())
        return f
    f = {
        "sketch_and_layouts": U * (sketch + 2 * (n - b) * r * r),      # + ones column of H_l
        "block_states_scan": U * 2 * (n - b) * r * r * d,               # H_l and Z_l
        # in-block pairs: score over d (or over r with the sketched in-block rule), weights x [V | 1]
        "output": U * (2 * (n - b) * r * r * (d + 1) + n * (b + 1) * ((r if local_sketch else d) + d + 1)),
    }
    f["total"] = sum(f.values())
    return f


def cpu_baseline_noncausal(cfg, q, k, v, G):
    """The float64 oracle of the unmasked attention: the first 1024 queries of `cores` units
    against all n keys of their unit, one unit per thread (the C loops release the lock)."""
    from concurrent.futures import ThreadPoolExecutor
    import oracle
    cores = min(os.cpu_count() or 1, 16)
    units = min(cores, cfg["batch"] * cfg["heads"])
    sel = [(i // cfg["heads"], i % cfg["heads"]) for i in range(units)]
    nq = min(cfg["n"], 1024)
    f64 = lambda t: t.double().numpy()

    def one(unit):
        bi, h = unit
        g = f64(G[h] if G.shape[0] > 1 else G[0])
        return oracle.attn_noncausal(f64(q[bi, h, :nq]), f64(k[bi, h]), f64(v[bi, h]), g, cfg["p"], cfg["r"])

    t0 = time.perf_counter()
    with ThreadPoolExecutor(units) as ex:
        list(ex.map(one, sel))
    dt = time.perf_counter() - t0
    return {"value": units * nq / dt, "unit": "tokens/s", "cores": units, "kind": "oracle",
            "sample": "first %d queries of %d units against all n=%d keys (float64 definition)" % (nq, units, cfg["n"]),
            "seconds_measured": dt}


def bwd_stage_flops(cfg, learned=False):
    """Algorithmic flops of one backward step (multiply-add = 2) by stage of
    psf_causal_attn_bwd.  F = r^2 features, kc = dv + 1 columns, pairs = causal pairs inside
    blocks; states cover n - b tokens (first / last block excluded as in the forward count)."""
    U = cfg["batch"] * cfg["heads"]
    n, d, r, b, p = cfg["n"], cfg["d"], cfg["r"], cfg["b"], cfg["p"]
    F, kc = r * r, d + 1
    pairs = n * (b + 1) // 2
    sketch = 8 * n * d * r if p == 4 else 16 * n * d * r + 8 * n * r * r      # Algorithm 1 for Q and K
    cross = 2 * (n - b) * F * kc                                             # one state-sized contraction
    f = {
        "sketches": U * sketch,
        "forward_rows": U * (2 * cross + pairs * 2 * (d + kc)),              # H_l, phi^T Z_l, in-block rows
        "reverse_states": U * cross,
        "query_side": U * (cross + 4 * (n - b) * F + pairs * 2 * (kc + 2 * d)),
        "key_side": U * (2 * cross + 4 * (n - b) * F + pairs * 2 * (kc + 2 * d + d)),
        "sketch_gradient": U * 2 * sketch,                                   # recompute + transposed products
    }
    if learned:
        # Algorithm 2: p - 2 networks per row and side; forward once in the sketch stage; in the
        # gradient stage the values again, a second forward per network, the products with the
        # transposed matrices (one forward's worth) and the outer products of the parameter
        # gradient (one more)
        net = lambda win: 2 * (win * 8 * r + 24 * r * r)
        nets = 2 * n * ((p // 2) * net(d) + max(p // 2 - 2, 0) * net(r))
        f["sketches"] = U * nets
        f["sketch_gradient"] = U * 4 * nets
    f["total"] = sum(f.values())
    return f


def bwd_stage_flops_mfma(cfg, learned=False):
    """The same count by stage of the MFMA backward kernels (d = dv, p = 4)."""
    U = cfg["batch"] * cfg["heads"]
    n, d, r, b, p = cfg["n"], cfg["d"], cfg["r"], cfg["b"], cfg["p"]
    F, kc = r * r, d + 1
    pairs = n * (b + 1) // 2
    cross = 2 * (n - b) * F * kc
    sketch = 8 * n * d * r if p == 4 else 16 * n * d * r + 8 * n * r * r      # Algorithm 1 for Q and K
    f = {
        "forward_again": stage_flops(cfg, learned=learned)["total"],
        "g_c_and_layouts": U * 4 * n * d,
        "mirror_states": U * cross,
        "in_block_and_dv": U * (pairs * 2 * 7 * d + cross),                  # 3 + 4 tile products per pair; phi'(K)^T R_l
        # dm(q), dm(k) with their S / Rc terms; projections again + transposed products
        "cross_block_and_sketch_gradient": U * (2 * cross + 8 * (n - b) * F + 2 * sketch),
    }
    if learned:
        # in place of Algorithm 1's reverse: the two networks of every row and side forward again,
        # their pre-activations per hidden chunk once more, the products with the transposed
        # matrices and the outer products of the parameter gradient (one forward's worth each)
        nets = 2 * n * 2 * 2 * (d * 8 * r + 24 * r * r)
        f["cross_block_and_sketch_gradient"] = U * (2 * cross + 8 * (n - b) * F + 4 * nets)
    f["total"] = sum(f.values())
    return f


# HBM bytes per step and stage of the MFMA backward pass (Gaussian sketches, exact in-block weights),
# from rocprofv3 FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0 summed over the stage's kernels
# (profiles/config3_backward_mfma_kernel_trace.md, profiles/config5_backward_mfma_kernel_trace.md)
MIB = 1048576
BWD_MEASURED_TRAFFIC_BYTES = {
    ("config3", "forward_again"): 2722 * MIB, ("config3", "g_c_and_layouts"): 1638 * MIB,
    ("config3", "mirror_states"): 2398 * MIB, ("config3", "in_block_and_dv"): 2675 * MIB,
    ("config3", "cross_block_and_sketch_gradient"): 2042 * MIB,
    ("config5", "forward_again"): 1695 * MIB, ("config5", "g_c_and_layouts"): 1088 * MIB,
    ("config5", "mirror_states"): 2551 * MIB, ("config5", "in_block_and_dv"): 1905 * MIB,
    ("config5", "cross_block_and_sketch_gradient"): 1999 * MIB,
}


def cpu_baseline_bwd(cfg, q, k, v, G, dO):
    """The float64 gradient oracle (O(n^2) pair loop) on `cores` units; sequences longer than
    8192 are cut to their first 8192 tokens (a prefix of a causal sequence is a smaller instance
    of the same problem) so that the sample stays within tens of seconds."""
    import numpy as np
    import oracle
    cores = min(os.cpu_count() or 1, 16)
    units = min(cores, cfg["batch"] * cfg["heads"])
    sel = [(i // cfg["heads"], i % cfg["heads"]) for i in range(units)]
    n_s = min(cfg["n"], 8192)
    f64 = lambda t: np.stack([t[bi, h, :n_s].double().numpy() for bi, h in sel])[None]
    Gs = G.double().numpy()
    Gs = Gs[[h for _, h in sel]] if Gs.shape[0] > 1 else Gs
    t0 = time.perf_counter()
    *_, threads = oracle.attn_bwd_batch(f64(q), f64(k), f64(v), Gs, f64(dO), cfg["p"], cfg["r"], cfg["b"],
                                        max_threads=cores)
    dt = time.perf_counter() - t0
    return {"value": units * n_s / dt, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": "%d units, first %d of n=%d tokens each (float64 pair-by-pair gradient, O(n^2))"
                      % (units, n_s, cfg["n"]),
            "seconds_measured": dt}


def run_backward(args, cfg, psf, inputs, torch, q, k, v, G, idx):
    dev = torch.device("cuda:0")
    dO = inputs.make_dout(cfg["batch"], cfg["heads"], cfg["n"], cfg["d"], seed=1000 + idx, dtype=cfg["dtype"])
    desc = psf.make_desc(cfg["batch"], cfg["heads"], cfg["n"], cfg["d"], cfg["p"], cfg["r"], cfg["b"],
                         cfg["dtype"], per_head=cfg["per_head"], learned=args.learned,
                         local=psf.LOCAL_SKETCH if args.local_sketch else psf.LOCAL_EXACT)
    qd, kd, vd, Gd, dOd = (x.to(dev) for x in (q, k, v, G, dO))
    ws = psf.alloc_bwd_workspace(desc, dev)
    stream = torch.cuda.current_stream()
    # learned sketches: the call that also returns the gradient of the networks' parameters
    step = psf.psf_causal_attn_bwd_learned if args.learned else psf.psf_causal_attn_bwd
    ramp_steps = ramp(lambda: step(desc, qd, kd, vd, Gd, dOd, workspace=ws, stream=stream), args.ramp_ms, torch)
    for _ in range(args.warmup):
        step(desc, qd, kd, vd, Gd, dOd, workspace=ws, stream=stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(desc, qd, kd, vd, Gd, dOd, workspace=ws, stream=stream)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3
    reps = max(2, min(args.steps, 5))
    acc = {}
    for _ in range(reps):
        _, st = psf.psf_causal_attn_bwd_timed(desc, qd, kd, vd, Gd, dOd, workspace=ws, stream=stream)
        for nm, ms in st.items():
            acc[nm] = acc.get(nm, 0.0) + ms / reps
    mfma = psf.bwd_kernel_path(desc) == 3
    fl = bwd_stage_flops_mfma(cfg, learned=args.learned) if mfma else bwd_stage_flops(cfg, learned=args.learned)
    dom = max(acc, key=lambda nm: acc[nm])
    achieved = fl[dom] / (acc[dom] * 1e-3) / 1e12
    peak = MFMA_BF16_PEAK_TFLOPS if mfma else FP32_VALU_PEAK_TFLOPS
    out = {
        "metric": "causal_polysketch_attention_bwd_tokens_per_s",
        "value": cfg["batch"] * cfg["n"] * args.steps / elapsed, "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "ramp_steps": ramp_steps,
        "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if mfma else "f32", "data": "synthetic",
        "config": {"workload": args.workload, "pass": "bwd", "batch": cfg["batch"], "heads": cfg["heads"],
                   "n": cfg["n"], "d": cfg["d"], "p": cfg["p"], "r": cfg["r"], "b": cfg["b"],
                   "in_block": "sketch" if args.local_sketch else "exact",
                   "sketch": "learned" if args.learned else "gaussian",
                   "storage": cfg["dtype"], "kernel_path": "mfma_bf16" if mfma else "general_fp32"},
        "stage_ms": {nm: round(ms, 4) for nm, ms in acc.items()},
        "tflops": fl["total"] / (ms_per_step * 1e-3) / 1e12,
        "roofline": {"kernel": dom, "bound": "mfma" if mfma else "alu", "achieved": achieved, "peak": peak,
                     "unit": "TFLOP/s", "frac": achieved / peak,
                     "traffic": (BWD_MEASURED_TRAFFIC_BYTES.get((args.workload, dom))
                                 if mfma and not args.learned and not args.local_sketch else None),
                     "per_stage_tflops": {nm: fl[nm] / (acc[nm] * 1e-3) / 1e12 for nm in acc}},
    }
    if args.learned:
        out["stage_note"] = ("stage_ms from the timed call, which leaves out the parameter sums; "
                             "ms_per_step is the whole call with them")
    if not args.no_cpu_baseline and not args.local_sketch and not args.learned:   # the oracle driver used here: Gaussian sketches, exact in-block weights
        out["cpu_baseline"] = cpu_baseline_bwd(cfg, q, k, v, G, dO)
    print(json.dumps(out))


def run_train(args, cfg, psf, inputs, torch, q, k, v, G, idx):
    """One training step of the attention layer: forward that keeps its states, then backward
    from them (psf_causal_attn_fwd_save + psf_causal_attn_bwd_saved)."""
    dev = torch.device("cuda:0")
    dO = inputs.make_dout(cfg["batch"], cfg["heads"], cfg["n"], cfg["d"], seed=1000 + idx, dtype=cfg["dtype"])
    desc = psf.make_desc(cfg["batch"], cfg["heads"], cfg["n"], cfg["d"], cfg["p"], cfg["r"], cfg["b"],
                         cfg["dtype"], per_head=cfg["per_head"], learned=args.learned)
    if psf.bwd_kernel_path(desc) != 3:
        sys.exit("--pass train needs a workload the MFMA backward kernels cover (config2, config3, config5, the sweep points; "
                 "with --learned: d = 64, p = 4)")
    qd, kd, vd, Gd, dOd = (x.to(dev) for x in (q, k, v, G, dO))
    ws = psf.alloc_bwd_workspace(desc, dev)
    save = torch.empty(psf.fwd_save_bytes(desc), dtype=torch.uint8, device=dev)
    O = torch.empty_like(vd)
    grads = (torch.empty_like(qd), torch.empty_like(kd), torch.empty_like(vd))
    stream = torch.cuda.current_stream()

    # learned sketches: the call that also returns the gradient of the networks' parameters
    bwd = psf.psf_causal_attn_bwd_saved_learned if args.learned else psf.psf_causal_attn_bwd_saved

    def step():
        psf.psf_causal_attn_fwd_save(desc, qd, kd, vd, Gd, O=O, save=save, stream=stream)
        bwd(desc, qd, kd, vd, Gd, O, dOd, save, workspace=ws, stream=stream, out=grads)

    ramp_steps = ramp(step, args.ramp_ms, torch)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3
    fb = bwd_stage_flops_mfma(cfg, learned=args.learned)
    total = fb["total"]                                     # forward once + the backward stages
    tfl = total / (ms_per_step * 1e-3) / 1e12
    out = {
        "metric": "causal_polysketch_attention_fwd_bwd_tokens_per_s",
        "value": cfg["batch"] * cfg["n"] * args.steps / elapsed, "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "ramp_steps": ramp_steps,
        "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": args.workload, "pass": "train (forward with saved states + backward)",
                   "batch": cfg["batch"], "heads": cfg["heads"], "n": cfg["n"], "d": cfg["d"], "p": cfg["p"],
                   "r": cfg["r"], "b": cfg["b"], "sketch": "learned" if args.learned else "gaussian",
                   "kernel_path": "mfma_bf16"},
        "tflops": tfl,
        "roofline": {"kernel": "whole step", "bound": "mfma", "achieved": tfl, "peak": MFMA_BF16_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": tfl / MFMA_BF16_PEAK_TFLOPS, "traffic": None},
    }
    if not args.no_cpu_baseline and not args.learned:
        out["cpu_baseline"] = cpu_baseline_bwd(cfg, q, k, v, G, dO)
        out["cpu_baseline"]["sample"] += "; gradient only, the oracle's forward is inside it"
    print(json.dumps(out))


# HBM bytes of one dec_state_kernel launch at the serving shape, mid-block (rocprofv3 counters,
# FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0; see profiles/decode_serving_kernel_trace.md)
DECODE_MEASURED_TRAFFIC_BYTES = 3.13e8


def run_decode(args, psf, inputs, torch):
    """Token-by-token evaluation at serving shape: 64 sequences x 12 heads, d = 64, r = 64,
    b = 1024 (the headline per-unit shape).  The first block and the first half of the second go
    in as a prompt (psf_decode_prefill), so that the prefix state is populated and the timed steps
    sit around the middle of a block, where the in-block part of a step has its average cost."""
    import numpy as np
    cfg = dict(batch=args.decode_batch, heads=12, n=32768, d=64, p=4, r=64, b=1024, dtype="bf16", per_head=False)
    dev = torch.device("cuda:0")
    U = cfg["batch"] * cfg["heads"]
    steps_total = 2 * cfg["b"]                              # two whole blocks of tokens are drawn
    assert args.warmup + args.steps + 64 < cfg["b"], "timed steps must stay inside the second block"
    untimed = max(cfg["b"] + args.warmup, cfg["b"] + cfg["b"] // 2 - args.steps // 2)
    q, k, v = inputs.make_qkv(cfg["batch"], cfg["heads"], steps_total, cfg["d"], seed=1006, dtype=cfg["dtype"])
    G = inputs.make_sketch_matrices(cfg["heads"], cfg["d"], cfg["r"], cfg["p"], seed=0, dtype=cfg["dtype"])
    desc = psf.make_desc(cfg["batch"], cfg["heads"], cfg["n"], cfg["d"], cfg["p"], cfg["r"], cfg["b"], cfg["dtype"])
    qd, kd, vd, Gd = q.to(dev), k.to(dev), v.to(dev), G.to(dev)
    toks = [(qd[:, :, i:i + 1].contiguous(), kd[:, :, i:i + 1].contiguous(), vd[:, :, i:i + 1].contiguous())
            for i in range(steps_total)]
    state = psf.decode_new_state(desc, dev)
    o = torch.empty(cfg["batch"], cfg["heads"], 1, cfg["d"], dtype=qd.dtype, device=dev)
    stream = torch.cuda.current_stream()
    # the prompt goes in through the hand-over entry point (timed on its own), then the warm-up
    # steps one by one
    n_prompt = untimed - args.warmup
    kp, vp = kd[:, :, :n_prompt].contiguous(), vd[:, :, :n_prompt].contiguous()
    ws = psf.psf_decode_prefill(desc, kp, vp, Gd, state, stream=stream)      # once untimed (kernels load on first use)
    torch.cuda.synchronize()
    tp = time.perf_counter()
    ws = psf.psf_decode_prefill(desc, kp, vp, Gd, state, stream=stream)
    torch.cuda.synchronize()
    ms_prefill = (time.perf_counter() - tp) * 1e3
    del ws, kp, vp
    pos = n_prompt
    for _ in range(args.warmup):
        psf.psf_decode_step(desc, *toks[pos], Gd, pos, state, o=o, stream=stream)
        pos += 1
    torch.cuda.synchronize()
    first_timed = pos
    t0 = time.perf_counter()
    for _ in range(args.steps):
        psf.psf_decode_step(desc, *toks[pos], Gd, pos, state, o=o, stream=stream)
        pos += 1
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_mid = elapsed / args.steps * 1e3
    # the last output against the oracle's row of the same position (one unit)
    got = o[0, 0, 0].float().cpu().numpy()
    last_timed = pos - 1
    # the step that completes the block also folds the block into the state: time it alone and
    # spread it over the b steps of a block
    while pos < steps_total - 1:
        psf.psf_decode_step(desc, *toks[pos], Gd, pos, state, o=o, stream=stream)
        pos += 1
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    psf.psf_decode_step(desc, *toks[pos], Gd, pos, state, o=o, stream=stream)
    torch.cuda.synchronize()
    ms_completion = (time.perf_counter() - t1) * 1e3
    ms_per_step = ms_mid + max(0.0, ms_completion - ms_mid) / cfg["b"]
    pos = last_timed + 1
    import oracle
    want = oracle.attn_def(q[0, 0].double().numpy(), k[0, 0].double().numpy(), v[0, 0].double().numpy(),
                           G[0].double().numpy(), cfg["p"], cfg["r"], cfg["b"], rows=[pos - 1])[0]
    assert np.abs(got - want).max() <= 2e-2, "decode output does not match the oracle"
    # bytes a step has to read: the prefix state once (r (r + 1) / 2 rows, the distinct pairs of
    # the symmetric feature grid), and the keys and values cached since the last block boundary
    # (storage type), on average over the timed positions
    mid_slot = (first_timed + pos - 1) / 2 - cfg["b"]
    esize = 2 if cfg["dtype"] == "bf16" else 4
    pairs = cfg["r"] * (cfg["r"] + 1) // 2
    # bf16 storage: the steps read the value columns of the state from its bf16 copy
    state_bytes = U * pairs * (cfg["d"] * esize + 4) + int(U * mid_slot * 2 * cfg["d"] * esize)
    achieved = state_bytes / (ms_per_step * 1e-3) / 1e9
    out = {
        "metric": "causal_polysketch_attention_decode_tokens_per_s", "value": cfg["batch"] / (ms_per_step * 1e-3),
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": cfg["dtype"], "data": "synthetic",
        "config": {"workload": "decode_b%d" % cfg["batch"], "pass": "decode", "batch": cfg["batch"], "heads": cfg["heads"],
                   "d": cfg["d"], "p": cfg["p"], "r": cfg["r"], "b": cfg["b"], "storage": cfg["dtype"],
                   "first_timed_position": first_timed, "state_bytes": psf.decode_state_bytes(desc),
                   "ms_mid_block_step": ms_mid, "ms_block_completion_step": ms_completion,
                   "prefill_tokens_per_sequence": n_prompt, "ms_prefill": ms_prefill},
        "roofline": {"kernel": "dec_state_kernel", "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": DECODE_MEASURED_TRAFFIC_BYTES if cfg["batch"] == 64 else None,
                     "note": "whole step time (the step is this one kernel, plus the block fold spread over "
                             "the block) against the bytes of the prefix states and of the block cache, each "
                             "read once per step; traffic: FETCH_SIZE + WRITE_SIZE counters of the kernel "
                             "averaged over the mid-block positions (profiles/decode_serving_kernel_trace.md)"},
    }
    if not args.no_cpu_baseline:
        cores = min(os.cpu_count() or 1, 16)
        nrow = 64                                              # rows of one unit at the timed positions
        rows = list(range(first_timed, first_timed + nrow))
        t0 = time.perf_counter()
        oracle.attn_def(q[0, 0].double().numpy(), k[0, 0].double().numpy(), v[0, 0].double().numpy(),
                        G[0].double().numpy(), cfg["p"], cfg["r"], cfg["b"], rows=rows)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": nrow / dt * cores / cfg["heads"], "unit": "tokens/s", "cores": 1, "kind": "oracle",
                               "sample": "%d rows (positions %d..) of one unit by the float64 definition on one core, "
                                         "including the sketches of two blocks; value scaled to %d cores / %d heads "
                                         "per token" % (nrow, first_timed, cores, cfg["heads"]),
                               "seconds_measured": dt}
    print(json.dumps(out))


def ramp(step, ramp_ms, torch):
    """Runs `step` untimed until ramp_ms of wall time have passed; returns the count."""
    count = 0
    t0 = time.perf_counter()
    while (time.perf_counter() - t0) * 1e3 < ramp_ms:
        for _ in range(8):
            step()
        torch.cuda.synchronize()
        count += 8
    return count


def event_times(step, steps, torch, stream):
    """Sorted per-step milliseconds of `steps` calls, each between two events on `stream`."""
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    ev[0].record(stream)
    for i in range(steps):
        step()
        ev[i + 1].record(stream)
    torch.cuda.synchronize()
    return sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(steps))


def context_peaks(psf, torch, stream):
    """What this GPU sustains on two plain loops, measured in this run (context for the roofline
    fractions, which keep the published peaks as divisors): a pure bf16 MFMA loop on all compute
    units and a 256 MiB device-to-device copy (read + write bytes)."""
    dev = torch.device("cuda:0")
    wgs, iters = 2048, 4096
    sink = torch.empty(wgs * 256, dtype=torch.float32, device=dev)
    src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).fill_(1)
    dst = torch.empty_like(src)
    best = {"mfma": 0.0, "copy": 0.0}
    for _ in range(3):
        e0, e1, e2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
        e0.record(stream)
        flops = psf.psf_probe_mfma_loop(wgs, iters, sink, stream=stream)
        e1.record(stream)
        dst.copy_(src)
        e2.record(stream)
        torch.cuda.synchronize()
        best["mfma"] = max(best["mfma"], flops / (e0.elapsed_time(e1) * 1e-3) / 1e12)
        best["copy"] = max(best["copy"], 2 * src.numel() / (e1.elapsed_time(e2) * 1e-3) / 1e9)
    return {"mfma_bf16_loop_tflops": best["mfma"], "published_mfma_bf16_tflops": MFMA_BF16_PEAK_TFLOPS,
            "device_copy_gbs": best["copy"], "published_hbm_gbs": HBM_PEAK_GBS,
            "note": "best of 3; the MFMA loop holds the chip at full matrix load for ~10 ms, where its clock "
                    "settles below the boost clock the published peak assumes"}


def cpu_baseline(cfg, q, k, v, G, rows_per_unit=16384):
    """The float64 oracle, as it stands, on a bounded sample: `cores` units, a uniform random
    sample of rows of each.  The full-unit time is estimated as sketch time + row time * n/rows
    (row cost grows with the row index; a uniform sample is unbiased for the sum)."""
    import numpy as np
    import oracle
    cores = min(os.cpu_count() or 1, 16)
    U = cfg["batch"] * cfg["heads"]
    units = min(cores, U)
    n = cfg["n"]
    sel = [(i // cfg["heads"], i % cfg["heads"]) for i in range(units)]
    f64 = lambda t: np.stack([t[bi, h].double().numpy() for bi, h in sel])[None]   # [1, units, n, d]
    Q, K, V = f64(q), f64(k), f64(v)
    Gs = G.double().numpy()
    Gs = Gs[[h for _, h in sel]] if Gs.shape[0] > 1 else Gs
    rng = np.random.default_rng(0)
    rows = np.sort(rng.choice(n, size=min(rows_per_unit, n), replace=False))
    t0 = time.perf_counter()
    _, threads = oracle.attn_def_batch(Q, K, V, Gs, cfg["p"], cfg["r"], cfg["b"], rows=[0], max_threads=cores)
    t_sketch = time.perf_counter() - t0
    t0 = time.perf_counter()
    oracle.attn_def_batch(Q, K, V, Gs, cfg["p"], cfg["r"], cfg["b"], rows=rows, max_threads=cores)
    t_all = time.perf_counter() - t0
    t_rows = max(t_all - t_sketch, 1e-9)
    est_full = t_sketch + t_rows * n / len(rows)
    return {"value": units * n / est_full, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": "%d units x %d uniformly sampled rows of n=%d (float64 definition, O(n^2)); "
                      "full-unit time estimated as sketch %.2fs + rows %.2fs * n/rows" %
                      (units, len(rows), n, t_sketch, t_rows),
            "seconds_measured": t_sketch + t_all}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default=None,
                    help="config1|config2|config3|config5|sweep_n.._r.._b.. (default config3; config2 with --pass bwd)")
    ap.add_argument("--pass", dest="which", default="fwd", choices=["fwd", "bwd", "train", "decode"],
                    help="fwd: psf_causal_attn_fwd (the headline); bwd: psf_causal_attn_bwd; train: forward "
                         "that keeps its states + backward from them; decode: psf_decode_step at a fixed "
                         "serving shape")
    ap.add_argument("--local-sketch", action="store_true",
                    help="in-block weights from the sketches ((L R^T)^2, Section 3.1) instead of exact ones")
    ap.add_argument("--noncausal", action="store_true",
                    help="forward pass without the causal mask (psf_noncausal_attn_fwd)")
    ap.add_argument("--learned", action="store_true",
                    help="forward pass with learned sketches (Algorithm 2) instead of Gaussian ones")
    ap.add_argument("--degree", type=int, default=None, choices=[2, 4, 8],
                    help="degree p of the polynomial in place of the workload's (a variant of the workload, "
                         "not the quoted configuration)")
    ap.add_argument("--decode-batch", type=int, default=64,
                    help="sequences decoded together by --pass decode (12 heads each)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-context-peaks", action="store_true",
                    help="skip the MFMA-loop and device-copy measurements printed as context")
    ap.add_argument("--ramp-ms", type=float, default=400.0,
                    help="untimed steps run for this long before the warm-up steps, so that the clock has "
                         "settled (reported as ramp_steps; 0 disables)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also issue one 256 MiB device copy, so that a counter run can scale "
                         "FETCH_SIZE / WRITE_SIZE by a transfer of known size")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (units = batch x heads would shard with "
                 "no communication); run with --gpus 1")

    import torch
    from paper_2310_01655_amd import binding as psf
    from paper_2310_01655_amd import inputs

    if args.which == "decode":
        assert torch.cuda.is_available(), "bench.py needs a GPU"
        run_decode(args, psf, inputs, torch)
        return
    wl = workloads()
    if args.workload is None:
        args.workload = "config3"
    if args.workload not in wl:
        sys.exit("unknown workload %s; choose from %s" % (args.workload, ", ".join(sorted(wl))))
    cfg = dict(wl[args.workload])
    if args.degree is not None:
        cfg["p"] = args.degree
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    idx = int(args.workload[6:]) if args.workload.startswith("config") else 4
    q, k, v = inputs.make_qkv(cfg["batch"], cfg["heads"], cfg["n"], cfg["d"], seed=1000 + idx,
                              dist=cfg["dist"], dtype=cfg["dtype"])
    if args.learned:
        G = inputs.make_learned_params(cfg["heads"], cfg["d"], cfg["r"], cfg["p"], per_head=cfg["per_head"],
                                       seed=0, dtype=cfg["dtype"])
    else:
        G = inputs.make_sketch_matrices(cfg["heads"], cfg["d"], cfg["r"], cfg["p"], per_head=cfg["per_head"],
                                        seed=0, dtype=cfg["dtype"])
    if args.which == "bwd":
        run_backward(args, cfg, psf, inputs, torch, q, k, v, G, idx)
        return
    if args.which == "train":
        run_train(args, cfg, psf, inputs, torch, q, k, v, G, idx)
        return
    desc = psf.make_desc(cfg["batch"], cfg["heads"], cfg["n"], cfg["d"], cfg["p"], cfg["r"], cfg["b"],
                         cfg["dtype"], per_head=cfg["per_head"], learned=args.learned,
                         local=psf.LOCAL_SKETCH if args.local_sketch else psf.LOCAL_EXACT)
    path = psf.kernel_path(desc)
    qd, kd, vd, Gd = q.to(dev), k.to(dev), v.to(dev), G.to(dev)
    O = torch.empty_like(vd)
    ws = psf.alloc_noncausal_workspace(desc, dev) if args.noncausal else psf.alloc_workspace(desc, dev)
    stream = torch.cuda.current_stream()
    fwd = psf.psf_noncausal_attn_fwd if args.noncausal else psf.psf_causal_attn_fwd
    fwd_timed = psf.psf_noncausal_attn_fwd_timed if args.noncausal else psf.psf_causal_attn_fwd_timed

    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    step = lambda: fwd(desc, qd, kd, vd, Gd, O=O, workspace=ws, stream=stream)
    # Untimed ramp: the GPU clock takes a few hundred milliseconds of load to settle after the
    # idle time of start-up (uploads, allocation); the same steps, counted and reported.
    ramp_steps = ramp(step, args.ramp_ms, torch)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3
    tokens = cfg["batch"] * cfg["n"]
    # the same K steps once more, each bracketed by events on the launch stream: median
    per_step = event_times(step, args.steps, torch, stream)

    # per-kernel durations: HIP events recorded by the library on the launch stream
    reps = max(3, min(args.steps, 10))
    acc = {}
    for _ in range(reps):
        _, st = fwd_timed(desc, qd, kd, vd, Gd, O=O, workspace=ws, stream=stream)
        for nm, ms in st.items():
            acc[nm] = acc.get(nm, 0.0) + ms / reps
    fl = stage_flops(cfg, learned=args.learned, noncausal=args.noncausal,
                     local_sketch=args.local_sketch) if path == 1 else None
    beside = 0 if args.noncausal else psf.fwd_beside_states(desc)
    if fl and beside & 1:
        # the launch of the state kernel also ran the in-block part of the output (and the query
        # sketch): count those flops where their time is
        U, n, d, b, r = cfg["batch"] * cfg["heads"], cfg["n"], cfg["d"], cfg["b"], cfg["r"]
        moved = U * n * (b + 1) * (2 * d + 1)
        fl["output"] -= moved
        fl["block_states_scan"] += moved
        if beside & 2:
            q_sketch = U * 4 * n * d * r
            fl["sketch_and_layouts"] -= q_sketch
            fl["block_states_scan"] += q_sketch
    out = {
        "metric": ("noncausal" if args.noncausal else "causal") + "_polysketch_attention_fwd_tokens_per_s",
        "value": tokens * args.steps / elapsed,
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "ms_per_step_median": per_step[len(per_step) // 2],
        "ms_per_step_min": per_step[0], "ramp_steps": ramp_steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if path == 1 else "f32", "data": "synthetic",
        "config": {"workload": args.workload, "sketch": "learned" if args.learned else "gaussian",
                   "mask": "none" if args.noncausal else "causal",
                   "in_block": "sketch" if args.local_sketch else "exact", "batch": cfg["batch"], "heads": cfg["heads"], "n": cfg["n"],
                   "d": cfg["d"], "p": cfg["p"], "r": cfg["r"], "b": cfg["b"],
                   "kernel_path": "mfma_bf16" if path == 1 else "general_fp32"},
        "stage_ms": {nm: round(ms, 4) for nm, ms in acc.items()},
    }
    if beside & 1:
        out["stage_note"] = ("block_states_scan = one launch: state kernel + in-block part of the output + denominator "
                             "scan" + (" + query sketch" if beside & 2 else "") + "; output = cross-block part + division")
    if fl:
        out["tflops"] = fl["total"] / (ms_per_step * 1e-3) / 1e12
        out["pct_mfma_peak"] = 100.0 * out["tflops"] / MFMA_BF16_PEAK_TFLOPS
        dom = max((nm for nm in acc if nm in fl), key=lambda nm: acc[nm])
        # The event-timed calls wait for the stream after every call, and the kernels of a call
        # that starts on an idle GPU run a few per cent faster than in the back-to-back steps of
        # the timed region (their sum is below the step time although nothing lies between
        # them): the stage times are stretched to add up to the measured step.
        stretch = max(1.0, ms_per_step / sum(acc.values()))
        achieved = fl[dom] / (acc[dom] * stretch * 1e-3) / 1e12
        kernel_of = {"sketch_and_layouts": "k_prep / k_sketch", "block_states_scan": "k_state", "output": "k_out"}
        if beside & 1:
            kernel_of.update({"block_states_scan": "k_state_and_in_block", "output": "k_out (cross-block part)"})
        out["roofline"] = {"kernel": dom, "kernel_name": kernel_of.get(dom, dom), "bound": "mfma", "achieved": achieved,
                           "duration_ms": acc[dom] * stretch, "stage_stretch": stretch,
                           "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                           "frac": achieved / MFMA_BF16_PEAK_TFLOPS,
                           "traffic": None if (args.noncausal or args.learned or args.local_sketch)
                           else MEASURED_TRAFFIC_BYTES.get((args.workload, dom)),
                           "per_stage_tflops": {nm: fl[nm] / (acc[nm] * stretch * 1e-3) / 1e12
                                                for nm in acc if nm in fl and acc[nm] > 0.02}}
    elif cfg["p"] == 4 and not args.learned:
        # general fp32 kernels (plain vector arithmetic): the whole step against the fp32 vector peak
        total = stage_flops(cfg, noncausal=args.noncausal, local_sketch=args.local_sketch)["total"]
        achieved = total / (ms_per_step * 1e-3) / 1e12
        out["tflops"] = achieved
        out["roofline"] = {"kernel": "whole step", "bound": "alu", "achieved": achieved,
                           "peak": FP32_VALU_PEAK_TFLOPS, "unit": "TFLOP/s",
                           "frac": achieved / FP32_VALU_PEAK_TFLOPS, "traffic": None}
    if not args.no_context_peaks:
        out["context_peaks"] = context_peaks(psf, torch, stream)
    if not args.no_cpu_baseline and not args.learned and not args.local_sketch:   # oracle drivers used here: Gaussian sketches, exact in-block
        out["cpu_baseline"] = cpu_baseline_noncausal(cfg, q, k, v, G) if args.noncausal else cpu_baseline(cfg, q, k, v, G)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
