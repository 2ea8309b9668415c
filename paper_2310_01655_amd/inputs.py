"""Seeded synthetic inputs shared by the CPU oracle's tests and the GPU path.

This module holds none of the method's arithmetic: it only draws Q, K, V and the
Gaussian sketch matrices, normalises Q/K rows to unit L2 norm (the stand-in for the
layer normalisation the paper applies before the kernel, Section 2.1) and rounds
everything to the storage dtype.  The very same tensors go to both sides.

Shapes follow the paper's GPT-2-small-style workloads (head size 64, block size
1024, sketch sizes 32 and 64, batches of 2^20 tokens; Section 4 and Appendix G);
the values are iid draws standing in for activations of models trained on PG-19,
Wiki-40B and C4, which are not available here.
"""
import torch

# p: degree, r: sketch size, b: block size of the lower-triangular algorithm
CONFIGS = {
    1: dict(batch=1, heads=1, n=1024, d=64, p=4, r=16, b=128, dtype="f32",
            per_head=False, dist="normal"),
    2: dict(batch=8, heads=12, n=4096, d=64, p=4, r=32, b=256, dtype="bf16",
            per_head=True, dist="normal"),
    3: dict(batch=2, heads=12, n=32768, d=64, p=4, r=64, b=1024, dtype="bf16",
            per_head=False, dist="normal"),
    5: dict(batch=1, heads=16, n=16384, d=128, p=8, r=64, b=512, dtype="bf16",
            per_head=False, dist="normal"),
}


def sweep_configs():
    """Config 4: 2^20 tokens per step, every (n, r, b) of the sweep."""
    out = []
    for n in (8192, 16384, 32768, 65536):
        for r in (32, 64):
            for b in (256, 512, 1024):
                out.append(dict(batch=(1 << 20) // n, heads=12, n=n, d=64, p=4, r=r, b=b,
                                dtype="bf16", per_head=False, dist="normal"))
    return out


def torch_dtype(name):
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


def num_sketch_matrices(p):
    """(count of d x r matrices, count of r x r matrices) for degree p (Theorem 1.1)."""
    half = p // 2
    return (half if half >= 2 else 0), (half - 2 if half >= 4 else 0)


def g_len(d, r, p):
    n_first, n_inner = num_sketch_matrices(p)
    return n_first * d * r + n_inner * r * r


def make_qkv(batch, heads, n, d, dv=None, seed=0, dist="normal", dtype="f32"):
    """Q, K, V as CPU tensors [batch, heads, n, d|dv] in the storage dtype.

    dist == "normal": entries N(0,1).  dist == "student_t3": Q and K entries are
    Student-t with 3 degrees of freedom (V stays normal).  Q and K rows are then
    scaled to unit L2 norm."""
    dv = d if dv is None else dv
    g = torch.Generator(device="cpu")
    g.manual_seed(int(seed))

    def draw(last):
        z = torch.randn(batch, heads, n, last, generator=g, dtype=torch.float32)
        if dist == "student_t3" and last == d:
            chi = torch.randn(batch, heads, n, last, 3, generator=g, dtype=torch.float32)
            z = z / torch.sqrt(chi.pow(2).sum(-1) / 3.0)
        return z

    q, k = draw(d), draw(d)
    v = torch.randn(batch, heads, n, dv, generator=g, dtype=torch.float32)
    q = q / q.norm(dim=-1, keepdim=True)
    k = k / k.norm(dim=-1, keepdim=True)
    td = torch_dtype(dtype)
    return q.to(td).contiguous(), k.to(td).contiguous(), v.to(td).contiguous()


def learned_len(d, r, p):
    """Entries of one parameter set of the learned sketch (Appendix D): p - 2 networks, each
    [g1, b1, W1 (in x 8r), g2, b2, W2 (8r x r), W3 (r x 8r), W4 (8r x r)]."""
    if p < 4:
        return 0
    net = lambda win: 2 * win + win * 8 * r + 16 * r + 24 * r * r
    return (p // 2) * net(d) + max(p // 2 - 2, 0) * net(r)


def make_learned_params(heads, d, r, p, per_head=False, seed=0, dtype="f32"):
    """Synthetic parameters of the learned sketch, [heads if per_head else 1, learned_len]:
    dense matrices N(0, 1/fan_in), layer-norm scales 1 + 0.1 N(0,1), biases 0.1 N(0,1) (random
    stand-ins for trained weights, which are not available), networks in the order the
    recursion of Algorithm 2 reaches them."""
    sets = heads if per_head else 1
    out = torch.empty(sets, max(learned_len(d, r, p), 1), dtype=torch.float32)
    widths = [d] * (p // 2) + [r] * max(p // 2 - 2, 0) if p >= 4 else []
    for h in range(sets):
        g = torch.Generator(device="cpu")
        g.manual_seed(int(seed) + 31 * h + 5)
        rn = lambda *shape: torch.randn(*shape, generator=g, dtype=torch.float32)
        pieces = []
        for win in widths:
            hid = 8 * r
            pieces += [1.0 + 0.1 * rn(win), 0.1 * rn(win), rn(win, hid) / win ** 0.5,
                       1.0 + 0.1 * rn(hid), 0.1 * rn(hid), rn(hid, r) / hid ** 0.5,
                       rn(r, hid) / r ** 0.5, rn(hid, r) / hid ** 0.5]
        if pieces:
            out[h] = torch.cat([x.reshape(-1) for x in pieces])
    return out.to(torch_dtype(dtype)).contiguous()


def make_dout(batch, heads, n, dv, seed=0, dtype="f32"):
    """dL/dO for the backward pass: entries N(0,1) (stand-in for the gradient that the layers
    after the attention send back), CPU tensor in the storage dtype."""
    g = torch.Generator(device="cpu")
    g.manual_seed(int(seed) + 7919)
    z = torch.randn(batch, heads, n, dv, generator=g, dtype=torch.float32)
    return z.to(torch_dtype(dtype)).contiguous()


def make_sketch_matrices(heads, d, r, p, per_head=False, seed=0, dtype="f32"):
    """Gaussian sketch matrices, [heads if per_head else 1, g_len(d, r, p)]; set h is
    drawn from seed + h.  Within a set: the p/2 matrices d x r, then the p/2 - 2
    matrices r x r, in the order Algorithm 1 samples them."""
    sets = heads if per_head else 1
    length = max(g_len(d, r, p), 1)
    out = torch.empty(sets, length, dtype=torch.float32)
    for h in range(sets):
        g = torch.Generator(device="cpu")
        g.manual_seed(int(seed) + h)
        out[h] = torch.randn(length, generator=g, dtype=torch.float32)
    return out.to(torch_dtype(dtype)).contiguous()


def make_config(idx, variant=None, **override):
    """Tensors for one of the numbered workloads; data seed 1000 + idx (+100 for the
    heavy-tailed variant of config 5), sketch seed 0 (+ head index when per head)."""
    cfg = dict(CONFIGS[idx])
    cfg.update(override)
    seed = 1000 + idx
    if variant == "heavy":
        cfg["dist"] = "student_t3"
        seed += 100
    q, k, v = make_qkv(cfg["batch"], cfg["heads"], cfg["n"], cfg["d"], seed=seed,
                       dist=cfg["dist"], dtype=cfg["dtype"])
    G = make_sketch_matrices(cfg["heads"], cfg["d"], cfg["r"], cfg["p"],
                             per_head=cfg["per_head"], seed=0, dtype=cfg["dtype"])
    return cfg, q, k, v, G
