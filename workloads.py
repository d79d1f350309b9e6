"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module holds none of the method's arithmetic: it only draws per-batch gradients, the
projection vector f, the Byzantine node set, and overwrites rows of the received matrix with
attack vectors.  It serves both the HIP path and the CPU oracle (each gets the same tensors,
copied, never regenerated).  Everything is torch so it runs on the GPU at full size and on
the CPU for small cases.

The five named configurations are the benchmark's (shape, dtype, value distribution and
attack of each); X1 is the shape of the paper's own cluster experiment (Sec. 4 and the
experimental-details appendix: P = 100, s = 5, r_c = 10, five groups of twenty, ResNet-18-sized d).
Gradient values stand in for ResNet-18 / ResNet-50 / GPT-2-small gradients: only d, dtype
and rough scale are taken from those models.  "N(a, b)" is read with b as the variance.
"""
import math

import torch

CONFIGS = {
    # name: P, s, m, d, gradient dtype, value recipe, attack recipe
    "C1": dict(P=7, s=1, m=1, d=4096, dtype="f32", dist="normal", sigma=0.1, attack="noise100"),
    "C2": dict(P=15, s=1, m=2, d=11_200_000, dtype="f32", dist="normal", sigma=0.01, attack="flip10"),
    "C3": dict(P=31, s=2, m=2, d=25_600_000, dtype="f32", dist="shared_mean", sigma=0.01,
               mu_sigma=math.sqrt(1e-3), attack="alie"),
    "C4": dict(P=63, s=3, m=4, d=124_000_000, dtype="f32", dist="normal", sigma=0.01, attack="collude50"),
    "C5": dict(P=100, s=5, m=4, d=124_000_000, dtype="bf16", dist="student3", sigma=1e-3, attack="mix"),
    "X1": dict(P=100, s=5, m=10, d=11_173_960, dtype="f32", dist="normal", sigma=0.01, attack="paper"),
}
CONFIG_INDEX = {"C1": 1, "C2": 2, "C3": 3, "C4": 4, "C5": 5, "X1": 6}


def seeds(name):
    c = CONFIG_INDEX[name]
    return dict(G=1000 + c, f=2000 + c, byz=3000 + c, attack=4000 + c)


def _gen(device, seed):
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def make_gradients(cfg, device, seed, d=None):
    """G: [P, d] in the config's dtype, drawn row by row (bounded temporaries)."""
    P = cfg["P"]
    d = cfg["d"] if d is None else d
    dtype = torch.bfloat16 if cfg["dtype"] == "bf16" else torch.float32
    gen = _gen(device, seed)
    G = torch.empty((P, d), dtype=dtype, device=device)
    mu = None
    if cfg["dist"] == "shared_mean":
        mu = torch.randn(d, generator=gen, device=device, dtype=torch.float32) * cfg["mu_sigma"]
    for k in range(P):
        if cfg["dist"] in ("normal", "shared_mean"):
            row = torch.randn(d, generator=gen, device=device, dtype=torch.float32) * cfg["sigma"]
            if mu is not None:
                row += mu
        elif cfg["dist"] == "student3":
            # Student-t with 3 degrees of freedom: z / sqrt(chi2_3 / 3)
            z = torch.randn(d, generator=gen, device=device, dtype=torch.float32)
            c = torch.randn(3, d, generator=gen, device=device, dtype=torch.float32).square_().sum(0)
            row = z / torch.sqrt(c / 3.0) * cfg["sigma"]
            del z, c
        else:
            raise ValueError(cfg["dist"])
        G[k] = row.to(dtype)
        del row
    return G


def make_projection(d_c, device, seed):
    """f: d_c i.i.d. N(1, 1) values, fp32 (Sec. 3.4, definition of phi)."""
    return 1.0 + torch.randn(d_c, generator=_gen(device, seed), device=device, dtype=torch.float32)


def pick_byzantine(P, count, seed, within=None):
    """`count` distinct node indices, ascending; `within` restricts the draw to a list of nodes."""
    gen = _gen("cpu", seed)
    pool = list(range(P)) if within is None else list(within)
    perm = torch.randperm(len(pool), generator=gen).tolist()
    return sorted(pool[i] for i in perm[:count])


def _honest_stats(Z, byz, block=1 << 22):
    """Per-coordinate mean and (unbiased) std over the rows not in `byz`, computed in column blocks."""
    P, n = Z.shape
    hon = [j for j in range(P) if j not in set(byz)]
    idx = torch.tensor(hon, device=Z.device)
    mean = torch.empty(n, dtype=torch.float32, device=Z.device)
    std = torch.empty(n, dtype=torch.float32, device=Z.device)
    for c0 in range(0, n, block):
        blk = Z[:, c0:c0 + block].index_select(0, idx).float()
        mean[c0:c0 + block] = blk.mean(0)
        std[c0:c0 + block] = blk.std(0)
        del blk
    return mean, std, hon


def apply_attack(R, byz, kind, seed):
    """Overwrite rows `byz` of R (which holds the honest messages Z on entry) in place."""
    if not byz:
        return R
    dev = R.device
    n = R.shape[1]
    gen = _gen(dev, seed)
    stats = None
    shared = None
    for t, j in enumerate(byz):
        k = kind
        if kind == "mix":
            k = ("flip10", "noise100", "alie")[t % 3]
        if kind == "paper":
            k = ("flip100", "const100")[t % 2]
        if k == "flip10":                      # sign-flipped honest message x 10
            R[j] *= -10.0
        elif k == "flip100":                   # the paper's reverse-gradient attack (kappa = -100)
            R[j] *= -100.0
        elif k == "const100":                  # the paper's constant attack (c = -100)
            R[j].fill_(-100.0)
        elif k == "noise100":                  # Gaussian noise, 100 x the honest message's std
            sd = float(R[j].float().std()) if n > 1 else 1.0
            R[j] = torch.randn(n, generator=gen, device=dev, dtype=torch.float32) * (100.0 * sd)
        elif k == "alie":                      # mean - 1.5 std of the honest messages, per coordinate
            if stats is None:
                stats = _honest_stats(R, byz)
            R[j] = stats[0] - 1.5 * stats[1]
        elif k == "collude50":                 # one shared random vector, norm 50 x mean honest-row norm
            if shared is None:
                hon = [i for i in range(R.shape[0]) if i not in set(byz)]
                norms = torch.stack([R[i].float().norm() for i in hon])
                v = torch.randn(n, generator=gen, device=dev, dtype=torch.float32)
                shared = v * (50.0 * float(norms.mean()) / float(v.norm()))
            R[j] = shared
        elif k == "nan":
            R[j].fill_(float("nan"))
        elif k == "inf":
            R[j, ::2] = float("inf")
        elif k == "huge":
            R[j].fill_(3.0e38)
        else:
            raise ValueError(k)
    return R
