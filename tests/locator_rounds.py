"""Seeded single-group rounds for the locator tests (CPU pins and GPU parity alike): messages are the oracle's
encode of seeded gradients, rounded to fp32 as on the wire, with the corrupted nodes all in the one group."""
import numpy as np
import torch

import workloads as wl
from oracle import solon_oracle as so

GROUP_SHAPES = [(14, 5, 4), (15, 5, 4), (11, 3, 4), (20, 5, 10)]     # (r_g, s, m): one group holding all nodes
RECIPES = [("C5", "mix"), ("X1", "paper"), ("C4", "collude50"), ("pin", "mix")]


def pin_corrupt(rng, Z, rows):
    """The four-way mix of tests/test_oracle_pins.py on fp32-rounded messages."""
    R = Z.copy()
    for t, j in enumerate(rows):
        k = ("flip", "noise", "const", "fake")[t % 4]
        if k == "flip":
            R[j] = -10.0 * Z[j]
        elif k == "noise":
            R[j] = rng.standard_normal(Z.shape[1]) * 100.0 * Z[j].std()
        elif k == "const":
            R[j] = -100.0
        else:
            R[j] = Z[j] + 0.37 * np.abs(Z).max()
    return R


def one_group_inputs(base, attack, P, s, m, d, n, n_byz):
    """(plan, R, f, planted set) of one round with all corrupted nodes in the single group.  Seeds: gradients n, Byzantine set 10000 + n,
    attack 20000 + n, projection 30000 + n.  Messages are the oracle's, rounded to fp32 as on the wire."""
    plan = so.make_plan(P, s, m)
    assert plan.q == 1
    if base == "pin":
        rng = np.random.default_rng(n)
        G = (rng.standard_normal((P, d)) * 0.01).astype(np.float32)
        Z = so.encode(plan, G).astype(np.float32).astype(np.float64)
        byz = sorted(rng.choice(P, size=n_byz, replace=False).tolist())
        R = pin_corrupt(rng, Z, byz)
        f = (1.0 + rng.standard_normal(Z.shape[1])).astype(np.float32)
        return plan, R.astype(np.float32), f, byz
    cfg = dict(wl.CONFIGS[base])
    cfg.update(P=P, s=s, m=m, d=d, attack=attack)
    G = wl.make_gradients(cfg, "cpu", n)
    Z = so.encode(plan, G.float().numpy()).astype(np.float32)
    R = torch.from_numpy(Z.copy())
    byz = wl.pick_byzantine(P, n_byz, 10000 + n)
    wl.apply_attack(R, byz, attack, 20000 + n)
    f = wl.make_projection(Z.shape[1], "cpu", 30000 + n)
    return plan, R.numpy(), f.numpy(), byz




def one_group_round(base, attack, P, s, m, d, n, n_byz):
    """(plan, rho, planted set) of the same round, projected by the oracle."""
    plan, R, f, byz = one_group_inputs(base, attack, P, s, m, d, n, n_byz)
    return plan, so.project(R, f), byz


def mixed_strength_projections(P, s, m, deltas, seed):
    """Projections of one group whose s corrupted nodes differ widely in strength: node t is scaled by -100 ("big") or has
    noise of deltas[t] times its message's mean magnitude added - the recipe under which weakly corrupted nodes come late
    in the order of the locator's roots.  Returns (plan, rho, planted set, smallest planted deviation in units of tau)."""
    rng = np.random.default_rng(seed)
    plan = so.make_plan(P, s, m)
    G = (rng.standard_normal((P, 512 * m)) * 0.01).astype(np.float32)
    Z = so.encode(plan, G).astype(np.float32).astype(np.float64)
    byz = sorted(rng.choice(P, size=s, replace=False).tolist())
    R = Z.copy()
    for t, j in enumerate(byz):
        dl = deltas[t % len(deltas)]
        R[j] = -100.0 * Z[j] if dl == "big" else Z[j] + dl * np.abs(Z[j]).mean() * rng.standard_normal(Z.shape[1])
    f = (1 + rng.standard_normal(Z.shape[1])).astype(np.float32)
    rho = so.project(R, f).astype(np.float32).astype(np.float64)       # what the HIP path is handed below, exactly
    dev = np.abs(so.project(R - Z, f)) / so._scale(rho)
    return plan, rho, byz, float(min(dev[j] for j in byz)) / so.TAU
