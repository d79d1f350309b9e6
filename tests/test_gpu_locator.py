"""GPU parity of the locator phi against BRUTE FORCE (the subset enumeration of the sparse-recovery appendix) and the
planted set, on single groups of the benchmark's and the paper's shapes with all corrupted nodes in the group -
including the rounds in which the order of the locator's roots alone does not name the corrupted nodes.
The received matrix is the oracle's (seeded, fp32 as on the wire); the HIP path projects and locates."""
import numpy as np
import pytest
import torch

import paper_2110_01595_amd as solon
from locator_rounds import GROUP_SHAPES, RECIPES, one_group_inputs
from oracle import solon_oracle as so

pytestmark = pytest.mark.gpu
DEV = torch.device("cuda:0")


def hip_located(plan, R, f):
    """(V or 'error <code>', rho) from solon_locate on the oracle's R and f."""
    hplan = solon.Plan(plan.P, plan.s, plan.m, R.shape[1] * plan.m)
    Rd, fd = torch.from_numpy(R).to(DEV), torch.from_numpy(f).to(DEV)
    try:
        V, rho = solon.solon_locate(hplan, Rd, fd, want_rho=True)
    except solon.SolonError as e:
        return "error %d" % e.code, None
    return V, rho


def oracle_located(plan, rho, method):
    try:
        return so.locate(plan, rho, method)
    except so.OracleError as e:
        return "error %d" % e.code


@pytest.mark.parametrize("base,attack,P,s,m,d,seeds", [
    ("C5", "mix", 14, 5, 4, 8192, (36, 56, 74)),
    ("X1", "paper", 20, 5, 10, 8000, (50, 305, 318)),
])
def test_rounds_with_a_weak_corruption_behind_an_honest_root(base, attack, P, s, m, d, seeds):
    for n in seeds:
        print("round", base, attack, (P, s, m), "seed", n, flush=True)
        plan, R, f, byz = one_group_inputs(base, attack, P, s, m, d, n, s)
        V, rho = hip_located(plan, R, f)
        rho_ref = so.project(R, f)
        assert np.abs(rho - rho_ref).max() <= 1e-12 * (np.abs(R).astype(np.float64) @ np.abs(f)).max()
        assert V == oracle_located(plan, rho_ref, "bruteforce_stacked") == byz


@pytest.mark.parametrize("P,s,m", GROUP_SHAPES)
def test_located_set_equals_bruteforce_over_seeds(P, s, m):
    wrong = []
    for n in range(48):
        base, attack = RECIPES[n % len(RECIPES)]
        n_byz = s if (n // len(RECIPES)) % 2 == 0 else (n // (2 * len(RECIPES))) % (s + 1)
        print("round", base, attack, (P, s, m), "seed", n, "corrupted", n_byz, flush=True)
        plan, R, f, byz = one_group_inputs(base, attack, P, s, m, 512 * m, n, n_byz)
        V, _ = hip_located(plan, R, f)
        V_bf = oracle_located(plan, so.project(R, f), "bruteforce_stacked")
        if not (V == V_bf == byz):
            wrong.append((n, base, byz, V, V_bf))
    assert not wrong, wrong


def test_more_than_s_corruptions_end_the_search_with_an_error():
    for n in range(4):
        plan, R, f, _ = one_group_inputs("X1", "paper", 11, 3, 4, 1024, n, 4)
        V, _ = hip_located(plan, R, f)
        assert V == oracle_located(plan, so.project(R, f), "bruteforce") == "error %d" % so.E_DECODE
