"""GPU parity of the locator phi against BRUTE FORCE (the subset enumeration of the sparse-recovery appendix) and the
planted set, on single groups of the benchmark's and the paper's shapes with all corrupted nodes in the group -
including the rounds in which the order of the locator's roots alone does not name the corrupted nodes.
The received matrix is the oracle's (seeded, fp32 as on the wire); the HIP path projects and locates."""
import numpy as np
import pytest
import torch

import paper_2110_01595_amd as solon
from locator_rounds import GROUP_SHAPES, RECIPES, mixed_strength_projections, one_group_inputs
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
    """Both ways the locator wavefront gets the orthonormal polynomials of its consistency test - from the table a plan holds, and
    rebuilt in the call (what it does anyway when a point dropped out as non-finite, or without a plan workspace) - name the
    planted set, as brute force does."""
    wrong = []
    try:
        for n in range(48):
            base, attack = RECIPES[n % len(RECIPES)]
            n_byz = s if (n // len(RECIPES)) % 2 == 0 else (n // (2 * len(RECIPES))) % (s + 1)
            print("round", base, attack, (P, s, m), "seed", n, "corrupted", n_byz, flush=True)
            plan, R, f, byz = one_group_inputs(base, attack, P, s, m, 512 * m, n, n_byz)
            V_bf = oracle_located(plan, so.project(R, f), "bruteforce_stacked")
            for table in (1, 0):
                solon.solon_tune("solve_basis_table", table)
                V, _ = hip_located(plan, R, f)
                if not (V == V_bf == byz):
                    wrong.append((n, base, byz, V, V_bf, table))
    finally:
        solon.solon_tune("solve_basis_table", 1)
    assert not wrong, wrong


def test_more_than_s_corruptions_end_the_search_with_an_error():
    for n in range(4):
        plan, R, f, _ = one_group_inputs("X1", "paper", 11, 3, 4, 1024, n, 4)
        V, _ = hip_located(plan, R, f)
        assert V == oracle_located(plan, so.project(R, f), "bruteforce") == "error %d" % so.E_DECODE


def is_explanation(plan, rho, V):
    """Do the nodes outside V lie within tau of one polynomial of degree m - 1, and is V no larger than s?"""
    if not isinstance(V, list) or len(V) > plan.s:
        return False
    wg = plan.w[plan.nodes[0]].astype(np.float64)
    flagged, _, _ = so._fit_and_test(wg, rho / so._scale(rho), set(V), plan.m, so.TAU)
    return set(flagged) <= set(V)


@pytest.mark.parametrize("P,s,m", [(20, 5, 10), (14, 5, 4), (15, 5, 4)])
def test_solve_on_projections_with_corruptions_of_very_different_strength(P, s, m):
    """The locator wavefront alone, on projections handed to it exactly: with one column (d = m, f = 1) the projection of
    node i IS the single entry of its row, so R[i][0] = rho_i feeds the solve any rho.  300 rounds per shape with s
    corruptions whose strengths span up to five decades, so that weakly corrupted nodes fall behind honest ones in the
    order of the locator's roots and the widened search is needed.  The reference is the enumeration of ALL smallest
    explaining sets.  Where every planted deviation is above 1000 tau and the planted set is the one smallest explanation
    - Lemma 1's case - the HIP path and the oracle's phi must return exactly it.  Below that the threshold itself is
    ambiguous (a deviation of some hundred tau on an end node of a 20-node group at m = 10 can be absorbed by leaving out
    its neighbour instead; deviations of a few tau by leaving out fewer nodes): any set that explains the data is a
    correct answer, and the HIP path's must be one."""
    recipes = (["big", 3.0, 1.0, 0.5, 0.3], ["big", "big", 1.0, 0.3, 0.3], [10.0, 3.0, 1.0, 0.3, 0.3],
               ["big", 1e-1, 1e-1, 1e-1, 1e-1], ["big", "big", 1e-2, 1e-2, 1e-3])
    hplan = solon.Plan(P, s, m, m)                                    # d = m: one chunk, one column
    f = torch.ones(1, dtype=torch.float32, device=DEV)
    clear = 0
    for r, deltas in enumerate(recipes):
        for seed in range(60):
            plan, rho, byz, margin = mixed_strength_projections(P, s, m, deltas, 1000 * r + seed)
            R = torch.from_numpy(rho.astype(np.float32).reshape(P, 1)).to(DEV)
            try:
                V, rho_gpu = solon.solon_locate(hplan, R, f, want_rho=True)
                assert np.array_equal(rho_gpu, rho)
            except solon.SolonError as e:
                V = "error %d" % e.code
            V_ref = oracle_located(plan, rho, "bw")
            valid = so.explanations(plan, rho, 0)
            if margin >= 1000.0 and valid == [byz]:
                clear += 1
                assert V == V_ref == byz, (deltas, seed, V, V_ref, byz)
            elif valid:
                assert is_explanation(plan, rho, V) and is_explanation(plan, rho, V_ref), (deltas, seed, V, V_ref, valid)
            else:
                assert V == V_ref == "error %d" % so.E_DECODE
    print("rounds with one smallest explanation, the planted set, and every deviation above 1000 tau:", clear, "of", 60 * len(recipes), flush=True)
    assert clear >= 80
