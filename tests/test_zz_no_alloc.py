"""The allocation-free locate entry point (static device scratch) against solon_locate on the same inputs: the located
set and the per-group status bit for bit, the projections to 1e-12 relative (the partial sums may be tiled
differently).  Two calls in a row, the second on a smaller input, so that stale contents of the shared array would
show; then a size beyond the array's limit, which must be refused."""
import numpy as np
import pytest
import torch

import paper_2110_01595_amd as solon
import workloads

pytestmark = pytest.mark.gpu
DEV = torch.device("cuda:0")


def one_call(P, s, m, d, attack, byz, seed, group_of_node=None, group_of_batch=None, B=None, expect=solon.SOLON_OK):
    print("static locate", dict(P=P, s=s, m=m, d=d, attack=attack, byz=byz, seed=seed), flush=True)
    plan = solon.Plan(P, s, m, d, B=B, group_of_node=group_of_node, group_of_batch=group_of_batch)
    cfg = dict(P=(P if B is None else B), d=d, dtype="f32", dist="normal", sigma=0.01)
    G = workloads.make_gradients(cfg, DEV, seed, d=d)
    Z = torch.zeros((P, plan.d_c), dtype=torch.float32, device=DEV)
    solon.solon_encode(plan, G, Z)
    R = workloads.apply_attack(Z.clone(), byz, attack, seed + 1)
    f = workloads.make_projection(plan.d_c, DEV, seed + 2)
    try:
        V_ref, rho_ref = solon.solon_locate(plan, R, f, want_rho=True)
        assert expect == solon.SOLON_OK
    except solon.SolonError as e:
        assert e.code == expect
        V_ref, rho_ref = None, None
    located = torch.full((P,), 7, dtype=torch.int32, device=DEV)
    status = torch.full((plan.q,), 7, dtype=torch.int32, device=DEV)
    rho = torch.full((P,), 7.0, dtype=torch.float64, device=DEV)
    solon.solon_locate_static(plan, R, f, located, status, rho)
    torch.cuda.synchronize()
    st = status.cpu().numpy()
    if expect != solon.SOLON_OK:
        assert st.min() == expect
        return
    assert np.all(st == solon.SOLON_OK)
    assert np.flatnonzero(located.cpu().numpy()).tolist() == V_ref == sorted(byz)
    active = plan.groups() >= 0
    rho_h = rho.cpu().numpy()
    assert np.abs(rho_h[active] - rho_ref[active]).max() <= 1e-12 * np.abs(rho_ref[active]).max()
    located.fill_(7)                                   # without the optional rho output
    solon.solon_locate_static(plan, R, f, located, status)
    torch.cuda.synchronize()
    assert np.flatnonzero(located.cpu().numpy()).tolist() == V_ref


def test_static_locate_matches_solon_locate_on_two_calls_in_a_row():
    one_call(100, 5, 4, 400_000, "mix", [3, 17, 44, 45, 99], 11)          # many tiles, seven groups
    one_call(15, 1, 2, 9_001, "flip10", [7], 21)                          # then a smaller one: fewer nodes, groups, tiles
    one_call(100, 5, 10, 50_010, "paper", [0, 1, 2, 3, 4], 31)            # all five in one group of twenty
    gon = [0] * 5 + [-1] + [1] * 6                                        # an idle node stays unlocated
    one_call(12, 1, 2, 50_000, "noise100", [8], 41, group_of_node=gon, group_of_batch=[0] * 6 + [1] * 6)
    one_call(15, 1, 2, 4_096, "noise100", [0, 2], 51, expect=solon.SOLON_E_DECODE)   # two in one group, s = 1


def test_static_locate_refuses_more_nodes_than_the_array_holds():
    plan = solon.Plan(129, 1, 2, 1000)
    R = torch.zeros((129, plan.d_c), dtype=torch.float32, device=DEV)
    f = torch.ones(plan.d_c, dtype=torch.float32, device=DEV)
    located = torch.zeros(129, dtype=torch.int32, device=DEV)
    status = torch.zeros(plan.q, dtype=torch.int32, device=DEV)
    with pytest.raises(solon.SolonError) as e:
        solon.solon_locate_static(plan, R, f, located, status)
    assert e.value.code == solon.SOLON_E_INVAL and "128" in str(e.value)
