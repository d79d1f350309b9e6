"""Repetition code (m = 1): majority-vote decoding as an independent check of the locate + decode path.

CPU part pins the oracle's majority decoder against a literal Boyer-Moore vote written out per coordinate and
against the general decoder; the GPU part checks solon_decode_majority against the oracle (values and dissenting
nodes) and against solon_locate + solon_decode on the same received matrix."""
import numpy as np
import pytest

from oracle import solon_oracle as so


def boyer_moore(items):
    """The streaming majority vote as the paper's appendix lists it."""
    cand, count = None, 0
    for it in items:
        if count == 0:
            cand, count = it, 1
        elif cand == it:
            count += 1
        else:
            count -= 1
    return cand


@pytest.mark.parametrize("P,s", [(7, 1), (15, 2), (23, 3)])
def test_oracle_majority_equals_streaming_vote_and_general_decoder(P, s):
    rng = np.random.default_rng(P)
    plan = so.make_plan(P, s, 1)
    d = 97
    G = (rng.standard_normal((P, d)) * 0.01).astype(np.float32)
    Z = so.encode(plan, G).astype(np.float32).astype(np.float64)
    bad = sorted(int(plan.nodes[g][i]) for g in range(plan.q) for i in rng.choice(len(plan.nodes[g]), size=s, replace=False))
    R = Z.copy()
    for t, j in enumerate(bad):
        R[j] = [Z[j] * -10.0, rng.standard_normal(d), np.full(d, np.nan)][t % 3]
    u, V = so.decode_majority(plan, R, d)
    assert V == bad
    expect = np.zeros(d)
    for g in range(plan.q):
        for c in range(d):
            expect[c] += boyer_moore([float(R[j, c]) for j in plan.nodes[g]])
    assert np.array_equal(u, expect)
    f = 1.0 + rng.standard_normal(d)
    assert so.locate(plan, so.project(R, f)) == bad
    assert so.rel_l2(so.decode(plan, R, bad, d), u) < 1e-12
    assert so.rel_l2(u, so.plain_sum(G)) < 1e-6


def test_oracle_majority_reports_missing_majority():
    plan = so.make_plan(7, 1, 1)                        # groups of 4 and 3
    R = np.arange(7 * 5, dtype=np.float64).reshape(7, 5)   # all rows differ: no majority anywhere
    with pytest.raises(so.OracleError) as e:
        so.decode_majority(plan, R, 5)
    assert e.value.code == so.E_DECODE
    with pytest.raises(so.OracleError):
        so.decode_majority(so.make_plan(8, 1, 2), R, 5)


@pytest.mark.gpu
@pytest.mark.parametrize("P,s,d,pad", [(7, 1, 4096, 0), (7, 1, 70_001, 0), (15, 2, 40_004, 0), (63, 3, 30_000, 2), (23, 3, 5, 0),
                                         (40, 9, 8192, 0), (100, 5, 20_000, 0)])
def test_gpu_majority_matches_oracle_and_general_path(P, s, d, pad):
    import torch

    import paper_2110_01595_amd as solon
    import workloads

    dev = torch.device("cuda:0")
    print("majority case", dict(P=P, s=s, d=d, pad=pad), flush=True)
    plan = solon.Plan(P, s, 1, d)
    oplan = so.make_plan(P, s, 1)
    cfg = dict(P=P, d=d, dtype="f32", dist="normal", sigma=0.1)
    G = workloads.make_gradients(cfg, dev, 31 + P, d=d)
    Zfull = torch.zeros((P, d + pad), dtype=torch.float32, device=dev)
    Z = Zfull[:, :d]
    solon.solon_encode(plan, G, Z)
    byz = workloads.pick_byzantine(P, s, 32 + P)
    R = workloads.apply_attack(Zfull.clone()[:, :d], byz, "mix", 33)
    u = torch.full((d + 3,), 5.0, dtype=torch.float32, device=dev)
    V = solon.solon_decode_majority(plan, R, u[:d])
    assert solon.solon_decode_status(plan) == solon.SOLON_OK
    assert bool((u[d:] == 5.0).all())
    # the persistent row-synchronous kernel forced onto this small input (two blocks: several ragged rounds; the full
    # grid: most lanes past the end of the rows) gives the same bits and the same set wherever it applies
    for grid in (2, 0):
        solon.solon_tune("majority_rows", 1)
        solon.solon_tune("majority_rows_grid", grid)
        try:
            u_rows = torch.full((d + 3,), 5.0, dtype=torch.float32, device=dev)
            V_rows = solon.solon_decode_majority(plan, R, u_rows[:d])
            assert solon.solon_decode_status(plan) == solon.SOLON_OK
        finally:
            solon.solon_tune("majority_rows", -1)
            solon.solon_tune("majority_rows_grid", 0)
        assert V_rows == V
        assert torch.equal(u_rows, u)
    u_ref, V_ref = so.decode_majority(oplan, R.cpu().numpy(), d)
    assert V == V_ref == byz
    assert so.rel_l2(u[:d].cpu().numpy(), u_ref) <= 1e-6
    # the general path on the same R gives the same set and the same aggregate
    f = workloads.make_projection(d, dev, 34)
    V2, _ = solon.solon_locate(plan, R, f)
    u2 = torch.empty(d, dtype=torch.float32, device=dev)
    solon.solon_decode(plan, R, u2)
    assert V2 == V
    assert so.rel_l2(u2.cpu().numpy(), u[:d].cpu().numpy()) <= 1e-6
    assert so.rel_l2(u[:d].cpu().numpy(), so.plain_sum(G.cpu().numpy())) <= 1e-6


@pytest.mark.gpu
def test_gpu_majority_error_paths():
    import torch

    import paper_2110_01595_amd as solon

    dev = torch.device("cuda:0")
    plan2 = solon.Plan(8, 1, 2, 64)
    with pytest.raises(solon.SolonError) as e:
        solon.solon_decode_majority(plan2, torch.zeros((8, 32), device=dev), torch.zeros(64, device=dev))
    assert e.value.code == solon.SOLON_E_INVAL
    plan = solon.Plan(7, 1, 1, 16)
    R = torch.arange(7 * 16, dtype=torch.float32, device=dev).reshape(7, 16)       # no two rows agree
    with pytest.raises(solon.SolonError) as e:
        solon.solon_decode_majority(plan, R, torch.zeros(16, device=dev))
    assert e.value.code == solon.SOLON_E_DECODE
