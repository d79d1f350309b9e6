"""CPU-only checks of the C ABI: the library loads, exports every declared symbol, and its host logic
(parameter checks of Thm. 2, group table, default evaluation points) agrees with the oracle."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2110_01595_amd as solon
from oracle import solon_oracle as so

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "solon.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(solon_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = solon.lib()
    names = declared_functions()
    assert set(names) == set(solon.EXPORTS)
    for n in names:
        assert hasattr(L, n), n


def test_every_launch_shape_knob_is_documented_in_the_header():
    """solon_tune stores unknown keys silently, so a knob the sources read but the header does not name could not be found."""
    import glob

    header = open(os.path.join(ROOT, "include", "solon.h")).read()
    used = set()
    for path in glob.glob(os.path.join(ROOT, "paper_2110_01595_amd", "csrc", "*.hip")):
        used |= set(re.findall(r'solon_tuning\("([a-z_0-9]+)"', open(path).read()))
    assert used, "no knobs found: the pattern is stale"
    missing = sorted(k for k in used if '"%s"' % k not in header)
    assert not missing, missing


@pytest.mark.parametrize("r_g", list(range(1, 65)))
def test_default_points_match_oracle(r_g):
    assert np.array_equal(solon.solon_default_points(r_g), so.default_points(r_g))


@pytest.mark.parametrize("P,s,m", [(7, 1, 1), (15, 1, 2), (31, 2, 2), (63, 3, 4), (100, 5, 4), (100, 5, 10), (4, 1, 2)])
def test_plan_tables_match_oracle(P, s, m):
    plan = solon.Plan(P, s, m, d=1000)
    oplan = so.make_plan(P, s, m)
    assert plan.q == oplan.q and plan.r == oplan.r and plan.d_c == so.message_length(1000, m)
    gon = plan.groups()
    for g in range(oplan.q):
        assert np.array_equal(np.flatnonzero(gon == g), oplan.nodes[g])
    assert np.array_equal(plan.points(), oplan.w)
    assert plan.query(solon.SOLON_Q_MAX_GROUP) == max(len(n) for n in oplan.nodes)


def test_bound_and_argument_checks():
    def code(**kw):
        with pytest.raises(solon.SolonError) as e:
            solon.Plan(**kw)
        return e.value.code
    assert code(P=5, s=2, m=2, d=10) == solon.SOLON_E_BOUND                       # s > (P - m) / 2
    assert code(P=8, s=1, m=2, d=10, group_of_node=[0, 0, 0, 0, 0, 1, 1, 1]) == solon.SOLON_E_BOUND
    assert code(P=4, s=1, m=2, d=10, w=[0.5, 0.5, -0.2, 0.1]) == solon.SOLON_E_POINTS
    assert code(P=4, s=1, m=2, d=10, w=[0.5, 0.0, -0.2, 0.1]) == solon.SOLON_E_POINTS
    assert code(P=4, s=1, m=2, d=10, w=[0.5, float("nan"), -0.2, 0.1]) == solon.SOLON_E_POINTS
    assert code(P=0, s=0, m=1, d=10) == solon.SOLON_E_INVAL
    assert code(P=4, s=1, m=2, d=0) == solon.SOLON_E_INVAL
    assert code(P=4, s=-1, m=2, d=10) == solon.SOLON_E_INVAL
    assert code(P=40, s=1, m=17, d=10) == solon.SOLON_E_INVAL                     # no kernel beyond m = 16
    assert code(P=4, s=1, m=2, d=10, dtype=7) == solon.SOLON_E_INVAL
    assert code(P=4, s=1, m=2, d=10, B=5) == solon.SOLON_E_INVAL                  # B != P needs group_of_batch
    assert code(P=130, s=0, m=1, d=10, group_of_node=[0] * 130) == solon.SOLON_E_INVAL   # group above 64 nodes
    assert b"64" in solon.lib().solon_last_error()


def test_idle_nodes_and_custom_batches():
    # "change P": 10 nodes, r = 4, two groups of 4 and two idle nodes; 6 gradients split 3 + 3
    gon = [0, 0, 0, 0, 1, 1, 1, 1, -1, -1]
    plan = solon.Plan(P=10, s=1, m=2, d=64, B=6, group_of_node=gon, group_of_batch=[0, 0, 0, 1, 1, 1])
    assert plan.q == 2 and list(plan.groups()) == gon


def test_null_arguments_are_rejected_not_dereferenced():
    L = solon.lib()
    assert L.solon_plan_create(None, 4, 4, 1, 2, 10, 0, None, None, None) == solon.SOLON_E_INVAL
    assert L.solon_encode(None, None, 0, None, 0, None) == solon.SOLON_E_INVAL
    assert L.solon_locate(None, None, 0, None, None, None, None, None) == solon.SOLON_E_INVAL
    assert L.solon_decode(None, None, 0, None, 0, None, None) == solon.SOLON_E_INVAL
    assert L.solon_default_points(0, None) == solon.SOLON_E_INVAL
    v = ctypes.c_int64()
    assert L.solon_plan_query(None, 0, ctypes.byref(v)) == solon.SOLON_E_INVAL
    L.solon_plan_destroy(None)


@pytest.mark.parametrize("name,enc,loc,dec", [("C2", 1.008, 0.358, 0.179), ("C3", 4.762, 1.638, 0.614), ("C4", 39.060, 7.936, 3.472),
                                               ("C5", 37.200, 12.524, 3.968), ("X1", 4.917, 0.451, 0.268)])
def test_bench_counts_the_bytes_the_method_must_move(name, enc, loc, dec):
    """bench.py's numerators, in GB, against the figures worked out by hand from the cost analysis (Sec. 3.4, complexity of the
    encoder and decoder): every gradient read once and every message written once (P d b + P d_c 4), every message and f read
    once by the projection (P d_c 4 + d_c 4), q m rows recombined into u (q m d_c 4 + d 4).  The one-pass call moves R, f and u
    once plus the sample behind its guess."""
    import bench
    import workloads

    cfg = workloads.CONFIGS[name]
    plan = solon.Plan(cfg["P"], cfg["s"], cfg["m"], cfg["d"], dtype=solon.SOLON_BF16 if cfg["dtype"] == "bf16" else solon.SOLON_F32)
    ab = bench.algorithmic_bytes(cfg, plan)
    assert round(ab["encode"] / 1e9, 3) == enc and round(ab["locate"] / 1e9, 3) == loc and round(ab["decode"] / 1e9, 3) == dec
    assert ab["total"] == ab["encode"] + ab["locate"] + ab["decode"]
    two = bench.moved_bytes(cfg, plan, False)
    assert two["total"] == ab["total"]
    one = bench.moved_bytes(cfg, plan, True)
    saved = ab["total"] - one["total"]
    sample = (cfg["P"] + 1) * min(plan.d_c, 1 << 17) * 4
    assert saved == plan.q * cfg["m"] * plan.d_c * 4 - sample        # the second read of psi's rows, less the sample projection
