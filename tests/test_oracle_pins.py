"""CPU-only pins of the fp64 oracle against what the paper and the mathematics fix.

None of these compares the oracle with itself through the same formula: each uses a definition,
a closed form, a special case, a brute force or an explicit construction from the paper.
"""
import os
from itertools import combinations

import numpy as np
import pytest

from oracle import solon_oracle as so

SHAPES = [  # (P, s, m)   r = 2s + m; most are ragged (r does not divide P)
    (4, 1, 2), (7, 1, 1), (8, 1, 2), (15, 1, 2), (12, 2, 2), (13, 2, 2), (10, 3, 4), (21, 3, 4), (14, 5, 4), (29, 5, 4),
]


def rand_G(rng, P, d, sigma=0.01, dtype=np.float32):
    return (rng.standard_normal((P, d)) * sigma).astype(dtype)


def corrupt(rng, Z, rows, kind):
    R = Z.copy()
    for t, j in enumerate(rows):
        k = kind if kind != "mix" else ("flip", "noise", "const", "fake")[t % 4]
        if k == "flip":
            R[j] = -10.0 * Z[j]
        elif k == "noise":
            R[j] = rng.standard_normal(Z.shape[1]) * 100.0 * Z[j].std()
        elif k == "const":
            R[j] = -100.0
        elif k == "fake":                      # shifted by a fixed vector: still an arbitrary vector
            R[j] = Z[j] + 0.37 * np.abs(Z).max()
    return R


# ---------------------------------------------------------------- plan / bound (Thm. 2, corollary)
def test_group_table_reduces_to_paper_when_r_divides_P():
    plan = so.make_plan(P=100, s=5, m=10)            # the paper's own experiment: 5 groups of 20
    assert plan.q == 5 and plan.r == 20
    assert [len(n) for n in plan.nodes] == [20] * 5
    A = np.zeros((100, 100), dtype=int)              # allocation matrix of Sec. 3.4: I_q (x) 1_{r x r}
    for g in range(plan.q):
        A[np.ix_(plan.nodes[g], plan.batches[g])] = 1
    assert np.array_equal(A, np.kron(np.eye(5, dtype=int), np.ones((20, 20), dtype=int)))
    assert A.sum() / 100 == plan.r                   # redundancy ratio ||A||_0 / P


@pytest.mark.parametrize("P,s,m", SHAPES + [(63, 3, 4), (100, 5, 4), (31, 2, 2)])
def test_ragged_groups_respect_bound(P, s, m):
    plan = so.make_plan(P, s, m)
    sizes = [len(n) for n in plan.nodes]
    assert sum(sizes) == P and min(sizes) >= 2 * s + m and max(sizes) - min(sizes) <= 1
    assert sorted(sizes, reverse=True) == sizes
    for g in range(plan.q):                          # every gradient is replicated on its whole group
        assert np.array_equal(plan.nodes[g], plan.batches[g])
        wg = plan.w[plan.nodes[g]]
        assert len(set(wg.tolist())) == len(wg) and np.all(wg != 0) and np.all(np.abs(wg) < 1)


def test_bound_violations_rejected():
    with pytest.raises(so.OracleError) as e:
        so.make_plan(P=5, s=2, m=2)                  # s > (P - m)/2
    assert e.value.code == so.E_BOUND
    with pytest.raises(so.OracleError) as e:
        so.make_plan(P=8, s=1, m=2, group_of_node=[0, 0, 0, 0, 0, 1, 1, 1])   # group of 3 < r = 4
    assert e.value.code == so.E_BOUND
    with pytest.raises(so.OracleError) as e:
        so.make_plan(P=4, s=1, m=2, w=[0.5, 0.5, -0.2, 0.1])
    assert e.value.code == so.E_POINTS
    with pytest.raises(so.OracleError) as e:
        so.make_plan(P=4, s=1, m=2, w=[0.5, 0.0, -0.2, 0.1])
    assert e.value.code == so.E_POINTS


def test_message_length_table2():
    path = os.path.join(os.path.dirname(__file__), "golden", "table2_message_sizes.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for name, full, c6, c8, c10 in rows:
        d = round(float(full) * 1e6 / 8)             # 8 bytes per parameter on the paper's wire
        for m, printed in ((6, c6), (8, c8), (10, c10)):
            mb = so.message_length(d, m) * 8 / 1e6
            assert abs(mb - float(printed)) / float(printed) < 3e-3, (name, m, mb, printed)
    assert so.message_length(4099, 4) == 1025 and so.message_length(4096, 4) == 1024 and so.message_length(1, 4) == 1


# ---------------------------------------------------------------- f of phi (Sec. 3.4), counter-based
def test_generator_matches_the_published_known_answers():
    path = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for words in rows:
        v = [int(x, 16) for x in words]
        assert so.philox4x32_10(v[0:4], v[4:6]) == v[6:10]


def test_drawn_projection_vector_is_the_documented_function_of_seed_and_column():
    """Element p of f depends on (seed, p) only: the block generator on counter (p // 4, 0, 0, 0), Box-Muller on word pair
    (p % 4) // 2 - checked element by element with scalar arithmetic; and f is N(1, 1) as Sec. 3.4 asks (first four moments)."""
    import math
    seed = (0x9abcdef0 << 32) | 0x12345678
    f = so.draw_projection(seed, 1003)
    assert f.shape == (1003,) and f.dtype == np.float32
    for p in (0, 1, 2, 3, 4, 517, 1001, 1002):
        x = so.philox4x32_10((p // 4, 0, 0, 0), (0x12345678, 0x9abcdef0))
        a, b = x[2 * ((p % 4) // 2)], x[2 * ((p % 4) // 2) + 1]
        r = math.sqrt(-2.0 * math.log((a + 0.5) / 2.0 ** 32))
        ang = 2.0 * math.pi * (b + 0.5) / 2.0 ** 32
        z = r * (math.cos(ang) if p % 2 == 0 else math.sin(ang))
        assert abs(float(f[p]) - (1.0 + z)) <= 2.0 ** -22 * max(1.0, abs(1.0 + z))
    assert np.array_equal(so.draw_projection(seed, 40)[:37], so.draw_projection(seed, 37))      # a prefix is a prefix
    assert not np.array_equal(so.draw_projection(seed + 1, 40), so.draw_projection(seed, 40))
    g = so.draw_projection(7, 2_000_000).astype(np.float64) - 1.0
    assert abs(g.mean()) < 4e-3 and abs(g.var() - 1.0) < 6e-3 and abs((g ** 3).mean()) < 2e-2 and abs((g ** 4).mean() - 3.0) < 5e-2


# ---------------------------------------------------------------- encode (Sec. 3.4)
def test_encode_coordinatewise_definition():
    """Z[j][p] = sum_l w_j^l * (sum of the group's gradients)[p m + l], written as scalar loops."""
    rng = np.random.default_rng(0)
    P, s, m, d = 9, 1, 3, 17                          # ragged, d not a multiple of m
    plan = so.make_plan(P, s, m)
    G = rand_G(rng, P, d)
    Z = so.encode(plan, G)
    assert Z.shape == (P, 6)
    for g in range(plan.q):
        for j in plan.nodes[g]:
            for p in range(6):
                acc = 0.0
                for l in range(m):
                    c = p * m + l
                    if c < d:
                        ysum = 0.0
                        for k in plan.batches[g]:
                            ysum += float(G[k, c])
                        acc += float(plan.w[j]) ** l * ysum
                assert abs(Z[j, p] - acc) <= 1e-14 * max(1.0, abs(acc))


def test_encode_unit_points_give_chunk_sums():
    rng = np.random.default_rng(1)
    P, s, m, d = 4, 1, 2, 10
    w = np.array([1.0, -1.0, 0.5, 2.0], dtype=np.float32)
    plan = so.make_plan(P, s, m, w=w)
    G = rand_G(rng, P, d)
    Z = so.encode(plan, G)
    ybar = G.astype(np.float64).sum(0)
    assert np.allclose(Z[0], ybar[0::2] + ybar[1::2], rtol=0, atol=1e-15)      # w = 1: plain chunk sum
    assert np.allclose(Z[1], ybar[0::2] - ybar[1::2], rtol=0, atol=1e-15)      # w = -1: alternating sum
    assert np.allclose(Z[3], ybar[0::2] + 2 * ybar[1::2], rtol=0, atol=1e-15)


def test_m1_is_repetition_code():
    """r_c = 1: W_j = I_d, every node of a group sends the group's gradient sum itself."""
    rng = np.random.default_rng(2)
    plan = so.make_plan(P=7, s=1, m=1)
    G = rand_G(rng, 7, 33)
    Z = so.encode(plan, G)
    for g in range(plan.q):
        ysum = G[plan.batches[g]].astype(np.float64).sum(0)
        for j in plan.nodes[g]:
            assert np.array_equal(Z[j], ysum)


def test_encode_linear():
    rng = np.random.default_rng(3)
    plan = so.make_plan(P=10, s=3, m=4)
    G1, G2 = rand_G(rng, 10, 41), rand_G(rng, 10, 41)
    a, b = 0.75, -2.0
    lhs = so.encode(plan, a * G1.astype(np.float64) + b * G2.astype(np.float64))
    rhs = a * so.encode(plan, G1) + b * so.encode(plan, G2)
    assert np.allclose(lhs, rhs, rtol=0, atol=1e-15)


# ---------------------------------------------------------------- Def. 1 / Thm. 3: exact recovery
@pytest.mark.parametrize("P,s,m", SHAPES)
@pytest.mark.parametrize("d", [1, 64, 4099])
def test_decode_equals_plain_sum_without_adversaries(P, s, m, d):
    rng = np.random.default_rng(10 + P + d)
    plan = so.make_plan(P, s, m)
    G = rand_G(rng, P, d)
    Z = so.encode(plan, G)
    f = 1.0 + rng.standard_normal(Z.shape[1])
    for method in ("bw", "bruteforce") if P <= 15 else ("bw",):
        assert so.locate(plan, so.project(Z, f), method) == []
    u = so.decode(plan, Z, [], d)
    assert so.rel_l2(u, so.plain_sum(G)) < 1e-11


@pytest.mark.parametrize("P,s,m", SHAPES)
@pytest.mark.parametrize("kind", ["flip", "noise", "const", "fake", "mix"])
def test_any_s_corruptions_are_located_and_removed(P, s, m, kind):
    rng = np.random.default_rng(100 + P)
    d = 515
    plan = so.make_plan(P, s, m)
    G = rand_G(rng, P, d)
    Z = so.encode(plan, G)
    f = 1.0 + rng.standard_normal(Z.shape[1])
    placements = [sorted(rng.choice(P, size=s, replace=False).tolist()),
                  plan.nodes[0][:s].tolist(),                         # all adversaries in one group
                  plan.nodes[plan.q - 1][-s:].tolist()]
    if s > 1:
        placements.append(sorted(rng.choice(P, size=s - 1, replace=False).tolist()))   # fewer than s
    for bad in placements:
        R = corrupt(rng, Z, bad, kind)
        rho = so.project(R, f)
        V = so.locate(plan, rho, "bw")
        assert V == sorted(bad), (bad, V)
        if max(len(n) for n in plan.nodes) <= 11:
            assert so.locate(plan, rho, "bruteforce") == sorted(bad)
        u = so.decode(plan, R, V, d)
        assert so.rel_l2(u, so.plain_sum(G)) < 1e-9


def test_update_is_the_plain_sgd_step_on_the_true_gradient_sum():
    """Sec. 3.1: w_t = w_{t-1} - gamma / |S| * sum_k g_k, written as scalar loops over the TRUE gradients - whatever
    up to s nodes sent instead."""
    rng = np.random.default_rng(21)
    P, s, m, d = 10, 3, 4, 37
    plan = so.make_plan(P, s, m)
    G = rand_G(rng, P, d)
    Z = so.encode(plan, G)
    w0 = rng.standard_normal(d)
    gamma = 0.05
    expect = np.empty(d)
    for c in range(d):
        total = 0.0
        for k in range(P):
            total += float(G[k, c])
        expect[c] = w0[c] - gamma / P * total
    for bad in ([], [0, 4, 9]):
        R = corrupt(rng, Z, bad, "mix")
        f = 1.0 + rng.standard_normal(Z.shape[1])
        V = so.locate(plan, so.project(R, f), "bw")
        assert V == bad
        assert np.allclose(so.decode_update(plan, R, V, w0, gamma / P), expect, rtol=0, atol=1e-12)


def test_colluding_valid_codeword_of_fake_gradient():
    """s nodes of one group send consistent messages of a different gradient: still out-voted."""
    rng = np.random.default_rng(5)
    P, s, m, d = 14, 5, 4, 256
    plan = so.make_plan(P, s, m)
    G = rand_G(rng, P, d)
    Gfake = rand_G(rng, P, d)
    Z, Zfake = so.encode(plan, G), so.encode(plan, Gfake)
    bad = [1, 4, 6, 9, 13]
    R = Z.copy()
    R[bad] = Zfake[bad]
    f = 1.0 + rng.standard_normal(Z.shape[1])
    V = so.locate(plan, so.project(R, f), "bw")
    assert V == bad
    assert so.rel_l2(so.decode(plan, R, V, d), so.plain_sum(G)) < 1e-9


def test_more_than_s_corruptions_in_a_group_is_an_error():
    rng = np.random.default_rng(6)
    plan = so.make_plan(P=8, s=1, m=2)
    Z = so.encode(plan, rand_G(rng, 8, 64))
    R = corrupt(rng, Z, [0, 2], "noise")
    f = 1.0 + rng.standard_normal(Z.shape[1])
    for method in ("bw", "bruteforce"):
        with pytest.raises(so.OracleError) as e:
            so.locate(plan, so.project(R, f), method)
        assert e.value.code == so.E_DECODE


def test_nonfinite_rows_are_located():
    rng = np.random.default_rng(7)
    P, s, m, d = 12, 2, 2, 100
    plan = so.make_plan(P, s, m)
    G = rand_G(rng, P, d)
    Z = so.encode(plan, G)
    R = Z.copy()
    R[3] = np.nan
    R[4, ::2] = np.inf
    f = 1.0 + rng.standard_normal(Z.shape[1])
    rho = so.project(R, f)
    for method in ("bw", "bruteforce"):
        assert so.locate(plan, rho, method) == [3, 4]
    assert so.rel_l2(so.decode(plan, R, [3, 4], d), so.plain_sum(G)) < 1e-11


# ---------------------------------------------------------------- locator internals
@pytest.mark.parametrize("P,s,m", [(4, 1, 2), (6, 2, 2), (10, 3, 4), (14, 5, 4)])
def test_quotient_matches_lemma_closed_form(P, s, m):
    """Lemma l9: P_j(w) = sum_k u_k w^k with u_k = sum_p f_p ybar[k + p m], whatever the corruption."""
    rng = np.random.default_rng(8)
    d = 64 * m
    plan = so.make_plan(P, s, m)
    assert plan.q == 1
    G = rand_G(rng, P, d)
    Z = so.encode(plan, G)
    f = 1.0 + rng.standard_normal(Z.shape[1])
    ybar = G.astype(np.float64).sum(0).reshape(-1, m)
    closed = (f[:, None] * ybar).sum(0)
    for bad in ([], list(range(s))):
        R = corrupt(rng, Z, bad, "noise")
        quo = so.quotient(plan, so.project(R, f), 0)
        assert np.allclose(quo, closed, rtol=1e-8, atol=1e-9 * np.abs(closed).max())


@pytest.mark.parametrize("P,s,m", [(4, 1, 2), (5, 1, 2), (3, 1, 1), (6, 2, 2)])
def test_printed_formula_agrees_on_small_cases(P, s, m):
    """phi exactly as printed (monomial basis, quotient by polynomial division) gives the same set
    and the same quotient when exactly s nodes are corrupted (the system is then nonsingular)."""
    rng = np.random.default_rng(9)
    d = 32 * m
    plan = so.make_plan(P, s, m)
    G = rand_G(rng, P, d)
    Z = so.encode(plan, G)
    f = 1.0 + rng.standard_normal(Z.shape[1])
    for bad in combinations(range(P), s):
        R = corrupt(rng, Z, list(bad), "flip")
        rho = so.project(R, f)
        assert so.locate(plan, rho, "literal") == so.locate(plan, rho, "bw") == list(bad)
        assert np.allclose(so.quotient(plan, rho, 0, "literal"), so.quotient(plan, rho, 0, "bw"), rtol=1e-7)


def test_m1_decode_is_majority_vote():
    """Repetition code: the decoded group value is the vector sent by the majority of its nodes."""
    rng = np.random.default_rng(11)
    plan = so.make_plan(P=7, s=1, m=1)               # groups of 4 and 3
    G = rand_G(rng, 7, 50)
    Z = so.encode(plan, G)
    R = Z.copy()
    R[2] = rng.standard_normal(50)
    f = 1.0 + rng.standard_normal(50)
    rho = so.project(R, f)
    V = so.locate(plan, rho, "bw")
    expect_u = np.zeros(50)
    expect_V = []
    for g in range(plan.q):
        rows = [tuple(np.round(R[j], 12)) for j in plan.nodes[g]]
        majority = max(set(rows), key=rows.count)     # textbook majority
        assert rows.count(majority) > len(rows) / 2
        expect_u += np.array(majority)
        expect_V += [int(j) for j, row in zip(plan.nodes[g], rows) if row != majority]
    assert V == expect_V == [2]
    assert np.allclose(so.decode(plan, R, V, 50), expect_u, rtol=0, atol=1e-11)


def test_any_honest_subset_gives_same_group_sum():
    """psi may use any >= m honest rows (Lemma 2): dropping further honest rows changes nothing."""
    rng = np.random.default_rng(12)
    P, s, m, d = 10, 3, 4, 40
    plan = so.make_plan(P, s, m)
    G = rand_G(rng, P, d)
    Z = so.encode(plan, G)
    ref = so.plain_sum(G)
    for drop in ([], [0, 1, 2], [7, 8, 9], [0, 3, 5, 6, 8, 9]):
        assert so.rel_l2(so.decode(plan, Z, drop, d), ref) < 1e-9


# ---------------------------------------------------------------- Thm. 2: the bound is tight
def test_below_the_bound_two_gradients_are_indistinguishable():
    """Proof of Thm. 2 made concrete for the linear block code: with one node fewer than 2s+m there are
    G1 != G2 and valid s-attacks N1, N2 with Z1 + N1 == Z2 + N2, so no decoder can be right for both;
    with 2s+m nodes the same attack is decoded correctly."""
    s, m, d = 2, 3, 12
    tau_nodes = 2 * s + m - 1
    w = so.default_points(tau_nodes + 1)
    plan_low = so.make_plan(P=tau_nodes, s=s, m=m, w=w[:tau_nodes], check_bound=False,
                            group_of_node=[0] * tau_nodes)
    with pytest.raises(so.OracleError):
        so.make_plan(P=tau_nodes, s=s, m=m, w=w[:tau_nodes], group_of_node=[0] * tau_nodes)
    rng = np.random.default_rng(13)
    G1 = rand_G(rng, tau_nodes, d).astype(np.float64)
    # x_hat: chunk by chunk the coefficients of prod_{i < m-1} (w - w_i): invisible to the first m-1 nodes
    coeffs = np.poly(w[:m - 1].astype(np.float64))[::-1]          # ascending, length m
    x_hat = np.tile(coeffs, d // m)
    G1[0] = 1.0
    G2 = G1.copy()
    G2[0] = 1.0 + x_hat
    Z1, Z2 = so.encode(plan_low, G1), so.encode(plan_low, G2)
    assert np.allclose(Z1[:m - 1], Z2[:m - 1], rtol=0, atol=1e-14)
    N1, N2 = np.zeros_like(Z1), np.zeros_like(Z1)
    N1[m - 1:m - 1 + s] = (Z2 - Z1)[m - 1:m - 1 + s]
    N2[m - 1 + s:] = (Z1 - Z2)[m - 1 + s:]
    assert np.count_nonzero(np.abs(N1).sum(1)) <= s and np.count_nonzero(np.abs(N2).sum(1)) <= s
    assert np.allclose(Z1 + N1, Z2 + N2, rtol=0, atol=1e-14)
    assert np.linalg.norm(so.plain_sum(G1) - so.plain_sum(G2)) > 0.1
    # at the bound: one more node, the same kind of attack is harmless
    P = tau_nodes + 1
    plan_ok = so.make_plan(P=P, s=s, m=m, w=w)
    G1b = np.vstack([G1, rand_G(rng, 1, d)])
    G2b = G1b.copy()
    G2b[0] = 1.0 + x_hat
    Z1b, Z2b = so.encode(plan_ok, G1b), so.encode(plan_ok, G2b)
    R = Z1b.copy()
    R[m - 1:m - 1 + s] = Z2b[m - 1:m - 1 + s]
    f = 1.0 + rng.standard_normal(Z1b.shape[1])
    V = so.locate(plan_ok, so.project(R, f), "bw")
    assert V == list(range(m - 1, m - 1 + s))
    assert so.rel_l2(so.decode(plan_ok, R, V, d), so.plain_sum(G1b)) < 1e-10


# ---------------------------------------------------------------- planted mistakes must be caught
def test_pins_catch_planted_mistakes(monkeypatch):
    """A transposed chunk layout or a dropped power in the encoder breaks exact recovery."""
    rng = np.random.default_rng(14)
    P, s, m, d = 8, 1, 2, 32
    plan = so.make_plan(P, s, m)
    G = rand_G(rng, P, d)
    good = so.encode(plan, G)
    bad = good.copy()
    ybar0 = G[plan.batches[0]].astype(np.float64).sum(0)
    j = plan.nodes[0][1]
    bad[j] = ybar0[:d // 2] + float(plan.w[j]) * ybar0[d // 2:]       # planar instead of interleaved chunks
    assert so.rel_l2(so.decode(plan, bad, [], d), so.plain_sum(G)) > 1e-3
    f = 1.0 + rng.standard_normal(d // 2)
    assert so.locate(plan, so.project(bad, f), "bw") == [int(j)]      # and the locator sees it as corrupt


@pytest.mark.parametrize("P,s,m", [(20, 5, 10), (16, 4, 8), (15, 5, 4), (11, 3, 4)])
def test_fewer_than_s_corruptions_with_fp32_rounded_messages(P, s, m):
    """Messages rounded to fp32 (as on the wire) and 0..s corrupted nodes: the located set is the planted one.
    With fewer than s corrupted nodes the locator polynomial has spare, arbitrary roots; honest nodes that
    happen to sit on them must not be flagged (they would be if P_j were fitted without them and extrapolated)."""
    rng = np.random.default_rng(77 + P)
    plan = so.make_plan(P, s, m)
    d = 300 * m
    wrong = 0
    for trial in range(60):
        G = rand_G(rng, P, d)
        Z = so.encode(plan, G).astype(np.float32).astype(np.float64)
        e = trial % (s + 1)
        bad = sorted(rng.choice(P, size=e, replace=False).tolist())
        R = corrupt(rng, Z, bad, "mix")
        f = (1.0 + rng.standard_normal(Z.shape[1])).astype(np.float32)
        V = so.locate(plan, so.project(R, f), "bw")
        wrong += (V != bad)
    assert wrong == 0
