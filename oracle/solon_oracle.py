"""Plain fp64 CPU oracle for the Solon linear block code (encode, locate, decode).

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only tests, the smoke check and the
CPU-baseline leg of the benchmark may import it.  It shares no code with the HIP
library and imports nothing from it.  Everything is numpy in float64; inputs that
arrive as fp32 (or bf16 widened to fp32) are widened exactly.  Nothing here is blocked,
fused or reordered beyond what the paper's definitions state.

Notation follows the paper (Sec. 3.1-3.4): P nodes, B = P per-batch gradients of
dimension d, at most s Byzantine nodes, compression ratio m (the paper's r_c),
message length d_c = ceil(d / m), redundancy r = 2 s + m (Thm. 2), q groups, evaluation
points w_j, projection vector f, received matrix R = Z + N.  Arrays are stored
row-major with one ROW per node / per batch (the paper writes them as columns).

Functions and the passage each follows
  make_plan          allocation A = I_q (x) 1_{r x r} (Sec. 3.4, "Linear Block Code"); Thm. 2 and
                     its corollary as parameter checks; ragged groups when r does not divide P
  default_points     "any distinct nonzero scalars" w_j (Sec. 3.4) - the values are this build's choice
  encode             z_j = W_j Y_j 1_P with W_j = I_{d_c} (x) [1, w_j, ..., w_j^{m-1}] (Sec. 3.4)
  draw_projection    the random vector f of phi (Sec. 3.4), counter-based
  project            r_{j,c} = f R_j (Sec. 3.4, definition of phi)
  locate_bruteforce  the combinatorial definition: smallest subset S whose complement is
                     consistent with the code (App. C, sparse-recovery equivalence)
  locate_bw          phi: the error-locator linear system of Sec. 3.4 solved in the least-squares
                     sense, then P_j and V = {i : P_j(w_i) != r_i} (Lemma 1, Lemma l9)
  locate_literal     phi exactly as printed (monomial basis, P_j by polynomial division); kept
                     only to tie locate_bw to the printed formula on tiny well-conditioned cases
  decode             Algorithm 1 with psi = least-squares inverse of the honest rows'
                     Vandermonde (Sec. 3.4, Lemma 2); u = sum over groups
  decode_update      decode followed by the training step w <- w - gamma / |S| * u (Sec. 3.1)
  plain_sum          the definition the whole mechanism must reproduce: G 1_P (Def. 1)

Pins (tests/test_oracle_*.py): decode == plain_sum with zero and with <= s corrupted rows (Def. 1,
Thm. 3); located set == planted set == brute force (Lemma 1, App. C); quotient coefficients ==
closed form of Lemma l9; m = 1 reduces to a repetition code with majority vote; w_j = 1 gives chunk
sums; linearity; message length of Table 2; bound tightness construction of Thm. 2's proof.

Parity unpinned by the paper: the numerical thresholds (TAU, the median scale, the rank tolerance).
The paper works over the reals ("!=", "with probability equal to unity"); these values are this
build's reading and are pinned only by requiring brute force, locate_bw, the HIP path and the planted
truth to coincide on every test and bench input, and - for TAU - by a window: at 1e-2 a corruption gets
through that costs the decoded sum more than 1e-4, at 1e-8 fp32 rounding of honest messages is reported.
"""
from itertools import combinations

import numpy as np
from numpy.polynomial import chebyshev as _cheb
from numpy.polynomial import polynomial as _poly

# status codes (same meaning as the C-ABI's, defined independently here)
OK, E_INVAL, E_BOUND, E_POINTS, E_DECODE, E_NUMERIC = 0, -1, -2, -3, -4, -5

TAU = 1e-4          # residual test threshold, relative to the group's median |rho|
RANK_RCOND = 1e-10  # relative singular-value cut-off of the locator system's least-squares solve
SEARCH_LIMIT = 1 << 16  # candidate sets phi tries beyond the locator's leading roots before it gives up


class OracleError(Exception):
    def __init__(self, code, msg):
        super().__init__(msg)
        self.code = code


class Plan:
    """Immutable description of one code instance."""

    def __init__(self, P, B, s, m, q, r, nodes, batches, w):
        self.P, self.B, self.s, self.m, self.q, self.r = P, B, s, m, q, r
        self.nodes = nodes      # list of q int arrays: node indices of each group, ascending
        self.batches = batches  # list of q int arrays: gradient indices of each group
        self.w = w              # float32[P]: evaluation point of every node


def default_group_sizes(P, r):
    """Balanced ragged blocks: q = floor(P / r) groups, the first (P mod q) one larger."""
    q = P // r
    base, extra = divmod(P, q)
    return [base + 1 if g < extra else base for g in range(q)]


def default_points(r_g):
    """Chebyshev-type points in (-1, 1), none zero, rounded to fp32 (treated as exact afterwards).

    K = 2 ceil(r_g / 2) first-kind Chebyshev nodes x_i = cos((2 i - 1) pi / (2 K)), i = 1..K;
    for odd r_g the node with 0-based index K/2 is left out.
    """
    K = 2 * ((r_g + 1) // 2)
    i = np.arange(1, K + 1, dtype=np.float64)
    x = np.cos((2.0 * i - 1.0) * np.pi / (2.0 * K))
    if r_g % 2 == 1:
        x = np.delete(x, K // 2)
    return x.astype(np.float32)


def make_plan(P, s, m, B=None, group_of_node=None, group_of_batch=None, w=None, check_bound=True):
    """Sec. 3.4 allocation.  Default: consecutive ragged blocks, batch k belongs to node k's group."""
    B = P if B is None else B
    if P < 1 or B < 1 or m < 1 or s < 0:
        raise OracleError(E_INVAL, "bad P, B, m or s")
    r = 2 * s + m
    if check_bound and 2 * s > P - m:                      # corollary of Thm. 2
        raise OracleError(E_BOUND, "s exceeds (P - m) / 2")
    if group_of_node is None:
        sizes = default_group_sizes(P, r)
        group_of_node = np.repeat(np.arange(len(sizes)), sizes)
    group_of_node = np.asarray(group_of_node, dtype=np.int64)
    if group_of_node.shape != (P,):
        raise OracleError(E_INVAL, "group_of_node must have P entries")
    if group_of_batch is None:
        if B != P:
            raise OracleError(E_INVAL, "group_of_batch is required when B != P")
        group_of_batch = group_of_node.copy()
    group_of_batch = np.asarray(group_of_batch, dtype=np.int64)
    if group_of_batch.shape != (B,):
        raise OracleError(E_INVAL, "group_of_batch must have B entries")
    q = int(group_of_node.max()) + 1
    if q < 1 or group_of_node.min() < -1 or group_of_batch.min() < 0 or group_of_batch.max() >= q:
        raise OracleError(E_INVAL, "bad group table")
    nodes = [np.flatnonzero(group_of_node == g) for g in range(q)]
    batches = [np.flatnonzero(group_of_batch == g) for g in range(q)]
    for g in range(q):
        if check_bound and len(nodes[g]) < r:              # Thm. 2: every gradient replicated >= 2s+m times
            raise OracleError(E_BOUND, "a group has fewer than 2s+m nodes")
    if w is None:
        w = np.zeros(P, dtype=np.float32)
        for g in range(q):
            w[nodes[g]] = default_points(len(nodes[g]))
    w = np.asarray(w, dtype=np.float32)
    if w.shape != (P,):
        raise OracleError(E_INVAL, "w must have P entries")
    for g in range(q):
        wg = w[nodes[g]]
        if np.any(wg == 0) or not np.all(np.isfinite(wg)) or len(np.unique(wg)) != len(wg):
            raise OracleError(E_POINTS, "evaluation points must be nonzero and distinct within a group")
    return Plan(P, B, s, m, q, r, nodes, batches, w)


def message_length(d, m):
    """d_c = ceil(d / m) (Sec. 3.1: r_c = d / d_c)."""
    return -(-d // m)


def plain_sum(G):
    """u = G 1_P: the sum of all per-batch gradients (Def. 1)."""
    return np.asarray(G, dtype=np.float64).sum(axis=0)


def encode(plan, G):
    """All P messages.  G: [B, d] -> Z: [P, d_c] float64.  Coordinates past d read as zero."""
    G = np.asarray(G, dtype=np.float64)
    B, d = G.shape
    m = plan.m
    d_c = message_length(d, m)
    Z = np.zeros((plan.P, d_c), dtype=np.float64)
    for g in range(plan.q):
        ybar = np.zeros(d_c * m, dtype=np.float64)
        ybar[:d] = G[plan.batches[g]].sum(axis=0)          # Y_j 1_P, identical for the whole group
        chunks = ybar.reshape(d_c, m)                      # chunk p holds coordinates p m .. p m + m - 1
        for j in plan.nodes[g]:
            wj = float(plan.w[j])
            powers = np.array([wj ** l for l in range(m)], dtype=np.float64)
            Z[j] = chunks @ powers                         # row p of W_j is [1, w_j, ..., w_j^{m-1}] on chunk p
    return Z


def draw_projection(seed, d_c):
    """f of phi (Sec. 3.4: i.i.d. normal, mean one, unit variance) as a pure function of (seed, column): the counter-based
    recipe the library documents - Philox-4x32 with ten rounds (Salmon et al., SC 2011) on the counter (column // 4, 0, 0, 0)
    under the key (seed mod 2^32, seed // 2^32); each pair of output words (x, y) gives the two normals
    sqrt(-2 ln u1) (cos, sin)(2 pi u2), u1 = (x + 1/2) 2^-32, u2 = (y + 1/2) 2^-32, in double precision; f = 1 + z as float32."""
    M0, M1, W0, W1 = 0xD2511F53, 0xCD9E8D57, 0x9E3779B9, 0xBB67AE85
    nq = -(-d_c // 4)
    q = np.arange(nq, dtype=np.uint64)
    c = [q & np.uint64(0xFFFFFFFF), q >> np.uint64(32), np.zeros(nq, np.uint64), np.zeros(nq, np.uint64)]
    k0, k1 = int(seed) & 0xFFFFFFFF, (int(seed) >> 32) & 0xFFFFFFFF
    mask = np.uint64(0xFFFFFFFF)
    for _ in range(10):
        p0 = np.uint64(M0) * c[0]                       # 32 x 32 -> 64 bit products (operands are below 2^32)
        p1 = np.uint64(M1) * c[2]
        c = [(p1 >> np.uint64(32)) ^ c[1] ^ np.uint64(k0), p1 & mask, (p0 >> np.uint64(32)) ^ c[3] ^ np.uint64(k1), p0 & mask]
        k0, k1 = (k0 + W0) & 0xFFFFFFFF, (k1 + W1) & 0xFFFFFFFF
    out = np.empty((nq, 4), dtype=np.float64)
    for a, (x, y) in enumerate(((c[0], c[1]), (c[2], c[3]))):
        u1 = (x.astype(np.float64) + 0.5) * 2.0 ** -32
        u2 = (y.astype(np.float64) + 0.5) * 2.0 ** -32
        r = np.sqrt(-2.0 * np.log(u1))
        out[:, 2 * a] = 1.0 + r * np.cos(2.0 * np.pi * u2)
        out[:, 2 * a + 1] = 1.0 + r * np.sin(2.0 * np.pi * u2)
    return out.reshape(-1)[:d_c].astype(np.float32)


def philox4x32_10(counter, key):
    """One block of the generator above for a single counter (c0, c1, c2, c3) and key (k0, k1): four 32-bit words."""
    c = [int(v) for v in counter]
    k0, k1 = int(key[0]), int(key[1])
    for _ in range(10):
        p0, p1 = 0xD2511F53 * c[0], 0xCD9E8D57 * c[2]
        c = [(p1 >> 32) ^ c[1] ^ k0, p1 & 0xFFFFFFFF, (p0 >> 32) ^ c[3] ^ k1, p0 & 0xFFFFFFFF]
        k0, k1 = (k0 + 0x9E3779B9) & 0xFFFFFFFF, (k1 + 0xBB67AE85) & 0xFFFFFFFF
    return c


def project(R, f):
    """rho_j = sum_p f_p R[j][p] in float64."""
    R = np.asarray(R, dtype=np.float64)
    f = np.asarray(f, dtype=np.float64)
    return (R * f[None, :]).sum(axis=1)


def _scale(y):
    """Median magnitude of the finite projections of one group (honest nodes are a strict majority)."""
    fin = np.abs(y[np.isfinite(y)])
    if fin.size == 0:
        return 0.0
    med = float(np.median(fin))
    if med == 0.0:
        med = float(fin.max())
    return med


def _fit_and_test(wg, y, excluded, m, tau):
    """Least-squares polynomial of degree m-1 through the points not in `excluded`;
    returns (indices whose value differs from it by more than tau, residuals, Chebyshev coefficients)."""
    keep = np.array([i for i in range(len(wg)) if i not in excluded], dtype=np.int64)
    A = _cheb.chebvander(wg[keep], m - 1)
    coef = np.linalg.lstsq(A, y[keep], rcond=None)[0]
    res = np.abs(_cheb.chebval(wg, coef) - y)
    flagged = [i for i in range(len(wg)) if not (res[i] <= tau)]
    return flagged, res, coef


def _locate_group_bruteforce(wg, rho_g, s, m, tau):
    n = len(wg)
    nonfinite = [i for i in range(n) if not np.isfinite(rho_g[i])]
    sc = _scale(rho_g)
    if sc == 0.0:
        return nonfinite if len(nonfinite) <= s else None
    y = np.where(np.isfinite(rho_g), rho_g / sc, 0.0)
    for e in range(len(nonfinite), s + 1):
        for S in combinations(range(n), e):
            if any(i not in S for i in nonfinite):
                continue
            flagged, _, _ = _fit_and_test(wg, y, set(S), m, tau)
            if all(i in S for i in flagged):
                return sorted(S)
    return None


def _locate_group_bruteforce_stacked(wg, rho_g, s, m, tau):
    """The same enumeration as _locate_group_bruteforce with all subsets of one size fitted in one stacked QR call
    (rows of the left-out points are zeroed instead of deleted, which leaves the least-squares solution unchanged).
    Only quicker; the loop above is the definition, and a test holds the two equal."""
    n = len(wg)
    nonfinite = [i for i in range(n) if not np.isfinite(rho_g[i])]
    sc = _scale(rho_g)
    if sc == 0.0:
        return nonfinite if len(nonfinite) <= s else None
    y = np.where(np.isfinite(rho_g), rho_g / sc, 0.0)
    A = _cheb.chebvander(wg, m - 1)
    for e in range(len(nonfinite), s + 1):
        subsets = [S for S in combinations(range(n), e) if all(i in S for i in nonfinite)]
        if not subsets:
            continue
        keep = np.ones((len(subsets), n))
        if e:
            keep[np.arange(len(subsets))[:, None], np.array(subsets)] = 0.0
        Qm, Rm = np.linalg.qr(A[None, :, :] * keep[:, :, None])
        coef = np.linalg.solve(Rm, (Qm.transpose(0, 2, 1) @ (y[None, :] * keep)[:, :, None]))[:, :, 0]
        res = np.abs(coef @ A.T - y[None, :])
        ok = np.all((res <= tau) | (keep == 0.0), axis=1)
        if ok.any():
            return sorted(subsets[int(np.argmax(ok))])
    return None


def _group_explanations(wg, rho_g, s, m, tau):
    """ALL subsets of the smallest size that explain the group (same fits and test as the enumeration above, stacked).
    Over the reals there is exactly one (Lemma 1); at a finite threshold a deviation that the fit can absorb by bending
    towards a neighbouring point - end points of a long group at large m - may leave two.  Tests use this to tell a
    unique located set from an ambiguous one."""
    n = len(wg)
    nonfinite = [i for i in range(n) if not np.isfinite(rho_g[i])]
    sc = _scale(rho_g)
    if sc == 0.0:
        return [nonfinite] if len(nonfinite) <= s else []
    y = np.where(np.isfinite(rho_g), rho_g / sc, 0.0)
    A = _cheb.chebvander(wg, m - 1)
    for e in range(len(nonfinite), s + 1):
        subsets = [S for S in combinations(range(n), e) if all(i in S for i in nonfinite)]
        if not subsets:
            continue
        keep = np.ones((len(subsets), n))
        if e:
            keep[np.arange(len(subsets))[:, None], np.array(subsets)] = 0.0
        Qm, Rm = np.linalg.qr(A[None, :, :] * keep[:, :, None])
        coef = np.linalg.solve(Rm, (Qm.transpose(0, 2, 1) @ (y[None, :] * keep)[:, :, None]))[:, :, 0]
        res = np.abs(coef @ A.T - y[None, :])
        ok = np.all((res <= tau) | (keep == 0.0), axis=1)
        if ok.any():
            return [sorted(subsets[i]) for i in np.flatnonzero(ok)]
    return []


def explanations(plan, rho, g, tau=TAU):
    """Every smallest set of nodes of group g (global indices) without which the group's projections are consistent."""
    idx = plan.nodes[g]
    sets = _group_explanations(plan.w[idx].astype(np.float64), np.asarray(rho, dtype=np.float64)[idx], plan.s, plan.m, tau)
    return [[int(idx[i]) for i in S] for S in sets]


def _locator_system(wg, y, m, s):
    """[W_{m+s-1}, -W_{s-1} .* (y 1^T)] a = y .* T_s(w): the system of Sec. 3.4 written in the
    Chebyshev basis (a change of basis of the unknown polynomials; the locator's leading
    Chebyshev coefficient is fixed to one), rows scaled by 1 / max(1, |y_i|)."""
    VN = _cheb.chebvander(wg, m + s - 1)
    VD = _cheb.chebvander(wg, s)
    A = np.hstack([VN, -VD[:, :s] * y[:, None]])
    b = y * VD[:, s]
    eq = 1.0 / np.maximum(1.0, np.abs(y))
    return A * eq[:, None], b * eq


def _accept(wf, y, S, m, tau):
    """Is S an explanation of the data?  Fit P_j without S; every other point must lie within tau of it.
    An accepted S is then reduced to a smallest one in the sense of App. C: a point goes back in whenever the
    rest stays consistent with it (so an honest point that was left out needlessly is never reported, however
    far the fit had to be extrapolated to reach it).  Returns (V, coefficients) or None."""
    S = set(S)
    fl, _, coef = _fit_and_test(wf, y, S, m, tau)
    if not set(fl) <= S:
        return None
    reduced = True
    while reduced:
        reduced = False
        for j in sorted(S):
            fl2, _, coef2 = _fit_and_test(wf, y, S - {j}, m, tau)
            if set(fl2) <= S - {j}:
                S, coef, reduced = S - {j}, coef2, True
                break
    return sorted(S), coef


def _candidate_sets(order, s_eff):
    """The sets phi tries as "corrupted", in order.  `order` lists the points by increasing |D(w_i)|.
    First the leading roots of the locator: {}, {o_0}, {o_0, o_1}, ... up to s_eff points - over the reals the first
    of them that explains the data is the answer (Lemma 1).  In floating point a weakly corrupted point's |D| can
    come out larger than an honest neighbour's, so the search then widens to every subset of at most s_eff points,
    ordered by the position c of its last point in `order`, then by size, then colexicographically: all subsets of
    the c leading points are tried before any that needs point c + 1.  Carried to the end this is the subset
    enumeration of the sparse-recovery appendix (App. C); it stops after SEARCH_LIMIT sets."""
    for e in range(s_eff + 1):
        yield list(order[:e])
    tried = 0
    for c in range(1, len(order) + 1):
        for e in range(1, min(s_eff, c) + 1):
            for T in sorted(combinations(range(c - 1), e - 1), key=lambda t: t[::-1]):
                if tried >= SEARCH_LIMIT:
                    return
                tried += 1
                yield [order[t] for t in T] + [order[c - 1]]


def _locate_group_bw(wg, rho_g, s, m, tau, want_quotient=False):
    n = len(wg)
    nonfinite = [i for i in range(n) if not np.isfinite(rho_g[i])]
    if len(nonfinite) > s:
        return None
    sc = _scale(rho_g)
    if sc == 0.0:
        return (nonfinite, None) if want_quotient else nonfinite
    fin = np.array([i for i in range(n) if i not in nonfinite], dtype=np.int64)
    y = rho_g[fin] / sc
    wf = wg[fin]
    s_eff = s - len(nonfinite)                  # locator degree left for the finite entries
    if s_eff > 0:
        A, b = _locator_system(wf, y, m, s_eff)
        a = np.linalg.lstsq(A, b, rcond=RANK_RCOND)[0]
        D = np.concatenate([a[m + s_eff:], [1.0]])
        # every corrupted point is a root of every solution's locator; when fewer than s nodes are corrupt the
        # locator has further, arbitrary roots, so order the points by |D(w_i)| (corrupted ones come first)
        absD = np.abs(_cheb.chebval(wf, D))
        order = np.argsort(absD, kind="stable").tolist()
    else:
        order = []
    # P_j: the degree-(m-1) polynomial through all points but the corrupted ones (equals N / D over the reals)
    found = None
    for S in _candidate_sets(order, s_eff):
        found = _accept(wf, y, S, m, tau)
        if found is not None:
            break
    if found is None:
        return None
    flagged, coef = found
    V = sorted(nonfinite + [int(fin[i]) for i in flagged])
    if want_quotient:
        return V, _cheb.cheb2poly(coef) * sc if m > 1 else coef * sc
    return V


def _locate_group_literal(wg, rho_g, s, m, tau):
    """phi as printed: monomial basis, unknowns a_1..a_{m+2s}, P_j = numerator / denominator."""
    sc = _scale(rho_g)
    y = rho_g / sc
    VN = np.vander(wg, m + s, increasing=True)
    VD = np.vander(wg, s + 1, increasing=True)
    A = np.hstack([VN, -VD[:, :s] * y[:, None]])
    b = y * VD[:, s]
    a = np.linalg.lstsq(A, b, rcond=RANK_RCOND)[0]
    num = a[:m + s]
    den = np.concatenate([a[m + s:], [1.0]])
    quo, _ = _poly.polydiv(num, den)
    res = np.abs(_poly.polyval(wg, quo) - y)
    return [i for i in range(len(wg)) if not (res[i] <= tau)], quo * sc


def locate(plan, rho, method="bw", tau=TAU):
    """V for all groups: sorted global node indices.  Raises OracleError(E_DECODE) when a group
    cannot be explained by <= s corrupted nodes."""
    rho = np.asarray(rho, dtype=np.float64)
    V = []
    for g in range(plan.q):
        idx = plan.nodes[g]
        wg = plan.w[idx].astype(np.float64)
        if method == "bw":
            Vg = _locate_group_bw(wg, rho[idx], plan.s, plan.m, tau)
        elif method == "bruteforce":
            Vg = _locate_group_bruteforce(wg, rho[idx], plan.s, plan.m, tau)
        elif method == "bruteforce_stacked":
            Vg = _locate_group_bruteforce_stacked(wg, rho[idx], plan.s, plan.m, tau)
        elif method == "literal":
            Vg, _ = _locate_group_literal(wg, rho[idx], plan.s, plan.m, tau)
            if len(Vg) > plan.s:
                Vg = None
        else:
            raise ValueError(method)
        if Vg is None:
            raise OracleError(E_DECODE, "group %d: more than s inconsistent nodes" % g)
        V.extend(int(idx[i]) for i in Vg)
    return sorted(V)


def quotient(plan, rho, g, method="bw", tau=TAU):
    """Monomial coefficients (ascending) of P_j for group g - Lemma l9 says they equal
    u_k = sum_p f_p ybar[k + p m]."""
    idx = plan.nodes[g]
    wg = plan.w[idx].astype(np.float64)
    if method == "literal":
        return _locate_group_literal(wg, np.asarray(rho, dtype=np.float64)[idx], plan.s, plan.m, tau)[1]
    return _locate_group_bw(wg, np.asarray(rho, dtype=np.float64)[idx], plan.s, plan.m, tau, want_quotient=True)[1]


def decode(plan, R, V, d):
    """Algorithm 1 given the located set V (global indices): per group, psi over ALL honest nodes
    (least-squares inverse of their m-column Vandermonde), then the sum over groups.  R: [P, d_c]."""
    R = np.asarray(R)
    m = plan.m
    d_c = message_length(d, m)
    if R.shape != (plan.P, d_c):
        raise OracleError(E_INVAL, "R must be P x d_c")
    Vset = set(int(v) for v in V)
    u = np.zeros(d_c * m, dtype=np.float64)
    for g in range(plan.q):
        U = np.array([j for j in plan.nodes[g] if int(j) not in Vset], dtype=np.int64)
        if len(U) < m:
            raise OracleError(E_DECODE, "group %d: fewer than m honest nodes" % g)
        W_U = np.vander(plan.w[U].astype(np.float64), m, increasing=True)   # [W_{m-1}]_{U,.}
        R_U = R[U].astype(np.float64)                                       # |U| x d_c
        coeffs = np.linalg.lstsq(W_U, R_U, rcond=None)[0]                   # m x d_c: chunk p's coefficients
        u += coeffs.T.reshape(-1)                                           # vec(): coordinate p m + l
    return u[:d]


def decode_update(plan, R, V, params, step):
    """The step that follows the path in training (Sec. 3.1, "Distributed learning"): w_t = w_{t-1} - gamma_t / |S_t| *
    (sum of the gradients), with the sum recovered by decode() and step = gamma / |S|.  Returns the new parameters."""
    params = np.asarray(params, dtype=np.float64)
    return params - float(step) * decode(plan, R, V, params.shape[0])


def decode_majority(plan, R, d):
    """Repetition code (m = 1): per group and coordinate the value held by more than half of the group's nodes
    (the paper's appendix on the repetition code), summed over groups.  The majority element of a list, if there
    is one, is the middle element of the sorted list; that it really is a majority is then counted.
    Returns (u, V) with V the nodes that differ from their group's majority anywhere."""
    if plan.m != 1:
        raise OracleError(E_INVAL, "majority decoding needs m = 1")
    R = np.asarray(R, dtype=np.float64)
    u = np.zeros(d, dtype=np.float64)
    V = []
    for g in range(plan.q):
        idx = plan.nodes[g]
        block = R[idx][:, :d]
        with np.errstate(invalid="ignore"):
            middle = np.sort(block, axis=0)[len(idx) // 2]       # NaNs sort last and never reach the middle of a majority
            same = block == middle[None, :]
        if np.any(2 * same.sum(axis=0) <= len(idx)):
            raise OracleError(E_DECODE, "group %d: a coordinate has no majority value" % g)
        u += middle
        V.extend(int(idx[i]) for i in range(len(idx)) if not same[i].all())
    return u, sorted(V)


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    nb = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / nb) if nb > 0 else float(np.linalg.norm(a - b))
