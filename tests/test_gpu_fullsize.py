"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.

Outputs too large to copy whole are checked on sampled column windows the oracle computes one by one
(encode, decode), rho and the located set are checked in full (the oracle streams R in windows), and the
decoded aggregate is additionally checked over ALL coordinates against the plain sum G 1_P accumulated in
fp64 by torch on the device (a property that holds at any size: Def. 1 of the paper)."""
import time

import numpy as np
import pytest
import torch

import paper_2110_01595_amd as solon
import workloads
from oracle import solon_oracle as so

pytestmark = pytest.mark.gpu
DEV = torch.device("cuda:0")
WIN = 4096          # chunks per sampled window
RHO_WIN = 1 << 20   # chunks per window when the oracle streams the projection


def say(*a):
    print(*a, flush=True)


def windows(d_c):
    starts = sorted(set([0, (d_c // 3) // 4 * 4 + 1, d_c // 2, max(0, d_c - WIN)]))
    return [(p0, min(d_c, p0 + WIN)) for p0 in starts]


@pytest.mark.timeout(900)
@pytest.mark.parametrize("name,u_tol", [("C1", 1e-4), ("C2", 1e-4), ("C3", 1e-4), ("C4", 1e-4), ("C5", 1e-4), ("X1", 1e-4)])
def test_full_size_config(name, u_tol):
    check_config(name, workloads.CONFIGS[name], workloads.seeds(name), u_tol)


@pytest.mark.timeout(900)
def test_rows_longer_than_2_to_the_31_elements():
    """Largest single dimension: gradients of 2^31 + 2052 coordinates (8.6 GB a row), so that every element index
    beyond a row's start, and every byte offset, leaves 32 bits; d_c = 2^30 + 1026 is not a multiple of four."""
    cfg = dict(P=4, s=1, m=2, d=2 ** 31 + 2052, dtype="f32", dist="normal", sigma=0.01, attack="flip10")
    check_config("long-rows", cfg, dict(G=1101, f=2101, byz=3101, attack=4101), 1e-4)


def check_config(name, cfg, sd, u_tol):
    t_start = time.time()
    P, s, m, d = cfg["P"], cfg["s"], cfg["m"], cfg["d"]
    say("full-size", name, dict(P=P, s=s, m=m, d=d, dtype=cfg["dtype"], attack=cfg["attack"]))
    plan = solon.Plan(P, s, m, d, dtype=solon.SOLON_BF16 if cfg["dtype"] == "bf16" else solon.SOLON_F32)
    oplan = so.make_plan(P, s, m)
    d_c = plan.d_c
    G = workloads.make_gradients(cfg, DEV, sd["G"])
    Z = torch.empty((P, d_c), dtype=torch.float32, device=DEV)
    solon.solon_encode(plan, G, Z)
    torch.cuda.synchronize()
    say("  encoded", round(time.time() - t_start, 1), "s")

    # encode: sampled windows against the oracle
    for p0, p1 in windows(d_c):
        c0, c1 = p0 * m, min(d, p1 * m)
        Z_ref = so.encode(oplan, G[:, c0:c1].float().cpu().numpy())
        Zh = Z[:, p0:p1].cpu().numpy()
        assert so.rel_l2(Zh, Z_ref) <= 1e-6, (name, p0)
        assert np.abs(Zh - Z_ref).max() <= 4e-6 * (np.abs(Z_ref).max() + 1e-30)

    # encode, every element: the defining sum written with torch ops in fp64 on the device (no oracle at this size)
    wpts = torch.tensor(np.asarray(oplan.w, dtype=np.float64), device=DEV)
    num = den = 0.0
    worst = 0.0
    blk = 1 << 21
    for p0 in range(0, d_c, blk):
        p1 = min(d_c, p0 + blk)
        c0, c1 = p0 * m, min(d, p1 * m)
        for g in range(oplan.q):
            ybar = G[oplan.batches[g].tolist(), c0:c1].sum(dim=0, dtype=torch.float64)
            if ybar.numel() < (p1 - p0) * m:
                ybar = torch.nn.functional.pad(ybar, (0, (p1 - p0) * m - ybar.numel()))
            ybar = ybar.view(p1 - p0, m)
            for j in oplan.nodes[g].tolist():
                ref = (ybar * wpts[j] ** torch.arange(m, dtype=torch.float64, device=DEV)).sum(dim=1)
                diff = Z[j, p0:p1].double() - ref
                num += float((diff * diff).sum())
                den += float((ref * ref).sum())
                worst = max(worst, float(diff.abs().max()) / (float(ref.abs().max()) + 1e-30))
    say("  rel_l2(Z, definition) over all P x d_c = %.3e, worst row window %.3e" % ((num / den) ** 0.5, worst), round(time.time() - t_start, 1), "s")
    assert (num / den) ** 0.5 <= 1e-6 and worst <= 4e-6

    byz = workloads.pick_byzantine(P, s, sd["byz"])
    R = Z                                                   # attack in place: Z is not needed any more
    workloads.apply_attack(R, byz, cfg["attack"], sd["attack"])
    f = workloads.make_projection(d_c, DEV, sd["f"])
    V, rho = solon.solon_locate(plan, R, f, want_rho=True)
    u = torch.empty(d, dtype=torch.float32, device=DEV)
    solon.solon_decode(plan, R, u)
    assert solon.solon_decode_status(plan) == solon.SOLON_OK
    torch.cuda.synchronize()
    say("  located", V, "planted", byz, round(time.time() - t_start, 1), "s")
    assert V == byz

    # the one-pass entry point (what bench.py times): same located set, same projections, same bits of u
    u1 = torch.empty(d, dtype=torch.float32, device=DEV)
    V1, rho1 = solon.solon_locate_decode(plan, R, f, u1, want_rho=True)
    assert solon.solon_decode_status(plan) == solon.SOLON_OK
    assert V1 == V and np.allclose(rho1, rho, rtol=1e-12, atol=0)
    assert torch.equal(u1, u)
    del u1

    # projection and located set: the oracle streams all of R
    rho_ref = np.zeros(P)
    mag = np.zeros(P)
    for p0 in range(0, d_c, RHO_WIN):
        Rw = R[:, p0:p0 + RHO_WIN].cpu().numpy()
        fw = f[p0:p0 + RHO_WIN].cpu().numpy()
        rho_ref += so.project(Rw, fw)
        mag += np.abs(Rw).astype(np.float64) @ np.abs(fw).astype(np.float64)
    say("  oracle projection done", round(time.time() - t_start, 1), "s")
    assert np.all(np.abs(rho - rho_ref) <= 1e-12 * mag.max())
    assert so.locate(oplan, rho_ref, "bw") == V
    assert so.locate(oplan, rho_ref, "bruteforce_stacked") == V     # groups of at most 20 nodes: the whole enumeration is affordable

    # decode: sampled windows against the oracle's decode of the same R, and against the plain sum
    for p0, p1 in windows(d_c):
        c0, c1 = p0 * m, min(d, p1 * m)
        Rw = R[:, p0:p1].cpu().numpy()
        u_ref = so.decode(oplan, Rw, V, c1 - c0)
        uh = u[c0:c1].cpu().numpy()
        assert so.rel_l2(uh, u_ref) <= u_tol, (name, p0)
        assert so.rel_l2(uh, so.plain_sum(G[:, c0:c1].float().cpu().numpy())) <= u_tol, (name, p0)
        rms_w = float(np.sqrt(np.mean(u_ref * u_ref)))
        assert float((np.abs(uh - u_ref) / (np.abs(u_ref) + rms_w + 1e-300)).max()) <= 8.0 * u_tol, (name, p0)

    # every coordinate: u against the fp64 column sum of G computed by torch on the device, in the norm and one by one
    # (each within 8 u_tol of its own magnitude + the rms of the aggregate: a single wrong coordinate is off by about one rms)
    num = 0.0
    den = 0.0
    blk = 1 << 22
    for c0 in range(0, d, blk):
        ref = G[:, c0:c0 + blk].sum(dim=0, dtype=torch.float64)
        diff = u[c0:c0 + blk].double() - ref
        num += float((diff * diff).sum())
        den += float((ref * ref).sum())
    rel = (num / den) ** 0.5
    rms = (den / d) ** 0.5
    worst = 0.0
    for c0 in range(0, d, blk):
        ref = G[:, c0:c0 + blk].sum(dim=0, dtype=torch.float64)
        worst = max(worst, float(((u[c0:c0 + blk].double() - ref).abs() / (ref.abs() + rms)).max()))
    say("  rel_l2(u, G 1_P) over all d = %.3e, worst coordinate %.3e of (|u_c| + rms)" % (rel, worst), round(time.time() - t_start, 1), "s")
    assert rel <= u_tol and worst <= 8.0 * u_tol
    del G, Z, R, u, f
    torch.cuda.empty_cache()
