"""Benchmark of the Solon hot path on one MI355X: encode -> locate -> decode per step.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config C5] [--also C4,C3,C2,X1] [--no-cpu-baseline]

A step is one pass of the whole path over one batch of synthetic gradients that are already resident in
HBM: solon_encode (G -> Z), then phi and psi (R, f -> V, u) on one stream - by default through solon_locate_decode,
which does both in one pass over R; --two-pass times solon_locate and solon_decode as separate calls instead (the
default run also reports those, from a few extra steps outside the timed region).
R is the encoder's output with the configuration's Byzantine rows overwritten; that harness step runs once,
before the timed region, into its own buffer, so each timed step moves exactly the method's bytes.  Every step
projects with a fresh f (drawn before the timed region).
Prints ONE JSON line (metric, value, roofline of the dominant kernel, CPU-oracle baseline).  Throughput is given twice:
against the ALGORITHMIC bytes of the three passes (encode, locate, decode: the numerator the metric is defined on) and
against the bytes the timed calls really MOVE (the one-pass path reads R once: fewer bytes in the same time).
`redo_path_ms` is the one-pass call when its guess of the honest rows is wrong and the recombination runs twice.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0


def algorithmic_bytes(cfg, plan):
    """Bytes the method must move per step on one device (each gradient read once, each message written
    once and inspected once, m honest rows per group recombined into u)."""
    bG = 2 if cfg["dtype"] == "bf16" else 4
    P, d, d_c, q, m = cfg["P"], cfg["d"], plan.d_c, plan.q, cfg["m"]
    enc = P * d * bG + P * d_c * 4
    loc = P * d_c * 4 + d_c * 4
    dec = q * m * d_c * 4 + d * 4
    return dict(encode=enc, locate=loc, decode=dec, total=enc + loc + dec)


def moved_bytes(cfg, plan, one_pass):
    """Bytes the timed calls move.  Two passes: the algorithmic bytes.  One pass: R and f once, u once, plus the sample
    projection behind the guess (2^17 columns of every row)."""
    ab = algorithmic_bytes(cfg, plan)
    if not one_pass:
        return dict(encode=ab["encode"], locate_decode=ab["locate"] + ab["decode"], total=ab["total"])
    P, d, d_c = cfg["P"], cfg["d"], plan.d_c
    sample = min(d_c, 1 << 17)
    ld = P * d_c * 4 + d_c * 4 + d * 4 + (P + 1) * sample * 4
    return dict(encode=ab["encode"], locate_decode=ld, total=ab["encode"] + ld)


def run_config(name, steps, warmup, want_cpu_baseline, cfg=None, check_sum=False, two_pass=False, events_in_timed_steps=True):
    import numpy as np
    import torch

    import paper_2110_01595_amd as solon
    import workloads

    dev = torch.device("cuda:0")
    if cfg is None:
        cfg = workloads.CONFIGS[name]
        sd = workloads.seeds(name)
    else:
        sd = dict(G=1, f=2, byz=3, attack=4)
    P, s, m, d = cfg["P"], cfg["s"], cfg["m"], cfg["d"]
    plan = solon.Plan(P, s, m, d, dtype=solon.SOLON_BF16 if cfg["dtype"] == "bf16" else solon.SOLON_F32)
    d_c = plan.d_c
    G = workloads.make_gradients(cfg, dev, sd["G"])
    ld = (d_c + 63) // 64 * 64                             # rows of Z and R start on 256-byte boundaries
    Z = torch.empty((P, ld), dtype=torch.float32, device=dev)[:, :d_c]
    u = torch.empty(d, dtype=torch.float32, device=dev)
    fs = [workloads.make_projection(d_c, dev, sd["f"] + 100 * k) for k in range(min(steps, 32))]   # a fresh f every step
    f = fs[0]
    byz = workloads.pick_byzantine(P, s, sd["byz"])
    solon.solon_encode(plan, G, Z)
    R = torch.empty((P, ld), dtype=torch.float32, device=dev)[:, :d_c]
    R.copy_(Z)
    workloads.apply_attack(R, byz, cfg["attack"], sd["attack"])
    torch.cuda.synchronize()

    def step(events=None, one_pass=not two_pass, f=f, all_events=True):
        """events: [before encode, after encode, after locate (or the one-pass call), after decode]; with all_events=False
        only the first two are recorded (every record is a marker in the stream: a few microseconds of a small step)."""
        if events is not None:
            events[0].record()
        solon.solon_encode(plan, G, Z)
        if events is not None:
            events[1].record()
        if one_pass:                                         # phi and psi in one pass over R
            solon.solon_locate_decode(plan, R, f, u, want_host=False)
            if events is not None and all_events:
                events[2].record()
        else:
            solon.solon_locate(plan, R, f, want_host=False)
            if events is not None and all_events:
                events[2].record()
            solon.solon_decode(plan, R, u)
        if events is not None and all_events:
            events[3].record()

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(steps)]
    torch.cuda.synchronize()
    # the timed region: K steps by the wall clock, with HIP events around the dominant kernel's call (solon_encode) only;
    # the other phase is the rest of the step (two_pass runs record every phase)
    # (events_in_timed_steps = False: the timed steps carry no events at all - two records cost a 0.28 ms step 3 % - and the
    # encoder is timed in separate steps after them; the headline workload keeps its events inside the timed region)
    in_loop = events_in_timed_steps or two_pass
    t0 = time.perf_counter()
    for k in range(steps):
        step(ev[k] if in_loop else None, f=fs[k % len(fs)], all_events=two_pass)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    if not in_loop:
        ev = ev[:max(5, steps // 2)]
        for k, e in enumerate(ev):
            step(e, f=fs[k % len(fs)], all_events=False)
        torch.cuda.synchronize()
    status = solon.solon_decode_status(plan)
    one_pass = (not two_pass) and plan.query(solon.SOLON_Q_LAST_ONE_PASS) == 1
    redone = plan.query(solon.SOLON_Q_LAST_REDO) if one_pass else 0
    located_ok = status == 0
    for fk in (fs[0], fs[-1]):                           # after the timed region: the located set, for the record
        V, _ = solon.solon_locate(plan, R, fk)
        located_ok = located_ok and V == byz
    ms_step = (t1 - t0) * 1e3 / steps
    if two_pass:
        phase = np.array([[e[i].elapsed_time(e[i + 1]) for i in range(3)] for e in ev])   # ms
        enc_ms, loc_ms, dec_ms = phase.mean(axis=0).tolist()
    else:
        enc_ms = float(np.mean([e[0].elapsed_time(e[1]) for e in ev]))
        loc_ms, dec_ms = ms_step - enc_ms, 0.0               # everything of a step that is not the encoder: the one-pass call (and the gaps)
    enc_all = sorted(e[0].elapsed_time(e[1]) for e in ev)
    enc_stats = dict(mean=enc_ms, median=enc_all[len(enc_all) // 2], min=enc_all[0], max=enc_all[-1])
    ab = algorithmic_bytes(cfg, plan)
    if not two_pass:                                         # for the record: the two separate passes, a few steps
        ev2 = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(max(3, steps // 4))]
        step(one_pass=False)
        for e in ev2:
            step(e, one_pass=False)
        torch.cuda.synchronize()
        two = np.array([[e[i].elapsed_time(e[i + 1]) for i in range(3)] for e in ev2]).mean(axis=0).tolist()
    mb = moved_bytes(cfg, plan, one_pass)
    res = dict(
        workload=name, P=P, s=s, m=m, d=d, d_c=d_c, q=plan.q, r=plan.r, grad_dtype=cfg["dtype"], attack=cfg["attack"],
        located_ok=located_ok, ms_per_step=ms_step,
        coords_per_s=P * d / (ms_step * 1e-3),
        effective_GBps=ab["total"] / (ms_step * 1e-3) / 1e9,
        pct_of_peak=100.0 * ab["total"] / (ms_step * 1e-3) / 1e9 / PEAK_HBM_GBS,
        algorithmic_bytes=ab,
        path="encode + " + ("locate + decode (two passes)" if two_pass else "locate_decode (one pass over R)" if one_pass
                            else "locate_decode (fell back to two passes: m not in {1, 2, 4} or input too small)"),
        bytes_moved=mb, GBps_moved=mb["total"] / (ms_step * 1e-3) / 1e9,
        pct_of_peak_moved=100.0 * mb["total"] / (ms_step * 1e-3) / 1e9 / PEAK_HBM_GBS,
        fresh_f_per_step=len(fs), recombination_repeated_in_last_step=bool(redone), encode_ms_over_steps=enc_stats,
        encode_events="around solon_encode in every timed step" if in_loop else "in %d separate steps after the timed ones (the timed steps carry no events)" % len(ev),
    )
    if two_pass:
        res["phase_ms"] = dict(encode=enc_ms, locate=loc_ms, decode=dec_ms)
        res["phase_GBps"] = dict(encode=ab["encode"] / enc_ms / 1e6, locate=ab["locate"] / loc_ms / 1e6, decode=ab["decode"] / dec_ms / 1e6)
        res["phase_GBps_moved"] = res["phase_GBps"]
    else:
        res["phase_ms"] = dict(encode=enc_ms, locate_decode=loc_ms)
        res["phase_GBps"] = dict(encode=ab["encode"] / enc_ms / 1e6, locate_decode=(ab["locate"] + ab["decode"]) / loc_ms / 1e6)
        res["phase_GBps_moved"] = dict(encode=mb["encode"] / enc_ms / 1e6, locate_decode=mb["locate_decode"] / loc_ms / 1e6)
        res["two_pass_phase_ms"] = dict(encode=two[0], locate=two[1], decode=two[2])
        two_ms = sum(two)
        res["two_pass"] = dict(ms_per_step=two_ms, GBps=ab["total"] / two_ms / 1e6, pct_of_peak=100.0 * ab["total"] / two_ms / 1e6 / PEAK_HBM_GBS)
    if one_pass:
        # worst case of the one-pass call: the guess of the honest rows is wrong (here: made blind, with the first node of
        # group 0 - which a clean group's choice always takes - among the corrupted) and the recombination runs twice
        first = int(plan.groups().tolist().index(0))
        byz_w = sorted(set([first] + [j for j in byz if j != first][: max(0, s - 1)]))
        R.copy_(Z)
        workloads.apply_attack(R, byz_w, cfg["attack"], sd["attack"])
        solon.solon_tune("fuse_blind_guess", 1)
        try:
            solon.solon_locate_decode(plan, R, f, u, want_host=False)
            n_redo = max(3, steps // 4)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for k in range(n_redo):
                solon.solon_locate_decode(plan, R, fs[k % len(fs)], u, want_host=False)
            e1.record()
            torch.cuda.synchronize()
            res["redo_path_ms"] = dict(locate_decode=e0.elapsed_time(e1) / n_redo, step=enc_ms + e0.elapsed_time(e1) / n_redo,
                                       recombination_repeated=bool(plan.query(solon.SOLON_Q_LAST_REDO)),
                                       located_ok=(solon.solon_locate(plan, R, f)[0] == byz_w))
        finally:
            solon.solon_tune("fuse_blind_guess", 0)
    if check_sum:   # Def. 1 of the paper over every coordinate: u against the fp64 column sum of G (torch, on the device)
        num = den = 0.0
        for c0 in range(0, d, 1 << 22):
            ref = G[:, c0:c0 + (1 << 22)].sum(dim=0, dtype=torch.float64)
            diff = u[c0:c0 + (1 << 22)].double() - ref
            num += float((diff * diff).sum())
            den += float((ref * ref).sum())
        res["rel_l2_u_vs_plain_sum"] = (num / den) ** 0.5
    cpu = None
    if want_cpu_baseline:
        if one_pass:                                          # the redo measurement changed R: back to the configuration's attack
            R.copy_(Z)
            workloads.apply_attack(R, byz, cfg["attack"], sd["attack"])
        cpu = cpu_baseline(cfg, plan, G, R, f, byz)
    del G, Z, R, u, f, fs
    torch.cuda.empty_cache()
    return res, cpu


def cpu_baseline(cfg, plan, G, R, f, byz):
    """The fp64 oracle as it stands, timed on the host on a bounded sample of the same workload: consecutive
    windows of W chunks of every row (all P nodes, all steps of the path).  Two legs of about 10 s each: one thread,
    and all host cores (one window per worker thread at a time - the oracle's numpy calls release the interpreter
    lock - with numpy's own thread pool held at one thread in both legs, so that `cores` is what actually ran)."""
    import concurrent.futures as cf

    import numpy as np
    from threadpoolctl import threadpool_limits

    from oracle import solon_oracle as so

    P, s, m = cfg["P"], cfg["s"], cfg["m"]
    W = int(min(plan.d_c, max(1024, 4.0e8 // (P * m))))      # about 4e8 per-batch coordinates per window
    oplan = so.make_plan(P, s, m)
    nwin_max = -(-plan.d_c // W)

    def load(k, W=W):
        p0 = k * W
        p1 = min(plan.d_c, p0 + W)
        c0, c1 = p0 * m, min(cfg["d"], p1 * m)
        return G[:, c0:c1].float().cpu().numpy(), R[:, p0:p1].cpu().numpy(), f[p0:p1].cpu().numpy(), c1 - c0

    def work(win):
        Gh, Rh, fh, n = win
        Zo = so.encode(oplan, Gh)
        rho = so.project(Rh, fh)
        V = so.locate(oplan, rho)
        uo = so.decode(oplan, Rh, V, n)
        return (V == byz) and so.rel_l2(uo, so.plain_sum(Gh)) < 1e-4 and Zo.shape == Rh.shape, P * n

    # leg 1: one thread
    spent, coords, nwin, ok = 0.0, 0, 0, True
    with threadpool_limits(limits=1):
        while spent < 10.0 and nwin < min(12, nwin_max):
            win = load(nwin)
            t0 = time.perf_counter()
            good, n = work(win)
            spent += time.perf_counter() - t0
            ok, coords, nwin = ok and good, coords + n, nwin + 1
            del win
    one = dict(value=coords / spent, unit="coords/s", cores=1, kind="oracle",
               sample="%d consecutive windows of %d chunks (of %d) of every row (P=%d rows), each one encode+project+locate+decode; "
                      "%.1f s of oracle time in total; located set %s" % (nwin, W, plan.d_c, P, spent, "matches" if ok else "MISMATCH"))
    # leg 2: all host cores (at most 16, the share of a one-GPU machine), sized from leg 1 to about 10 s
    # (windows of a quarter of the size, to bound host memory: every worker holds one window and its fp64 copies)
    cores = max(1, min(16, os.cpu_count() or 1))
    W2 = max(1024, W // 4)
    per_win = spent / max(1, nwin) * W2 / W
    rounds = max(1, min(int(10.0 / max(1.5 * per_win, 1e-3)), 8))
    todo = cores * rounds
    wins = [load(k, W2) for k in range(min(cores, -(-plan.d_c // W2)))]   # loaded before the clock starts; later rounds reuse them
    with threadpool_limits(limits=1), cf.ThreadPoolExecutor(max_workers=cores) as pool:
        t0 = time.perf_counter()
        out = list(pool.map(work, [wins[k % len(wins)] for k in range(todo)]))
        wall = time.perf_counter() - t0
    one["all_cores"] = dict(value=sum(n for _, n in out) / wall, unit="coords/s", cores=min(cores, todo), kind="oracle",
                            sample="%d windows of %d chunks on %d worker threads, %.1f s wall; results %s"
                                   % (todo, W2, min(cores, todo), wall, "match" if all(g for g, _ in out) else "MISMATCH"))
    return one


# Shapes of the paper's own cost study (time-breakdown figures of Sec. 4 and of the appendix): P = 100 nodes,
# s = 5 with r_c in {2, 4, 6, 8, 10}, and r_c = 10 with s in {1..5}, on the three model sizes of Table 1.
PAPER_MODELS = {"ResNet18": 11_173_000, "VGG13": 9_923_000, "LSTM": 7_332_000}


def sweep_paper_shapes(steps, warmup):
    shapes = [(5, m) for m in (2, 4, 6, 8, 10)] + [(s, 10) for s in (1, 2, 3, 4)]
    for model, d in PAPER_MODELS.items():
        for s, m in shapes:
            cfg = dict(P=100, s=s, m=m, d=d, dtype="f32", dist="normal", sigma=0.01, attack="paper")
            name = "%s_P100_s%d_m%d" % (model, s, m)
            r, _ = run_config(name, steps, warmup, False, cfg=cfg, check_sum=True, events_in_timed_steps=False)
            keep = ("workload", "P", "s", "m", "d", "q", "r", "ms_per_step", "coords_per_s", "effective_GBps", "phase_ms", "phase_GBps",
                    "located_ok", "rel_l2_u_vs_plain_sum")
            print(json.dumps({k: r[k] for k in keep}), flush=True)


def sweep_conditioning():
    """How far the compression ratio can go on an fp32 wire (the paper reports numerical trouble beyond r_c = 14):
    m = 6..16 with s in {1, 3, 5}, four groups of r = 2s + m nodes, all s corrupted nodes in group 0 (the paper's
    reverse-gradient and constant attacks), three seeds each.  Per shape: is the located set the planted one and the one
    brute force finds (oracle, on the HIP path's projections); the largest honest residual of the locator's fit in units
    of tau; rel-L2 and worst coordinate of u against the plain sum over all d (fp64 on the device), next to the rel-L2 of
    the ORACLE's decode (fp64 least squares over all honest rows) of the same fp32 messages on a window - the error the
    code itself leaves on this wire, whatever decodes it."""
    import numpy as np
    import torch

    import paper_2110_01595_amd as solon
    import workloads
    from oracle import solon_oracle as so

    dev = torch.device("cuda:0")
    for m in range(6, 17):
        for s in (1, 3, 5):
            r = 2 * s + m
            P, d = 4 * r, m * (1 << 18)
            cfg = dict(P=P, s=s, m=m, d=d, dtype="f32", dist="normal", sigma=0.01, attack="paper")
            plan = solon.Plan(P, s, m, d)
            oplan = so.make_plan(P, s, m)
            out = dict(m=m, s=s, r=r, P=P, d=d, located_planted=True, located_bruteforce=True, honest_residual_over_tau=0.0,
                       rel_l2_u=0.0, worst_coordinate=0.0, rel_l2_u_oracle_window=0.0, status_ok=True)
            for seed in range(3):
                G = workloads.make_gradients(cfg, dev, 100 + seed)
                Z = torch.empty((P, plan.d_c), dtype=torch.float32, device=dev)
                solon.solon_encode(plan, G, Z)
                byz = workloads.pick_byzantine(P, s, 200 + seed, within=oplan.nodes[0].tolist())
                R = workloads.apply_attack(Z, byz, "paper", 300 + seed)
                f = workloads.make_projection(plan.d_c, dev, 400 + seed)
                u = torch.empty(d, dtype=torch.float32, device=dev)
                try:
                    V, rho = solon.solon_locate(plan, R, f, want_rho=True)
                    solon.solon_decode(plan, R, u)
                    out["status_ok"] = out["status_ok"] and solon.solon_decode_status(plan) == 0
                except solon.SolonError:
                    V, rho = None, None
                    out["status_ok"] = False
                out["located_planted"] = out["located_planted"] and V == byz
                if rho is not None:
                    try:
                        out["located_bruteforce"] = out["located_bruteforce"] and so.locate(oplan, rho, "bruteforce_stacked") == V
                    except so.OracleError:
                        out["located_bruteforce"] = False
                    for g in range(oplan.q):
                        idx = oplan.nodes[g]
                        hon = [j for j in idx if j not in byz]
                        wg = oplan.w.astype(np.float64)
                        y = rho / np.median(np.abs(rho[idx]))
                        coef = np.linalg.lstsq(np.polynomial.chebyshev.chebvander(wg[hon], m - 1), y[hon], rcond=None)[0]
                        res = np.abs(np.polynomial.chebyshev.chebval(wg[hon], coef) - y[hon]).max()
                        out["honest_residual_over_tau"] = max(out["honest_residual_over_tau"], float(res / so.TAU))
                if V == byz and out["status_ok"]:
                    num = den = 0.0
                    worst = 0.0
                    refs = []
                    for c0 in range(0, d, 1 << 22):
                        ref = G[:, c0:c0 + (1 << 22)].sum(dim=0, dtype=torch.float64)
                        diff = u[c0:c0 + (1 << 22)].double() - ref
                        num += float((diff * diff).sum())
                        den += float((ref * ref).sum())
                        refs.append((ref, diff))
                    rms = (den / d) ** 0.5
                    for ref, diff in refs:
                        worst = max(worst, float((diff.abs() / (ref.abs() + rms)).max()))
                    out["rel_l2_u"] = max(out["rel_l2_u"], (num / den) ** 0.5)
                    out["worst_coordinate"] = max(out["worst_coordinate"], worst)
                    del refs
                    win = 4096
                    u_or = so.decode(oplan, R[:, :win].cpu().numpy(), byz, win * m)
                    out["rel_l2_u_oracle_window"] = max(out["rel_l2_u_oracle_window"],
                                                        so.rel_l2(u_or, so.plain_sum(G[:, :win * m].cpu().numpy())))
                del G, Z, R, f, u
            torch.cuda.empty_cache()
            print(json.dumps(out), flush=True)


def sweep_two_streams(steps, warmup):
    """Two independent rounds (two jobs served by the same GPU: own plan, gradients, messages, f, u) issued on ONE stream one
    after the other, and on TWO streams side by side.  Every phase is bound by the same HBM, so the streams can only fill each
    other's gaps: launch latencies, the latency-bound solves, ramp-up and drain of every kernel."""
    import torch

    import paper_2110_01595_amd as solon
    import workloads

    dev = torch.device("cuda:0")
    shapes = [(n, workloads.CONFIGS[n], workloads.seeds(n)) for n in ("C5", "C4", "C3", "C2", "X1")]
    shapes.append(("LSTM_P100_s5_m10", dict(P=100, s=5, m=10, d=7_332_000, dtype="f32", dist="normal", sigma=0.01, attack="paper"), dict(G=1, f=2, byz=3, attack=4)))
    for name, cfg, sd in shapes:
        P, s, m, d = cfg["P"], cfg["s"], cfg["m"], cfg["d"]
        jobs = []
        for j in range(2):
            plan = solon.Plan(P, s, m, d, dtype=solon.SOLON_BF16 if cfg["dtype"] == "bf16" else solon.SOLON_F32)
            d_c = plan.d_c
            G = workloads.make_gradients(cfg, dev, sd["G"] + 50 * j)
            ld = (d_c + 63) // 64 * 64
            Z = torch.empty((P, ld), dtype=torch.float32, device=dev)[:, :d_c]
            R = torch.empty((P, ld), dtype=torch.float32, device=dev)[:, :d_c]
            u = torch.empty(d, dtype=torch.float32, device=dev)
            f = workloads.make_projection(d_c, dev, sd["f"] + 50 * j)
            byz = workloads.pick_byzantine(P, s, sd["byz"] + 50 * j)
            solon.solon_encode(plan, G, Z)
            R.copy_(Z)
            workloads.apply_attack(R, byz, cfg["attack"], sd["attack"] + 50 * j)
            jobs.append(dict(plan=plan, G=G, Z=Z, R=R, u=u, f=f, byz=byz))
        torch.cuda.synchronize()

        def round_(job):
            solon.solon_encode(job["plan"], job["G"], job["Z"])
            solon.solon_locate_decode(job["plan"], job["R"], job["f"], job["u"], want_host=False)

        streams = [torch.cuda.Stream(), torch.cuda.Stream()]
        ms = {}
        ref = None
        for mode in ("one_stream", "two_streams"):
            def both():
                for j, job in enumerate(jobs):
                    if mode == "two_streams":
                        with torch.cuda.stream(streams[j]):
                            round_(job)
                    else:
                        round_(job)
            for _ in range(warmup):
                both()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                both()
            torch.cuda.synchronize()
            ms[mode] = (time.perf_counter() - t0) * 1e3 / steps / 2          # per round
            ok = all(solon.solon_decode_status(job["plan"]) == 0 for job in jobs)
            got = [job["u"].clone() for job in jobs]
            if ref is None:
                ref = got
            same = all(torch.equal(a, b) for a, b in zip(ref, got))
        ab = algorithmic_bytes(cfg, jobs[0]["plan"])
        print(json.dumps(dict(workload=name, ms_per_round=ms, speedup=ms["one_stream"] / ms["two_streams"],
                              pct_of_peak={k: ab["total"] / (v * 1e-3) / 1e9 / PEAK_HBM_GBS * 100 for k, v in ms.items()},
                              status_ok=ok, same_u_both_ways=same)), flush=True)
        del jobs
        torch.cuda.empty_cache()


def sweep_graph(steps, warmup):
    """A step (solon_encode + solon_locate_decode) launched eagerly and replayed from a HIP graph captured once: what the gaps
    between the six to nine launches of a step cost at the small shapes."""
    import torch

    import paper_2110_01595_amd as solon
    import workloads

    dev = torch.device("cuda:0")
    shapes = [(n, workloads.CONFIGS[n], workloads.seeds(n)) for n in ("C2", "C3", "X1")]
    shapes.append(("LSTM_P100_s5_m10", dict(P=100, s=5, m=10, d=7_332_000, dtype="f32", dist="normal", sigma=0.01, attack="paper"), dict(G=1, f=2, byz=3, attack=4)))
    shapes.append(("C5", workloads.CONFIGS["C5"], workloads.seeds("C5")))
    for name, cfg, sd in shapes:
        P, s, m, d = cfg["P"], cfg["s"], cfg["m"], cfg["d"]
        plan = solon.Plan(P, s, m, d, dtype=solon.SOLON_BF16 if cfg["dtype"] == "bf16" else solon.SOLON_F32)
        d_c = plan.d_c
        G = workloads.make_gradients(cfg, dev, sd["G"])
        ld = (d_c + 63) // 64 * 64
        Z = torch.empty((P, ld), dtype=torch.float32, device=dev)[:, :d_c]
        R = torch.empty((P, ld), dtype=torch.float32, device=dev)[:, :d_c]
        u = torch.empty(d, dtype=torch.float32, device=dev)
        f = workloads.make_projection(d_c, dev, sd["f"])
        byz = workloads.pick_byzantine(P, s, sd["byz"])
        solon.solon_encode(plan, G, Z)
        R.copy_(Z)
        workloads.apply_attack(R, byz, cfg["attack"], sd["attack"])

        def step():
            solon.solon_encode(plan, G, Z)
            solon.solon_locate_decode(plan, R, f, u, want_host=False)

        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        eager = (time.perf_counter() - t0) * 1e3 / steps
        u_eager = u.clone()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                step()
        torch.cuda.current_stream().wait_stream(side)
        for _ in range(warmup):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            graph.replay()
        torch.cuda.synchronize()
        replay = (time.perf_counter() - t0) * 1e3 / steps
        ab = algorithmic_bytes(cfg, plan)
        print(json.dumps(dict(workload=name, ms_per_step=dict(eager=eager, graph_replay=replay), speedup=eager / replay,
                              pct_of_peak={k: ab["total"] / (v * 1e-3) / 1e9 / PEAK_HBM_GBS * 100 for k, v in (("eager", eager), ("graph_replay", replay))},
                              same_u=bool(torch.equal(u, u_eager)), status_ok=solon.solon_decode_status(plan) == 0)), flush=True)
        del G, Z, R, u, f, graph
        torch.cuda.empty_cache()


def sweep_repetition(steps, warmup):
    """m = 1 (repetition code): the general locate + decode path next to the majority-vote decoder, same inputs."""
    import torch

    import paper_2110_01595_amd as solon
    import workloads

    dev = torch.device("cuda:0")
    for P, s, d in ((63, 3, 25_600_000), (100, 5, 11_173_000), (15, 1, 11_200_000)):
        cfg = dict(P=P, s=s, m=1, d=d, dtype="f32", dist="normal", sigma=0.01, attack="mix")
        plan = solon.Plan(P, s, 1, d)
        G = workloads.make_gradients(cfg, dev, 1)
        ld = (d + 63) // 64 * 64
        R = torch.empty((P, ld), dtype=torch.float32, device=dev)[:, :d]
        solon.solon_encode(plan, G, R)
        byz = workloads.pick_byzantine(P, s, 3)
        workloads.apply_attack(R, byz, "mix", 4)
        f = workloads.make_projection(d, dev, 2)
        u1 = torch.empty(d, dtype=torch.float32, device=dev)
        u2 = torch.empty(d, dtype=torch.float32, device=dev)

        def general():
            solon.solon_locate(plan, R, f, want_host=False)
            solon.solon_decode(plan, R, u1)

        def majority():
            solon.solon_decode_majority(plan, R, u2, want_host=False)

        times = {}
        for name, fn in (("locate+decode", general), ("majority", majority)):
            for _ in range(warmup):
                fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(steps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            times[name] = e0.elapsed_time(e1) / steps
        V1, _ = solon.solon_locate(plan, R, f)
        V2 = solon.solon_decode_majority(plan, R, u2)
        same = float((u1 - u2).norm() / u2.norm())
        bytes_general = P * d * 4 + d * 4 + plan.q * d * 4 + d * 4
        bytes_majority = P * d * 4 + d * 4
        print(json.dumps(dict(workload="repetition_P%d_s%d_d%d" % (P, s, d), q=plan.q, ms=times,
                              GBps={"locate+decode": bytes_general / times["locate+decode"] / 1e6,
                                    "majority": bytes_majority / times["majority"] / 1e6},
                              located_equal=(V1 == V2 == byz), rel_l2_between_paths=same)), flush=True)
        del G, R, f, u1, u2
        torch.cuda.empty_cache()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="C5")
    ap.add_argument("--also", default="C4,C3,C2,X1", help="comma-separated further workloads reported inside the same line ('' = none)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--two-pass", action="store_true", help="time solon_locate + solon_decode instead of solon_locate_decode")
    ap.add_argument("--tune", action="append", default=[], metavar="KEY=INT",
                    help="launch-shape knob passed to solon_tune before the run (measurement aid; may be repeated)")
    ap.add_argument("--sweep", choices=["paper", "repetition", "conditioning", "two_streams", "graph"], default=None,
                    help="instead of the headline line: 'paper' runs the paper's cost-study shapes, 'repetition' compares the "
                         "m = 1 majority-vote decoder with the general path, 'conditioning' takes the compression ratio up to "
                         "16 and records where located set and decode error leave the bar, 'two_streams' times two independent rounds on one "
                         "stream and on two, 'graph' a step launched eagerly and replayed from a HIP graph; one JSON line per shape")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="first run one plain device copy of 4 GiB (reads 4 GiB, writes 4 GiB): the dispatch whose rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE readings scale the counters of the other kernels")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: the path has no collectives and every box has one GPU (--gpus %d refused)" % args.gpus)

    import paper_2110_01595_amd as solon
    solon.lib()                                              # fail loudly if the HIP library is missing
    for kv in args.tune:
        key, val = kv.split("=")
        solon.solon_tune(key, int(val))

    if args.calibrate_copy:
        import torch
        src = torch.ones(1 << 30, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)                                       # elementwise copy kernel, 2^32 bytes each way
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()

    if args.sweep == "paper":
        sweep_paper_shapes(args.steps, args.warmup)
        return
    if args.sweep == "repetition":
        sweep_repetition(args.steps, args.warmup)
        return
    if args.sweep == "conditioning":
        sweep_conditioning()
        return
    if args.sweep == "two_streams":
        sweep_two_streams(args.steps, args.warmup)
        return
    if args.sweep == "graph":
        sweep_graph(args.steps, args.warmup)
        return

    main_res, cpu = run_config(args.config, args.steps, args.warmup, not args.no_cpu_baseline, two_pass=args.two_pass)
    others = []
    for name in [n for n in args.also.split(",") if n and n != args.config]:
        r, _ = run_config(name, args.steps, args.warmup, False, two_pass=args.two_pass, events_in_timed_steps=False)
        others.append(r)

    enc_bytes = main_res["algorithmic_bytes"]["encode"]
    enc_s = main_res["phase_ms"]["encode"] * 1e-3
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        traffic = json.load(open(tpath)).get(args.config, {}).get("encode_bytes_per_launch")
    line = {
        "metric": "encode+decode gradient coords/sec and achieved HBM GB/s (% of peak), 1 GPU",
        "value": main_res["coords_per_s"], "unit": "coords/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": main_res["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": args.config, **{k: main_res[k] for k in ("P", "s", "m", "d", "d_c", "q", "r", "grad_dtype", "attack")}},
        "path": main_res["path"],
        "effective_GBps": main_res["effective_GBps"], "pct_of_peak": main_res["pct_of_peak"],
        "bytes_algorithmic": main_res["algorithmic_bytes"], "bytes_moved": main_res["bytes_moved"],
        "GBps_moved": main_res["GBps_moved"], "pct_of_peak_moved": main_res["pct_of_peak_moved"],
        "phase_ms": main_res["phase_ms"], "phase_GBps": main_res["phase_GBps"], "phase_GBps_moved": main_res["phase_GBps_moved"],
        "two_pass_phase_ms": main_res.get("two_pass_phase_ms"), "two_pass": main_res.get("two_pass"),
        "redo_path_ms": main_res.get("redo_path_ms"), "fresh_f_per_step": main_res["fresh_f_per_step"],
        "encode_ms_over_steps": main_res["encode_ms_over_steps"], "encode_events": main_res["encode_events"],
        "located_ok": main_res["located_ok"],
        "roofline": {"kernel": "encode_phase_kernel (solon_encode; the persistent phase-separated encoder serves this size)", "bound": "hbm", "achieved": enc_bytes / enc_s / 1e9,
                     "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": enc_bytes / enc_s / 1e9 / PEAK_HBM_GBS, "traffic": traffic,
                     "traffic_source": "profiles/traffic.json: FETCH_SIZE + WRITE_SIZE of a separate rocprofv3 --pmc run of this command, not measured in this run"},
        "cpu_baseline": cpu,
        "also": [{k: r.get(k) for k in ("workload", "path", "ms_per_step", "coords_per_s", "effective_GBps", "pct_of_peak", "GBps_moved",
                                        "pct_of_peak_moved", "phase_ms", "phase_GBps", "phase_GBps_moved", "redo_path_ms", "located_ok", "encode_events")
                  + (() if args.two_pass else ("two_pass_phase_ms",))} for r in others],
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
