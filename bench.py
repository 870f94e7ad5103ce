#!/usr/bin/env python3
"""Benchmark of the R-FAST activation round on one MI355X.

A step is one round of the whole hot path (resolver + state update + local
gradients) over one batch of synthetic input that is already resident in HBM.
The default workload is config 2 (n=16 bidirectional ring, diagonal quadratic,
p = 11.2 M, every node active), the configuration the HBM-roofline target is
quoted on.  Prints ONE JSON line.

Three legs, all on the same context, one after the other:
  1. W warm-up rounds, then the K timed rounds as one rfast_run call (wall clock between two
     device synchronisations): `value`, `ms_per_step`.
  2. the next K rounds once more with HIP events around every launch on the library's stream, in
     calls cut where the counters and stamps can be read between launches: `roofline` of the kernel
     that ran them.  A launch of the multi-round kernel is priced against whichever of its two needs
     takes longer at the published peaks: the method's arithmetic (40 flop per coordinate and
     node-update, 157.3 TFLOP/s) or the bytes it moves (8 TB/s), the bytes computed from the counters
     and stamps read before and after the launch by the rules the kernel moves its tiles by.  Rounds
     that run one pass over HBM each are priced in bytes, counted per round from the stamps that moved.
  3. (where leg 2 ran several rounds per launch) up to 20 further rounds with one kernel pass per
     round (rfast_use_blocks off), events around every pass: `roofline_one_pass`, the HBM view of
     `rfast_state_kernel<FUSED>`.
Nothing in the output is a constant taken from a file, except `traffic` (HBM bytes counted by
rocprofv3 --pmc in a run of its own, see profiles/), which is carried only when the summary
names the same kernel, workload and launch length, and is labelled as not measured here.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

HBM_PEAK_GBS = 8000.0        # MI355X, published
FP32_VECTOR_PEAK_TFLOPS = 157.3
REBASE_INTERVAL = 512        # rounds between rebases of the running sums (set below; also the library's default)
FLOPS_PER_COORDINATE = 40.0  # Algorithm 1 with two in-edges per graph: 21; the float side of the Gaussian noise: the rest


def degrees(w):
    Rd, Cd = w.R.dense(), w.C.dense()
    return (Rd != 0).sum(axis=1) - 1, (Cd != 0).sum(axis=1) - 1, (Cd != 0).sum(axis=0) - 1   # dR, dI, dO


def algorithmic_bytes_per_round(w, active_counts, layout=False):
    """Literal traffic of Algorithm 1 per node-update: 7 + dR + 3 dI + 2 dO fp32 words
    per coordinate (reads x, z, g_prev, dR v's, dI rho's, dI rho~'s, dO current rho's;
    writes x, z, g, v, dO new rho's, dI rho~'s), plus the objective data (h, c) of the
    diagonal quadratic, or the re-read of g_new by the split mix/track pair.
    layout=True: the words this library's layout has to move (one running sum per
    sender instead of one per out-edge: 2 words instead of 2 dO; no write of the S4
    buffer; no stored sample for the separable objective), skips not credited."""
    dR, dI, dO = degrees(w)
    push = 2 * np.minimum(dO, 1) if layout else 2 * dO
    words = 7 + dR + 3 * dI + push + (2 if w.objective == "diag_quadratic" else 1)
    if layout:
        words = words - dI      # the buffer of S4 is read from the sender's ring and (almost) never written
        if w.objective == "diag_quadratic":
            words = words - 2   # the old sample is recomputed from (x_i, t_i): g is neither read nor written
    return float((words * active_counts).sum() * 4.0 * w.p)


def edge_lists(w):
    """(sender, receiver) of the off-diagonal entries of R and C in CSR order (row = receiver)."""
    out = []
    for g in (w.R, w.C):
        src, dst = [], []
        for i in range(w.n):
            for k in range(g.rowptr[i], g.rowptr[i + 1]):
                if g.col[k] != i:
                    src.append(int(g.col[k]))
                    dst.append(i)
        out.append((np.array(src, dtype=np.int64), np.array(dst, dtype=np.int64)))
    return out


def read_stamps(gpu):
    return {"t": gpu.read("T_NODE").astype(np.int64), "tau_r": gpu.read("TAU_R").astype(np.int64),
            "tau_c": gpu.read("TAU_C").astype(np.int64)}


def one_pass_bytes(w, edges, before, after, active):
    """Bytes the state kernels move for one round that ran one pass (two for the objectives whose gradient kernels
    run between a mixing and a tracking pass), from the stamps before and after it.  Per active node and coordinate,
    separable objective (`rfast_state_kernel<FUSED>`): reads x, z, h, c, one v per in-edge of R, the node's own current
    running sum (if it has out-edges over C) and two running sums (the one consumed now, the one consumed last time)
    per in-edge of C whose stamp moved; writes x, z, v and the new running sum.  Other objectives (`<MIX>` then
    `<TRACK>`): x, z, the v's in and x, v out (softmax: plus the bf16 copy of the weights, half a word), then z, the old
    and the new sample, the own running sum and the two sums per moved edge in, z and the new running sum out.  (The
    rare copies of an S4 buffer that leaves its sender's ring are not counted.)"""
    dR, dI, dO = degrees(w)
    (_, _), (c_src, c_dst) = edges
    live = np.zeros(w.n, dtype=np.int64)
    moved = after["tau_c"] != before["tau_c"]
    np.add.at(live, c_dst[moved], 1)
    act = np.asarray(active).astype(bool)
    pushes = (dO > 0).astype(np.float64)
    if w.objective == "diag_quadratic":
        words = (4 + dR + pushes + 2 * live) + (3 + pushes)
    else:
        words = (2 + dR) + 2 + (0.5 if w.objective == "softmax_bf16" else 0.0) + (3 + pushes + 2 * live) + (1 + pushes)
    return float(words[act].sum()) * 4.0 * w.p


def multi_round_bytes(w, edges, before, after, rebased):
    """Bytes one launch of the multi-round kernel moves, from the counters and stamps before and after it,
    by the kernel's rules: of every node it reads x, z, h, c, the ring slots whose version a receiver could
    still pick up before the launch, and the S4 buffers that were outside their sender's ring; it writes x, z
    of the nodes it activated, the ring slots it wrote (or shifted) that a receiver can still pick up after
    the launch, and the S4 buffers that are outside their sender's ring then."""
    M = w.D + 2
    (r_src, _), (c_src, c_dst) = edges
    big = np.iinfo(np.int64).max
    rows_in = rows_out = 0
    for kind, src, tau0, tau1 in (("v", r_src, before["tau_r"], after["tau_r"]), ("s", c_src, before["tau_c"], after["tau_c"])):
        lo0, lo1 = np.full(w.n, big), np.full(w.n, big)
        np.minimum.at(lo0, src, tau0)
        np.minimum.at(lo1, src, tau1)
        for j in range(w.n):
            t0, te = int(before["t"][j]), int(after["t"][j])
            for m in range(M):
                ver0, ver1 = t0 - ((t0 - m) % M), te - ((te - m) % M)
                rows_in += ver0 >= lo0[j]
                shift = rebased and kind == "s" and lo1[j] != big
                rows_out += (ver1 > t0 or shift) and ver1 >= lo1[j]
    rows_in += 4 * w.n + int((before["tau_c"] < before["t"][c_src] - (M - 2)).sum())
    rows_out += 2 * int((after["t"] != before["t"]).sum()) + int((after["tau_c"] < after["t"][c_src] - (M - 2)).sum())
    return float(rows_in + rows_out) * 4.0 * w.p, int(rows_in), int(rows_out)


def counted_traffic(workload_name, kernel, rounds_per_launch):
    """HBM bytes per launch counted by rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE) in a run of its own, from the
    committed summary, if that summary is about this kernel, workload and launch length; else None."""
    path = os.path.join(ROOT, "profiles", f"{workload_name}_{kernel}_kernel_hbm_traffic.md")
    fields = {}
    try:
        with open(path) as f:
            for line in f:
                if ":" in line and not line.startswith(("#", "|", " ")):
                    k, v = line.split(":", 1)
                    fields[k.strip()] = v.strip()
    except OSError:
        return None
    try:
        if fields.get("workload") != workload_name or not fields.get("kernel", "").startswith(f"rfast_{kernel}_kernel"):
            return None
        return {"bytes_per_launch": float(fields[f"traffic_bytes_per_launch@{int(rounds_per_launch)}"]),
                "source": f"profiles/{os.path.basename(path)} (rocprofv3 --pmc run of its own on this workload, kernel and "
                          f"launch length; not measured in this run)"}
    except (KeyError, ValueError):
        return None


def _time_rounds(step, w, seconds_target):
    rounds, updates = 0, 0
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < seconds_target and rounds < w.rounds:
        q = w.sched.round(rounds)
        step(q)
        updates += int(q.active.sum())
        rounds += 1
    return rounds, updates, time.perf_counter() - t0


def cpu_baseline(w, seconds_target=8.0):
    """The fp64 oracles as they stand, on a coordinate subset of the same workload
    (the separable objective costs exactly its share on a subset).  For the
    separable objective: the plain-C oracle on all host threads (`value`), the
    same on one thread, and the NumPy oracle; otherwise the NumPy oracle only."""
    from oracle.from_workload import make_oracle
    if w.objective == "diag_quadratic":
        p_sub = min(w.p, 400_000)
        coords = np.arange(p_sub, dtype=np.int64) * (w.p // p_sub)
    else:
        coords, p_sub = None, w.p
    frac = p_sub / w.p
    what = f"the same schedule on {p_sub} of {w.p} coordinates (every {w.p // p_sub}-th), scaled by {frac:.4g}"
    orc = make_oracle(w, coords)
    rounds, updates, dt = _time_rounds(
        lambda q: orc.round(q.active, q.delay_R, q.delay_C, q.drop_R, q.drop_C, w.gamma, q.batch_idx), w, seconds_target)
    numpy_rate = updates * frac / dt
    out = {"value": numpy_rate, "unit": "node-updates/s", "cores": 1, "kind": "oracle",
           "param_elements_per_s": updates * p_sub / dt,
           "sample": f"{rounds} rounds of {what}; NumPy fp64 oracle, single thread"}
    if w.objective != "diag_quadratic":
        return out
    del orc
    from oracle.c_oracle import COracle, default_threads
    h, c = w.data["h"][:, coords], w.data["c"][:, coords]
    rates = {}
    for label, threads in (("one_thread", 1), ("all_threads", default_threads())):
        co = COracle(w.n, p_sub, w.R, w.C, w.D, w.burst, h, c, w.noise_std, w.noise_seed, threads=threads)
        r, u, t = _time_rounds(lambda q: co.round(q.active, q.delay_R, q.delay_C, q.drop_R, q.drop_C, w.gamma), w,
                               seconds_target)
        rates[label] = (u * frac / t, r, co.threads)
        co.close()
    val, r_all, cores = rates["all_threads"]
    return {"value": val, "unit": "node-updates/s", "cores": cores, "kind": "oracle",
            "param_elements_per_s": val * w.p,
            "sample": f"{r_all} rounds of {what}; plain-C fp64 oracle (gcc -O2 -fopenmp, OpenMP over the coordinates), "
                      f"{cores} threads; noise counters index the subset",
            "one_thread": {"value": rates["one_thread"][0], "rounds": rates["one_thread"][1]},
            "numpy_oracle": {"value": numpy_rate, "rounds": rounds, "cores": 1}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None,
                    help="timed rounds (default: the 500 rounds of config 2, the headline workload; 100 for the other configs)")
    ap.add_argument("--warmup", type=int, default=None,
                    help="untimed rounds before them (default 12 with config 2, so that the timed rounds end where launches are cut "
                         "anyway, at a multiple of 512 rounds; else 10)")
    ap.add_argument("--config", type=int, default=2)
    ap.add_argument("--p", type=int, default=0, help="override p (not the headline workload)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sync", action="store_true",
                    help="time the synchronous push-pull step (eq. (2)) on the same workload instead of the round")
    ap.add_argument("--generated", action="store_true",
                    help="generate the schedule on the device (rfast_run_generated) instead of uploading it")
    ap.add_argument("--graphs", action="store_true", help="with --generated: replay HIP graphs of 16 rounds")
    ap.add_argument("--momentum", type=float, default=0.0,
                    help="optimizer variant (not the headline workload): heavy-ball buffer, +2 words per coordinate")
    ap.add_argument("--weight-decay", type=float, default=0.0, help="optimizer variant: weight decay inside the gradient")
    ap.add_argument("--no-blocks", action="store_true",
                    help="one kernel pass per round even where several rounds per launch are possible")
    ap.add_argument("--force-blocks", action="store_true",
                    help="several rounds per launch wherever possible, also where streaming is faster (measurement)")
    ap.add_argument("--tile-group", type=int, default=0, help="wavefronts per workgroup of the multi-round kernel (0: automatic)")
    ap.add_argument("--one-pass-rounds", type=int, default=20,
                    help="rounds of the one-pass-per-round leg (roofline_one_pass); 0 skips it")
    ap.add_argument("--noise-std", type=float, default=None, help="override the gradient noise (not the headline workload)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="run only a plain 1 GiB device copy (10 launches): calibrates HBM byte counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives exist in it); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    if args.copy_probe:
        a = torch.full((1 << 28,), 1.0, dtype=torch.float32, device="cuda:0")
        b = torch.empty_like(a)
        for _ in range(10):
            b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe_bytes_read": a.numel() * 4, "copy_probe_bytes_written": a.numel() * 4, "launches": 10}))
        return
    from rfast_workloads import configs
    from rfast_workloads.device import make_gpu, upload_chunk
    import paper_2307_11617_amd as rf

    kw = {"p": args.p} if args.p else {}
    t_gen = time.perf_counter()
    w = configs.CONFIGS[args.config](**kw)
    gen_s = time.perf_counter() - t_gen
    # Config 2 is a run of 500 rounds: by default all of them are timed, as one launch of the multi-round kernel
    # (launches are cut at multiples of 512 rounds, so 12 warm-up rounds put the timed 500 into one launch).
    K = args.steps if args.steps is not None else (500 if args.config == 2 and not args.p else 100)
    W = args.warmup if args.warmup is not None else (12 if args.config == 2 and not args.p and args.steps is None else 10)
    if args.noise_std is not None:
        w.noise_std = args.noise_std
    separable = w.objective == "diag_quadratic"
    K1 = 0 if (args.sync or args.generated or not separable) else max(0, min(args.one_pass_rounds, K))
    gpu = make_gpu(w)
    if args.no_blocks:
        rf.rfast_use_blocks(gpu.ctx, False)
    if args.force_blocks:
        rf.rfast_use_blocks(gpu.ctx, 2)
    rf.rfast_set_rebase_interval(gpu.ctx, REBASE_INTERVAL)
    if args.tile_group:
        rf.rfast_set_tile_group(gpu.ctx, args.tile_group)
    variant = args.momentum != 0.0 or args.weight_decay != 0.0
    if variant:
        gpu.set_optimizer(args.momentum, args.weight_decay)
    gpu.init(None, w.sched.initial_batch())
    st, dev = upload_chunk(gpu, w, 0, W + 2 * K + K1)
    names = ("active", "delay_R", "delay_C", "drop_R", "drop_C", "batch_idx")
    cut = lambda a, b: [None if dev[k] is None else dev[k][a:b].contiguous() for k in names]   # noqa: E731
    run_args = lambda c, n_rounds: (n_rounds, c[0], c[1], c[2], c[3], c[4], w.gamma, c[5])      # noqa: E731
    run = lambda c, n_rounds: gpu.run(*run_args(c, n_rounds))                                    # noqa: E731
    if args.generated:
        p_act = torch.from_numpy(w.sched.p_active.astype(np.float32)).to(gpu.device)
        if args.graphs:
            rf.rfast_use_graphs(gpu.ctx, True)
        run = lambda c, n_rounds: gpu.run_generated(n_rounds, 20231117, p_act, w.sched.d_max, w.sched.p_drop, w.gamma)  # noqa: E731
    if args.sync:
        run = lambda c, n_rounds: gpu.sync_run(n_rounds, w.gamma, c[5])   # noqa: E731
    c_warm, c_timed, c_prof = cut(0, W), cut(W, W + K), cut(W + K, W + 2 * K)

    # ---- leg 1: warm-up, then the timed rounds
    run(c_warm, W)
    torch.cuda.synchronize()
    t_before = int(gpu.read("T_NODE").sum()) if args.generated else 0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(c_timed, K)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    gpu.check()
    t_after = int(gpu.read("T_NODE").sum()) if args.generated else 0

    # ---- leg 2: the next K rounds with HIP events around every kernel launch (on the library's stream), in calls cut
    # so that the counters and stamps can be read between the launches: where the library takes several rounds per
    # launch, at the multiples of the rebase interval (where it cuts its launches itself); else round by round.
    multi = not args.sync and separable and rf.rfast_block_info(gpu.ctx) != 0
    # least squares / logistic problems that fit the LDS of one CU: one workgroup takes a stretch of rounds per launch
    tiny = not args.sync and not separable and rf.rfast_block_info(gpu.ctx) != 0
    momentum_words = 2.0 if args.momentum != 0.0 else 0.0
    edges = edge_lists(w)
    segs, r = [], W + K
    while r < W + 2 * K:
        if args.sync:
            nxt = W + 2 * K
        elif multi or tiny:
            nxt = min(W + 2 * K, (r // REBASE_INTERVAL + 1) * REBASE_INTERVAL)
        else:
            nxt = r + 1
        segs.append((r, nxt))
        r = nxt
    ms_state = ms_grad = ms_res = 0.0
    n_state = n_grad = n_res = 0
    # launches of the multi-round kernel (rounds, ms, bytes, rows in, rows out, node-updates) and, of the rounds that ran
    # one pass each, time, bytes and node-updates
    launches_multi, one_ms, one_bytes, one_updates, one_launches = [], 0.0, 0.0, 0, 0
    lanes, per_wave = rf.rfast_block_info(gpu.ctx, with_kind=True) if multi else (0, False)
    for lo, hi in segs:
        before = None if args.sync else read_stamps(gpu)
        rf.rfast_profile_enable(gpu.ctx, True)
        run(cut(lo, hi), hi - lo)
        ms, cnt = rf.rfast_kernel_time(gpu.ctx, 0)
        ms_g, cnt_g = rf.rfast_kernel_time(gpu.ctx, 1)
        ms_r, cnt_r = rf.rfast_kernel_time(gpu.ctx, 2)
        rf.rfast_profile_enable(gpu.ctx, False)
        ms_state, ms_grad, ms_res = ms_state + ms, ms_grad + ms_g, ms_res + ms_r
        n_state, n_grad, n_res = n_state + cnt, n_grad + cnt_g, n_res + cnt_r
        if args.sync:
            continue
        after = read_stamps(gpu)
        done = int((after["t"] - before["t"]).sum())
        if tiny and cnt == 1 and hi - lo > 1:
            # the whole state once in and once out per launch: x, z, the stored sample, every ring slot, every S4 buffer
            rows_state = w.n * (3 + 2 * (w.D + 2)) + w.C.nnz_off
            launches_multi.append((hi - lo, ms, 2.0 * rows_state * 4.0 * w.p, rows_state, rows_state, done))
        elif multi and cnt == 1 and hi - lo > 1:
            if per_wave:
                mv, ri, ro = multi_round_bytes(w, edges, before, after, hi % REBASE_INTERVAL == 0)
            else:   # the workgroup-tile kernel moves every ring slot and every buffer in and out
                ri = w.n * (2 * (w.D + 2) + 4) + w.C.nnz_off
                ro = w.n * (2 * (w.D + 2) + 2) + w.C.nnz_off
                mv = float(ri + ro) * 4.0 * w.p
            mv += momentum_words * 4.0 * w.p * w.n
            launches_multi.append((hi - lo, ms, mv, ri, ro, done))
        elif hi - lo == 1:
            act = (after["t"] != before["t"])
            one_bytes += one_pass_bytes(w, edges, before, after, act) + momentum_words * 4.0 * w.p * float(act.sum())
            one_ms, one_updates, one_launches = one_ms + ms, one_updates + done, one_launches + cnt

    act_timed = st["active"][W:W + K].astype(np.int64)
    act_prof = st["active"][W + K:W + 2 * K].astype(np.int64)
    updates = (t_after - t_before) if args.generated else (w.n * K if args.sync else int(act_timed.sum()))
    headline = not (args.p or args.sync or variant or args.generated or args.noise_std is not None)

    def hbm_or_alu(moved, flops, secs):
        """The roofline of work that needs `moved` bytes of HBM traffic and `flops` of fp32 vector arithmetic and took
        `secs`: the bound is whichever takes longer at the published peak, and the fraction is against that peak."""
        t_alu, t_hbm = flops / (FP32_VECTOR_PEAK_TFLOPS * 1e12), moved / (HBM_PEAK_GBS * 1e9)
        if t_hbm >= t_alu:
            roof = {"bound": "hbm", "achieved": moved / secs / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s"}
        else:
            roof = {"bound": "alu", "achieved": flops / secs / 1e12, "peak": FP32_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s"}
        roof["frac"] = roof["achieved"] / roof["peak"]
        roof.update({"bytes_per_launch": moved, "flops_per_launch": flops, "intensity_flop_per_byte": flops / moved,
                     "ridge_flop_per_byte": FP32_VECTOR_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9),
                     "time_at_hbm_peak_ms": t_hbm * 1e3, "time_at_fp32_vector_peak_ms": t_alu * 1e3,
                     "achieved_gbs": moved / secs / 1e9, "achieved_tflops": flops / secs / 1e12})
        return roof

    if args.sync:
        # eq. (2), all nodes at once.  One step per launch pair: descent x, z -> v (3 words), step 1 + dR v's and 1 + dI
        # z's in, x and z out, plus the old x, h, c (separable objective: its sample is recomputed) or the old and the
        # new sample.  Several steps per launch: x, z, h, c in, x, z, v out once per launch.
        dR, dI, _ = degrees(w)
        many = 0 < n_state < K
        if many:
            moved = (7.0 + momentum_words) * 4.0 * w.p * w.n
            kernel = "rfast_sync_wave_kernel (several steps per launch, state in registers and LDS)"
        else:
            moved = float((3 + (1 + dR) + (1 + dI) + 2 + (3 if separable else 2) + momentum_words).sum()) * 4.0 * w.p
            kernel = "rfast_sync_descent_kernel + rfast_sync_step_kernel"
        per = max(n_state if many else K, 1)
        flops = FLOPS_PER_COORDINATE * w.p * w.n * (K / per if many else 1.0) if separable else 0.0
        roof = hbm_or_alu(moved, flops, ms_state * 1e-3 / per)
        roof.update({"kernel": kernel, "avg_kernel_ms": ms_state / per, "launches": per, "traffic": None})
    elif launches_multi:
        # Launches that took their rounds with the state in LDS.  Such a launch has to do the method's arithmetic for its
        # rounds and to move the live state once in and once out.
        n_multi = len(launches_multi)
        rounds_multi = sum(l[0] for l in launches_multi)
        secs = sum(l[1] for l in launches_multi) * 1e-3 / n_multi
        moved = sum(l[2] for l in launches_multi) / n_multi
        flops = FLOPS_PER_COORDINATE * w.p * sum(l[5] for l in launches_multi) / n_multi
        if tiny:   # the GEMV pair of the sampled gradient: 4 B p flop per node-update, plus Algorithm 1's own 21 per coordinate
            flops = (4.0 * (w.sched.batch or w.data["A" if w.objective == "least_squares" else "X"].shape[1]) + 21.0) * w.p * \
                sum(l[5] for l in launches_multi) / n_multi
        kernel = f"rfast_wave_kernel<{lanes} lanes per node>" if per_wave else f"rfast_block_kernel<{lanes} lanes per node>"
        if tiny:
            kernel = "rfast_tiny_kernel (one workgroup, the whole problem in LDS)"
        counted = counted_traffic(w.name, "wave", rounds_multi // n_multi) if headline and per_wave and rounds_multi % n_multi == 0 else None
        roof = hbm_or_alu(moved, flops, secs)
        roof.update({"kernel": kernel, "avg_kernel_ms": secs * 1e3, "launches": n_multi, "rounds_per_launch": rounds_multi / n_multi,
                     "rows_per_node_in": sum(l[3] for l in launches_multi) / n_multi / w.n,
                     "rows_per_node_out": sum(l[4] for l in launches_multi) / n_multi / w.n,
                     "traffic": counted["bytes_per_launch"] if counted else None,
                     "traffic_source": counted["source"] if counted else None,
                     "note": "bytes_per_launch: what the launch moves by its own rules (live ring slots, x, z, h, c, buffers "
                             "outside their ring), computed here from the counters and stamps read before and after it; "
                             "flops_per_launch: 40 per coordinate and node-update (Algorithm 1 and the float side of the "
                             "Gaussian noise; the integer work of the counter-based generator is not a flop)"
                             if not tiny else
                             "one workgroup on one of 256 compute units, bound by instruction issue and LDS latency: the "
                             "fraction of the chip's peak says how small the problem is, not how good the kernel is; "
                             "bytes_per_launch: the whole state in and out once (the objective data, copied to LDS once per "
                             "launch when they fit, not counted); flops_per_launch: (4 B + 21) p per node-update"})
    else:
        # One pass over HBM per round (two for the objectives whose gradient runs between them).
        secs = one_ms * 1e-3
        launches = max(one_launches, 1)
        kernel = "rfast_state_kernel" + ("<FUSED>" if separable else "<MIX> + <TRACK>")
        if w.objective in ("least_squares", "logistic") and not args.no_blocks:
            # this leg runs its rounds in calls of one: a mixing pass, then the kernel that does the column sums and the
            # tracker update (in a longer call it also mixes for the next round and the mixing pass runs once per stretch)
            kernel = "rfast_state_kernel<MIX> + rfast_cols_track_mix_kernel"
        act1 = act_prof
        alg1 = sum(algorithmic_bytes_per_round(w, a) for a in act1)
        lay1 = sum(algorithmic_bytes_per_round(w, a, layout=True) for a in act1)
        counted = counted_traffic(w.name, "state", 1) if headline and separable else None
        roof = {"bound": "hbm", "kernel": kernel, "achieved": one_bytes / secs / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": one_bytes / secs / 1e9 / HBM_PEAK_GBS, "avg_kernel_ms": one_ms / launches, "launches": one_launches,
                "bytes_per_launch": one_bytes / launches,
                "layout_bytes_per_launch": lay1 / launches, "layout_gbs": lay1 / secs / 1e9,
                "algorithmic_bytes_per_launch": alg1 / launches, "algorithmic_gbs": alg1 / secs / 1e9,
                "traffic": counted["bytes_per_launch"] if counted else None,
                "traffic_source": counted["source"] if counted else None,
                "note": "bytes_per_launch counts what the state kernels read and write, edges whose stamp did not move "
                        "skipped (computed per round from the stamps before and after it); layout_*: the words of this "
                        "layout with no skip credited; algorithmic_*: the literal count of Algorithm 1, which the layout "
                        "undercuts, so its rate may exceed the peak and is not a fraction of it"}

    out = {
        "metric": "node-updates/sec",
        "value": updates / dt,
        "unit": "node-updates/s",
        "param_elements_per_s": updates * w.p / dt,
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": dt / K * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name + ("/synchronous-push-pull" if args.sync else "") +
                               ("/generated-schedule" if args.generated else "") + ("/hip-graphs" if args.graphs else "") +
                               (f"/momentum={args.momentum},weight_decay={args.weight_decay}" if variant else ""),
                   "n": w.n, "p": w.p, "D": w.D, "ring_slots": w.D + 2, "objective": w.objective,
                   "mean_active_per_round": updates / K, "gamma": w.gamma},
        "roofline": roof,
        "kernel_ms": {"state": ms_state, "gradient": ms_grad, "resolver": ms_res,
                      "launches": {"state": n_state, "gradient": n_grad, "resolver": n_res}},
        "host_data_generation_s": gen_s,
    }

    # ---- leg 3 (where leg 2 ran several rounds per launch): one kernel pass per round, the HBM view of the fused round kernel
    if K1 > 0 and launches_multi:
        rf.rfast_use_blocks(gpu.ctx, False)
        r0 = W + 2 * K
        moved = 0.0
        ms_one = 0.0
        for q in range(K1):
            before = read_stamps(gpu)
            rf.rfast_profile_enable(gpu.ctx, True)
            run(cut(r0 + q, r0 + q + 1), 1)
            ms, cnt = rf.rfast_kernel_time(gpu.ctx, 0)
            rf.rfast_profile_enable(gpu.ctx, False)
            assert cnt == 1, cnt
            ms_one += ms
            after = read_stamps(gpu)
            act = after["t"] != before["t"]
            moved += one_pass_bytes(w, edges, before, after, act) + momentum_words * 4.0 * w.p * float(act.sum())
        act1 = st["active"][r0:r0 + K1].astype(np.int64)
        alg1 = sum(algorithmic_bytes_per_round(w, a) for a in act1)
        lay1 = sum(algorithmic_bytes_per_round(w, a, layout=True) for a in act1)
        s1 = ms_one * 1e-3
        counted = counted_traffic(w.name, "state", 1) if headline else None
        out["roofline_one_pass"] = {
            "bound": "hbm", "kernel": "rfast_state_kernel<FUSED>", "launches": K1, "avg_kernel_ms": ms_one / K1,
            "achieved": moved / s1 / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": moved / s1 / 1e9 / HBM_PEAK_GBS,
            "bytes_per_launch": moved / K1,
            "layout_bytes_per_launch": lay1 / K1, "layout_gbs": lay1 / s1 / 1e9,
            "algorithmic_bytes_per_launch": alg1 / K1, "algorithmic_gbs": alg1 / s1 / 1e9,
            "node_updates_per_s": float(act1.sum()) / s1,
            "traffic": counted["bytes_per_launch"] if counted else None,
            "traffic_source": counted["source"] if counted else None,
            "note": "one pass over HBM per round; bytes_per_launch counts what the pass reads and writes, edges whose stamp did "
                    "not move skipped (computed per round from the stamps before and after it); layout_*: the words of this "
                    "layout with no skip credited; algorithmic_*: the literal count of Algorithm 1 (7 + dR + 3 dI + 2 dO + 2 "
                    "words), which the layout undercuts, so its rate may exceed the peak and is not a fraction of it"}
    if w.objective == "softmax_bf16":
        # the two GEMMs of the softmax gradient: 2*B*d*K flops each per node-update
        gflops = 4.0 * w.sched.batch * w.extra["d"] * w.extra["K"] * float(act_prof.sum())
        tf = gflops / (ms_grad * 1e-3) / 1e12 if ms_grad > 0 else 0.0
        out["roofline_mfma"] = {"bound": "mfma", "kernel": "rfast_softmax_prep+forward+backward", "achieved": tf,
                                "peak": 2500.0, "unit": "TFLOP/s", "frac": tf / 2500.0,
                                "intensity_limited_peak": 680.0, "avg_ms_per_round": ms_grad / max(n_grad, 1)}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w)
        out["gpu_over_cpu"] = out["value"] / out["cpu_baseline"]["value"]
    print(json.dumps(out))


if __name__ == "__main__":
    main()
