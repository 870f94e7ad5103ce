#!/usr/bin/env python3
"""Benchmark of the R-FAST activation round on one MI355X.

A step is one round of the whole hot path (resolver + state update + local
gradients) over one batch of synthetic input that is already resident in HBM.
The default workload is config 2 (n=16 bidirectional ring, diagonal quadratic,
p = 11.2 M, every node active), the configuration the HBM-roofline target is
quoted on.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
for pth in (ROOT, os.path.join(ROOT, "tests")):
    if pth not in sys.path:
        sys.path.insert(0, pth)

import numpy as np  # noqa: E402

HBM_PEAK_GBS = 8000.0


def algorithmic_bytes_per_round(w, active_counts, layout=False):
    """Literal traffic of Algorithm 1 per node-update: 7 + dR + 3 dI + 2 dO fp32 words
    per coordinate (reads x, z, g_prev, dR v's, dI rho's, dI rho~'s, dO current rho's;
    writes x, z, g, v, dO new rho's, dI rho~'s), plus the objective data (h, c) of the
    diagonal quadratic, or the re-read of g_new by the split mix/track pair.
    layout=True: the words this library's layout has to move (one running sum per
    sender instead of one per out-edge: 2 words instead of 2 dO; no write of the S4
    buffer; no stored sample for the separable objective), skips not credited."""
    Rd, Cd = w.R.dense(), w.C.dense()
    dR = (Rd != 0).sum(axis=1) - 1
    dI = (Cd != 0).sum(axis=1) - 1
    dO = (Cd != 0).sum(axis=0) - 1
    push = 2 * np.minimum(dO, 1) if layout else 2 * dO
    words = 7 + dR + 3 * dI + push + (2 if w.objective == "diag_quadratic" else 1)
    if layout:
        words = words - dI      # the buffer of S4 is read from the sender's ring and (almost) never written
        if w.objective == "diag_quadratic":
            words = words - 2   # the old sample is recomputed from (x_i, t_i): g is neither read nor written
    return float((words * active_counts).sum() * 4.0 * w.p)


def profile_figure(workload_name, kernel, key):
    """A figure per launch of the dominant kernel from the committed rocprofv3 --pmc summary, if any."""
    for suffix in ("hbm_traffic", "stats"):
        path = os.path.join(ROOT, "profiles", f"{workload_name}_{kernel}_kernel_{suffix}.md")
        try:
            with open(path) as f:
                for line in f:
                    if line.startswith(key + ":"):
                        return float(line.split(":")[1])
        except OSError:
            pass
    return None


def measured_traffic(workload_name, kernel="state"):
    return profile_figure(workload_name, kernel, "traffic_bytes_per_launch")


# vector ALU: 256 CUs x 4 SIMDs x 16 lanes, one instruction per lane and clock at 2.4 GHz (the published
# 157.3 TFLOP/s counts a packed fp32 FMA on each lane as 4 flops)
VALU_LANE_PEAK = 256 * 4 * 16 * 2.4e9


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
    import harness
    if w.objective == "diag_quadratic":
        p_sub = min(w.p, 400_000)
        coords = np.arange(p_sub, dtype=np.int64) * (w.p // p_sub)
    else:
        coords, p_sub = None, w.p
    frac = p_sub / w.p
    what = f"the same schedule on {p_sub} of {w.p} coordinates (every {w.p // p_sub}-th), scaled by {frac:.4g}"
    orc = harness.make_oracle(w, coords)
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
    import harness
    from rfast_workloads import configs
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
    gpu = harness.make_gpu(w)
    if args.no_blocks:
        rf.rfast_use_blocks(gpu.ctx, False)
    if args.force_blocks:
        rf.rfast_use_blocks(gpu.ctx, 2)
    variant = args.momentum != 0.0 or args.weight_decay != 0.0
    if variant:
        gpu.set_optimizer(args.momentum, args.weight_decay)
    gpu.init(None, w.sched.initial_batch())
    st, dev = harness.upload_chunk(gpu, w, 0, W + 2 * K)
    sl = lambda name, a, b: None if dev[name] is None else dev[name][a:b].contiguous()
    run = lambda a, b: gpu.run(b - a, sl("active", a, b), sl("delay_R", a, b), sl("delay_C", a, b), sl("drop_R", a, b),
                               sl("drop_C", a, b), w.gamma, sl("batch_idx", a, b))
    if args.generated:
        p_act = torch.from_numpy(w.sched.p_active.astype(np.float32)).to(gpu.device)
        if args.graphs:
            rf.rfast_use_graphs(gpu.ctx, True)
        run = lambda a, b: gpu.run_generated(b - a, 20231117, p_act, w.sched.d_max, w.sched.p_drop, w.gamma)
    if args.sync:
        bi = lambda a, b: sl("batch_idx", a, b)
        run = lambda a, b: gpu.sync_run(b - a, w.gamma, bi(a, b))
    run(0, W)
    torch.cuda.synchronize()
    t_before = int(gpu.read("T_NODE").sum()) if args.generated else 0
    t0 = time.perf_counter()
    run(W, W + K)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    gpu.check()
    t_after = int(gpu.read("T_NODE").sum()) if args.generated else 0

    # second pass with HIP events around every kernel launch (on the library's stream)
    rf.rfast_profile_enable(gpu.ctx, True)
    run(W + K, W + 2 * K)
    ms_state, n_state = rf.rfast_kernel_time(gpu.ctx, 0)
    ms_grad, n_grad = rf.rfast_kernel_time(gpu.ctx, 1)
    ms_res, n_res = rf.rfast_kernel_time(gpu.ctx, 2)
    rf.rfast_profile_enable(gpu.ctx, False)

    act_timed = st["active"][W:W + K].astype(np.int64)
    act_prof = st["active"][W + K:W + 2 * K].astype(np.int64)
    if args.sync:
        act_timed, act_prof = np.ones_like(act_timed), np.ones_like(act_prof)
    if args.generated:   # the masks live on the device; count the activations from the counters
        updates = t_after - t_before
    else:
        updates = int(act_timed.sum())
    bytes_prof = sum(algorithmic_bytes_per_round(w, a) for a in act_prof)
    bytes_layout = sum(algorithmic_bytes_per_round(w, a, layout=True) for a in act_prof)
    if args.sync:
        # descent: x, z -> v (3 words); step: 1+dR v's, 1+dI z's in, x and z out, plus
        #   separable objective: the old x (its sample is recomputed, not stored), h, c in (3 words)
        #   otherwise: the old and the new sample in (2 words)
        dR = (w.R.dense() != 0).sum(axis=1) - 1
        dI = (w.C.dense() != 0).sum(axis=1) - 1
        words = 3 + (1 + dR) + (1 + dI) + 2 + (3 if w.objective == "diag_quadratic" else 2)
        bytes_prof = bytes_layout = float(words.sum() * 4.0 * w.p * K)
    if args.momentum != 0.0:   # read and write of the buffer m_i
        extra = 8.0 * w.p * (w.n * K if args.sync else float(act_prof.sum()))
        bytes_prof, bytes_layout = bytes_prof + extra, bytes_layout + extra
    launches = max(n_state, 1)
    avg_ms = ms_state / launches
    # several rounds per launch with the state resident in LDS (the default where it applies)
    # (graph replays, which the timed pass of --graphs uses, are one pass per round; the event-timed pass cannot replay)
    blocked = not args.sync and not args.graphs and w.objective == "diag_quadratic" and 0 < n_state < K
    lanes, per_wave = rf.rfast_block_info(gpu.ctx, with_kind=True) if blocked else (0, False)
    if args.sync:
        kernel = "rfast_sync_wave_kernel (several steps per launch, state in registers and LDS)" if 0 < n_state < K else "rfast_sync_descent+step"
    elif blocked:
        kernel = f"rfast_wave_kernel<{lanes} lanes per node>" if per_wave else f"rfast_block_kernel<{lanes} lanes per node>"
    else:
        kernel = "rfast_state_kernel" + ("<FUSED>" if w.objective == "diag_quadratic" else "<MIX>+<TRACK>")
    headline = not (args.p or args.sync or variant or args.generated)
    achieved = bytes_prof / (ms_state * 1e-3) / 1e9 if ms_state > 0 else 0.0
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
                               (f"/momentum={args.momentum},weight_decay={args.weight_decay}" if variant else ""), "n": w.n, "p": w.p, "D": w.D, "ring_slots": w.D + 2, "objective": w.objective,
                   "mean_active_per_round": updates / K, "gamma": w.gamma},
        "roofline": {"bound": "hbm", "kernel": kernel, "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "avg_kernel_ms": avg_ms, "launches": n_state,
                     "algorithmic_bytes_per_launch": bytes_prof / launches,
                     "layout_bytes_per_launch": bytes_layout / launches,
                     "achieved_layout": achieved * bytes_layout / bytes_prof if bytes_prof else 0.0,
                     "frac_layout": achieved * bytes_layout / bytes_prof / HBM_PEAK_GBS if bytes_prof else 0.0,
                     "traffic": measured_traffic(w.name, ("wave" if per_wave else "block") if blocked else "state") if headline else None},
        "kernel_ms": {"state": ms_state, "gradient": ms_grad, "resolver": ms_res,
                      "launches": {"state": n_state, "gradient": n_grad, "resolver": n_res}},
        "host_data_generation_s": gen_s,
    }
    if blocked:
        # The launch keeps the state in LDS over rounds_per_launch rounds, so the HBM traffic the
        # algorithmic figure counts per round is not moved: frac above 1 says so, and what bounds the
        # kernel is instruction issue.  VALU instructions per wavefront from the committed counter summary.
        out["roofline"]["rounds_per_launch"] = K / launches
        out["roofline"]["note"] = ("state resident in LDS over rounds_per_launch rounds: HBM moves every ring slot once "
                                   "per launch (traffic), not the per-round words of the algorithmic figure")
        per_round = profile_figure(w.name, "wave" if per_wave else "block", "valu_wave_instructions_per_round") if headline else None
        if per_round:
            # the bound that holds: vector instructions issued (64 lanes per wavefront instruction)
            rate = per_round * 64.0 * K / (ms_state * 1e-3)
            hbm = out["roofline"]
            out["roofline_hbm"] = hbm
            out["roofline"] = {"bound": "alu", "kernel": kernel, "achieved": rate / 1e12, "peak": VALU_LANE_PEAK / 1e12,
                               "unit": "T lane-instructions/s", "frac": rate / VALU_LANE_PEAK,
                               "avg_kernel_ms": avg_ms, "launches": n_state, "rounds_per_launch": K / launches,
                               "instructions_per_launch": per_round * 64.0 * K / launches,
                               "traffic": hbm["traffic"],
                               "source": "VALU instructions per round from the committed counter summary (SQ_INSTS_VALU) "
                                         "x rounds / kernel time measured here with HIP events"}
            # for context, the arithmetic of the method alone against the fp32 vector peak: about 40 flops per
            # coordinate and node-update (Algorithm 1 with two in-edges per graph: 21; the rest the float side of
            # the noise), the integer work of the counter-based generator not counted
            flops = 40.0 * w.p * float(act_prof.sum())
            out["roofline"]["algorithmic_tflops"] = flops / (ms_state * 1e-3) / 1e12
            out["roofline"]["algorithmic_frac_of_fp32_vector_peak"] = out["roofline"]["algorithmic_tflops"] / 157.3
    if w.objective == "softmax_bf16":
        # the two GEMMs of the softmax gradient: 2*B*d*K flops each per node-update
        flops = 4.0 * w.sched.batch * w.extra["d"] * w.extra["K"] * float(act_prof.sum())
        tf = flops / (ms_grad * 1e-3) / 1e12 if ms_grad > 0 else 0.0
        out["roofline_mfma"] = {"bound": "mfma", "kernel": "rfast_softmax_prep+forward+backward", "achieved": tf,
                                "peak": 2500.0, "unit": "TFLOP/s", "frac": tf / 2500.0,
                                "intensity_limited_peak": 680.0, "avg_ms_per_round": ms_grad / max(n_grad, 1)}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w)
        out["gpu_over_cpu"] = out["value"] / out["cpu_baseline"]["value"]
    print(json.dumps(out))


if __name__ == "__main__":
    main()
