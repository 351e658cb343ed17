#!/usr/bin/env python3
"""Benchmark of the block-level scheduling path on one MI355X.

Workload (`config.workload` = "cfg1"): a best-effort bf16 GEMM, M = N = K = 4096 with
256x256 logical tiles, run back to back as a preemptible persistent-worker kernel,
next to a high-priority bf16 GEMV (1x4096 by 4096x4096) that arrives every 1 ms.

A "step" is PERIODS_PER_STEP (100) high-priority periods: 100 arrivals, each with its
preempt + native launch, and the best-effort work scheduled around them, so that the
default 20 steps give the configuration's 2000 arrivals per run.  K steps are timed, after
W warm-up steps, for (1) the high-priority job alone, (2) the best-effort job alone, (3) both
co-located under the priority scheduler.  (1) and (3) alternate INSIDE every run, in blocks of
100 arrivals with the best-effort side switched off and on, so that both see the same host
noise and machine state; the run is made `--repeats` times and the reported percentiles are
the medians over the repeats (pooled ones beside them).  From those: p50/p99 of the high-priority latency alone and co-located, the
p99 overhead, best-effort throughput retained, preemption latency.  A p99 is only reported
from 1000 samples per run upwards; below that the fields are null and the line says why.
Two latencies are given per request: the host clock's (scheduled arrival to completion
observed) and the device-side one (the part after the host's launch calls returned).
A separate leg times single launches of the dominant kernel (GEMM, native and
persistent-worker form) with HIP events for the roofline figures, and the CPU oracle is
timed on a bounded sample of the same work.

Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

METRIC = "co-located hi-pri p99 latency overhead %; best-effort tput %; preempt latency µs"
PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 matrix peak
PEAK_HBM_GBS = 8000.0


def pct(a, q):
    """Nearest-rank percentile."""
    s = np.sort(np.asarray(a))
    if len(s) == 0:
        return float("nan")
    k = max(int(np.ceil(q / 100.0 * len(s))) - 1, 0)
    return float(s[k])


def time_kernel_events(torch, ctx, B, be_stream, launch, reps, warm=3, batch=10):
    """Average duration of one launch: HIP events on the stream the kernel runs on, around
    `batch` launches enqueued back to back (as the scheduler enqueues them), so that the
    host's own time between the first event and the first launch is not counted as kernel
    time.  Returns (mean, min) of the per-launch figure over `reps` batches, in ms."""
    ms = []
    for i in range(warm + reps):
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        jobs = []
        e0.record(be_stream)
        for _ in range(batch):
            jobs.append(launch())
        e1.record(be_stream)
        for job in jobs:
            if job is not None:
                assert job.wait() == B.JOB_COMPLETE
                job.free()
        be_stream.synchronize()
        if i >= warm:
            ms.append(e0.elapsed_time(e1) / batch)
    return float(np.mean(ms)), float(np.min(ms))


def _oracle_leg(g, gv, budget_s):
    """Logical GEMM tiles through the oracle until the budget is used, then three GEMV calls."""
    from oracle import kernels as OK
    a = dict(g, C=np.zeros((1, g["m"], g["n"]), np.uint16))
    t0 = time.perf_counter()
    tiles = 0
    while tiles < 256 and (time.perf_counter() - t0) < budget_s:
        OK.exec_block("gemm_bf16", (tiles % 16, tiles // 16, 0), (16, 16, 1), a)
        tiles += 1
    t_gemm = time.perf_counter() - t0
    v = dict(gv, y=np.zeros(gv["n"], np.uint16))
    t1 = time.perf_counter()
    for _ in range(3):
        for b in range(OK.grid_of("gemv_bf16", v)[0]):
            OK.exec_block("gemv_bf16", (b, 0, 0), None, v)
    t_gemv = (time.perf_counter() - t1) / 3
    return tiles, t_gemm, t_gemv


def cpu_baseline(g, gv, budget_s=9.0):
    """The CPU oracle, as it stands, on a bounded sample of the same workload: once on one
    thread and once on every core this process may use (the oracle's matrix products run in
    NumPy's BLAS, whose thread pool is what spreads a logical tile over the cores)."""
    from threadpoolctl import threadpool_info, threadpool_limits
    allowed = len(os.sched_getaffinity(0))
    pool = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    with threadpool_limits(limits=1):
        tiles1, t1, gv1 = _oracle_leg(g, gv, budget_s)
    tilesn, tn, gvn = _oracle_leg(g, gv, budget_s)
    per_tile = 2.0 * 256 * 256 * g["k"]
    return {
        "value": tilesn * per_tile / tn / 1e9, "unit": "GFLOP/s (best-effort GEMM tiles)",
        "cores": int(min(pool, allowed)), "kind": "oracle",
        "sample": f"{tilesn} of 256 logical GEMM tiles in {tn:.1f} s on all cores; "
                  f"hi-pri GEMV {gvn * 1e3:.1f} ms per call (3 calls)",
        "affinity_cores": allowed, "blas_threads": int(pool),
        "gemv_latency_us": gvn * 1e6,
        "single_thread": {"value": tiles1 * per_tile / t1 / 1e9, "cores": 1,
                          "sample": f"{tiles1} of 256 logical GEMM tiles in {t1:.1f} s",
                          "gemv_latency_us": gv1 * 1e6},
    }


def profile_traffic():
    """HBM-side bytes of one persistent-worker GEMM launch, from the committed rocprofv3
    counter summary (the line that starts with TRAFFIC): FETCH_SIZE and WRITE_SIZE in KiB per
    dispatch, each scaled by what the same counter read for a plain copy of known size."""
    path = os.path.join(ROOT, "profiles", "gemm_bf16_cfg1_rocprofv3.txt")
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("TRAFFIC gemm_ptb"):
                    kv = dict(t.split("=") for t in line.split()[2:])
                    return (float(kv["fetch_kib"]) * 1024 * float(kv["fetch_scale"]) +
                            float(kv["write_kib"]) * 1024 * float(kv["write_scale"]),
                            os.path.relpath(path, ROOT))
    except (OSError, KeyError, ValueError):
        pass
    return None, None


PERIODS_PER_STEP = 100     # arrivals of the high-priority job in one step
MIN_P99_SAMPLES = 1000     # a nearest-rank p99 of fewer samples is one of its ten largest
HW_QUEUES = 20             # hardware queues asked of HIP (its default is 4), see main()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None,
                    help=f"timed steps; one step = {PERIODS_PER_STEP} high-priority arrivals")
    ap.add_argument("--warmup", type=int, default=None, help="untimed steps before them")
    ap.add_argument("--workload", choices=["cfg0", "cfg1", "cfg2", "cfg3", "cfg4", "sweep_threshold", "sweep_load", "multi_be"], default="cfg1",
                    help="cfg1 is the headline workload; the others print one JSON line each "
                         "with that configuration's figures")
    ap.add_argument("--period-us", type=float, default=1000.0)
    ap.add_argument("--workers", type=int, default=None,
                    help="persistent workers of the best-effort GEMM; default: the profiler's choice "
                         "from the Section 4.2 candidate set under --threshold-ms (0.0316)")
    ap.add_argument("--threshold-ms", type=float, default=None,
                    help="turnaround-latency threshold of the profile-guided choice (cfg3, cfg4)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--roofline-reps", type=int, default=20)
    ap.add_argument("--repeats", type=int, default=5,
                    help="cfg1: the (alone, co-located) pair of K-step runs is made this many times, "
                         "alternating, and the median over the repeats of each percentile is "
                         "reported; the p99 of one 2000-sample run moves by several microseconds")
    ap.add_argument("--leg", choices=["all", "roofline", "coloc"], default="all",
                    help="roofline: only single launches of the GEMM/GEMV kernels plus a plain "
                         "copy of known size (for rocprofv3 counter runs); coloc: only the "
                         "co-located scheduling run")
    args = ap.parse_args()
    defaults = {"cfg0": (1, 0), "cfg1": (20, 5), "cfg2": (20, 1), "cfg3": (20, 1),
                "cfg4": (20, 1), "sweep_threshold": (15, 1),
                "sweep_load": (20, 1), "multi_be": (20, 1)}[args.workload]
    if args.steps is None:
        args.steps = defaults[0]
    if args.warmup is None:
        args.warmup = defaults[1]
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the method is a per-GPU mechanism); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    args.n_arrivals = args.steps * PERIODS_PER_STEP      # timed arrivals per run
    args.n_warm = args.warmup * PERIODS_PER_STEP         # untimed arrivals before them

    # The scheduler needs a hardware queue each for the high-priority stream, the best-effort
    # stream and the relay stream (two more per further best-effort client) beside the null
    # stream's; HIP folds a process's streams onto GPU_MAX_HW_QUEUES queues (4 unless set) and
    # reads the variable when it initialises.  This program raises a smaller (or absent) value
    # to 20, keeps a larger one, and every JSON line records the value in effect.
    try:
        have = int(os.environ.get("GPU_MAX_HW_QUEUES", "4"))
    except ValueError:
        have = 4
    if have < HW_QUEUES:
        os.environ["GPU_MAX_HW_QUEUES"] = str(HW_QUEUES)
    hwq = os.environ["GPU_MAX_HW_QUEUES"]

    import torch
    import tally_inputs as TI
    import paper_2410_07381_amd.binding as B

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    torch.cuda.set_device(0)
    hi_stream, be_stream = torch.cuda.Stream(), torch.cuda.Stream()
    ctx = B.Context(hi_stream, be_stream)
    streams = ctx.stream_report()
    spare = []
    while streams["be_delays_hi"] and len(spare) < 4:
        # the best-effort stream got a hardware queue on the high-priority queue's pipe: take
        # the next stream instead (the library reports it, only the caller can change it)
        ctx.close()
        spare.append(be_stream)
        be_stream = torch.cuda.Stream()
        ctx = B.Context(hi_stream, be_stream)
        streams = ctx.stream_report()

    if args.workload != "cfg1":
        import bench_configs
        out = bench_configs.WORKLOADS[args.workload](torch, B, ctx, be_stream, args)
        out.update({"n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "data": "synthetic",
                    "arrivals_per_step": PERIODS_PER_STEP, "gpu_max_hw_queues": hwq})
        out["streams"] = ctx.stream_report()
        ctx.close()
        print(json.dumps(out))
        return

    # ---- inputs, resident in HBM before any timed region --------------------------------
    g = TI.gemm_inputs(4096, 4096, 4096, config_index=1)
    gv = TI.gemv_inputs(4096, 4096, config_index=1)

    def dev(a):
        a = np.ascontiguousarray(a)
        return torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).cuda()

    A, Bt = dev(g["A"]), dev(g["Bt"])
    Cd = torch.zeros((1, 4096, 4096), dtype=torch.int16, device="cuda")
    x, W = dev(gv["x"]), dev(gv["W"])
    y = torch.zeros(4096, dtype=torch.int16, device="cuda")
    torch.cuda.synchronize()
    gemm = B.gemm_bf16(A, Bt, Cd)
    gemv = B.gemv_bf16(x, W, y)
    thr = args.threshold_ms if args.threshold_ms is not None else 0.0316
    if args.workers is None:
        # profile-guided choice (Section 4.2): every candidate really runs the kernel
        meas, chosen = ctx.profile(gemm, ctx.candidate_configs(gemm), runs=5, threshold_ms=thr)
        pick = meas[chosen]
        be_cfg = (pick["kind"], pick["param"], pick["chunk"])
        choice = {"by": "profiler", "threshold_ms": thr, "candidates": len(meas),
                  "form": "ptb" if pick["kind"] == B.CFG_PTB else "sliced", "param": pick["param"],
                  "chunk": pick["chunk"], "kernel_latency_us": pick["latency_ms"] * 1e3,
                  "turnaround_estimate_us": pick["turnaround_ms"] * 1e3}
    else:
        be_cfg = (B.CFG_PTB, args.workers, 1)
        choice = {"by": "--workers", "form": "ptb", "param": args.workers, "chunk": 1}
    args.workers = be_cfg[1] if be_cfg[0] == B.CFG_PTB else ctx.max_workers(gemm)

    if args.leg == "roofline":
        # counter runs: a plain copy of known size calibrates FETCH_SIZE / WRITE_SIZE
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        for _ in range(args.roofline_reps):
            ctx.launch_native(gemm)
            be_stream.synchronize()
            job = ctx.launch_ptb(gemm, args.workers)
            assert job.wait() == B.JOB_COMPLETE
            job.free()
            ctx.launch_native(gemv)
            be_stream.synchronize()
        ctx.close()
        print(json.dumps({"leg": "roofline", "reps": args.roofline_reps,
                          "copy_bytes_read": 4 << 28, "copy_bytes_written": 4 << 28}))
        return

    K, Wm = args.n_arrivals, args.n_warm
    arrivals = TI.periodic_arrivals_us(args.period_us, K + Wm)
    if args.leg == "coloc":
        co = ctx.sched_run([gemv], arrivals, [(gemm, be_cfg)], policy=B.POLICY_TALLY, tail_us=0.0)
        lat = co["latency_us"][Wm:]
        ctx.close()
        print(json.dumps({"leg": "coloc", "n": int(len(lat)), "p50": pct(lat, 50), "p90": pct(lat, 90),
                          "p99": pct(lat, 99) if len(lat) >= MIN_P99_SAMPLES else None,
                          "max": float(lat.max()),
                          "be_kernels": int(co["be_kernels_done"])}))
        return

    # ---- (2) best-effort alone -----------------------------------------------------------
    ctx.sched_run([], [], [(gemm, be_cfg)], tail_us=max(Wm, 100) * args.period_us)   # warm-up
    be_solo = ctx.sched_run([], [], [(gemm, be_cfg)], tail_us=K * args.period_us)
    tput_solo = be_solo["be_kernels_done"] / (be_solo["window_us"] * 1e-6)
    # ---- (1) high-priority alone and (3) co-located, alternating INSIDE each run ----------
    # Blocks of 100 arrivals alternate between "best-effort side switched off" (the job
    # alone) and "on" (co-located), so both populations see the same host noise and the
    # same machine state; a run holds Wm warm-up arrivals, then K alone and K co-located.
    # Every block starts with SETTLE extra arrivals that are left out (the switch takes a
    # best-effort kernel's drain, or its launch, to take effect).
    SETTLE = 5
    T = PERIODS_PER_STEP + SETTLE                  # a block: 5 arrivals to settle, 100 that count
    Wb = -(-Wm // (2 * T)) * 2 * T                 # warm-up rounded up to whole block pairs
    arrivals = TI.periodic_arrivals_us(args.period_us, Wb + 2 * args.steps * T)
    idx = np.arange(len(arrivals))
    timed = (idx >= Wb) & (idx % T >= SETTLE)
    solo_mask = timed & ((idx // T) % 2 == 0)
    co_mask = timed & ((idx // T) % 2 == 1)
    runs = []
    t_wall = 0.0
    for _ in range(max(args.repeats, 1)):
        t_wall0 = time.perf_counter()
        runs.append(ctx.sched_run([gemv], arrivals, [(gemm, be_cfg)], policy=B.POLICY_TALLY,
                                  tail_us=0.0, be_toggle_every=T))
        t_wall += time.perf_counter() - t_wall0
    solo_runs = [{"lat": r["latency_us"][solo_mask], "dev": (r["latency_us"] - r["issue_us"])[solo_mask]}
                 for r in runs]
    co_runs = [{"lat": r["latency_us"][co_mask], "dev": (r["latency_us"] - r["issue_us"])[co_mask]}
               for r in runs]
    host_lat = lambda r: r["lat"]
    # the part of a latency that follows the host's launch calls (device side and completion)
    dev_lat = lambda r: r["dev"]
    co = {"window_us": sum(r["window_us"] for r in runs),
          "be_enabled_us": sum(r["be_enabled_us"] for r in runs),
          "be_kernels_done": sum(r["be_kernels_done"] for r in runs),
          "n_preempts": sum(r["n_preempts"] for r in runs),
          "preempt_latency_us": np.concatenate([r["preempt_latency_us"] for r in runs])}
    tput_co = co["be_kernels_done"] / (co["be_enabled_us"] * 1e-6)
    n_run = int(len(host_lat(co_runs[0])))
    p99_ok = n_run >= MIN_P99_SAMPLES
    arrivals = TI.periodic_arrivals_us(args.period_us, K + Wm)     # for the decomposition runs
    # ---- decomposition: same load with native best-effort kernels, and with no scheduling -
    n_dec = Wm + max(K // 2, min(K, MIN_P99_SAMPLES))
    nat = ctx.sched_run([gemv], arrivals[:n_dec], [(gemm, (B.CFG_NATIVE, 1, 1))],
                        policy=B.POLICY_PRIORITY_NATIVE, tail_us=0.0)
    nos = ctx.sched_run([gemv], arrivals[:n_dec], [(gemm, (B.CFG_NATIVE, 1, 1))],
                        policy=B.POLICY_NONE, tail_us=0.0)

    # Percentiles: the median over the repeats of each run's own p50 / p99.  The p99 of one
    # 2000-sample run is its 20th largest value; an otherwise idle GPU answers a handful of
    # requests late (40-50 us) in some runs and not in others, so one bad run must not decide
    # the figure (pooling the samples lets it).  The pooled percentiles are reported beside
    # these.  Below MIN_P99_SAMPLES samples per run no p99 is reported at all.
    def summary(get):
        med = lambda runs, q: float(np.median([pct(get(r), q) for r in runs]))
        o = {"solo_p50": med(solo_runs, 50), "coloc_p50": med(co_runs, 50), "n_per_run": n_run,
             "runs": len(co_runs)}
        o["p50_overhead_pct"] = (o["coloc_p50"] - o["solo_p50"]) / o["solo_p50"] * 100.0
        if p99_ok:
            o["solo_p99"], o["coloc_p99"] = med(solo_runs, 99), med(co_runs, 99)
            o["p99_overhead_pct"] = (o["coloc_p99"] - o["solo_p99"]) / o["solo_p99"] * 100.0
            o["p99_us_per_repeat"] = {"solo": [pct(get(r), 99) for r in solo_runs],
                                      "coloc": [pct(get(r), 99) for r in co_runs]}
            o["p99_overhead_pct_per_repeat"] = [
                (pct(get(c), 99) / pct(get(s_), 99) - 1.0) * 100.0 for s_, c in zip(solo_runs, co_runs)]
            ps = np.concatenate([get(r) for r in solo_runs])
            pc = np.concatenate([get(r) for r in co_runs])
            o["pooled"] = {"n": int(len(pc)), "solo_p50": pct(ps, 50), "solo_p99": pct(ps, 99),
                           "coloc_p50": pct(pc, 50), "coloc_p99": pct(pc, 99),
                           "p99_overhead_pct": (pct(pc, 99) / pct(ps, 99) - 1.0) * 100.0}
        else:
            o["solo_p99"] = o["coloc_p99"] = o["p99_overhead_pct"] = None
            o["p99_undefined"] = (f"{n_run} samples per run: a p99 needs at least {MIN_P99_SAMPLES} "
                                  f"(--steps {MIN_P99_SAMPLES // PERIODS_PER_STEP} or more)")
        return o
    host_side, device_side = summary(host_lat), summary(dev_lat)
    overhead = host_side["p99_overhead_pct"]
    retained = tput_co / tput_solo * 100.0
    pre = co["preempt_latency_us"]

    # ---- roofline leg: single launches of the dominant kernel, HIP events ----------------
    flops = 2.0 * 4096 ** 3
    ms_nat, ms_nat_min = time_kernel_events(
        torch, ctx, B, be_stream, lambda: (ctx.launch_native(gemm), None)[1], args.roofline_reps)
    ms_ptb, ms_ptb_min = time_kernel_events(
        torch, ctx, B, be_stream, lambda: ctx.launch_ptb(gemm, args.workers), args.roofline_reps)
    ms_gemv, _ = time_kernel_events(
        torch, ctx, B, be_stream, lambda: (ctx.launch_native(gemv), None)[1], args.roofline_reps,
        batch=1)  # one at a time: back to back the 32 MB matrix is served by the Infinity Cache
    ceiling = ctx.mfma_ceiling_tflops(10)
    tf_nat = flops / (ms_nat * 1e-3) / 1e12
    tf_ptb = flops / (ms_ptb * 1e-3) / 1e12
    gemv_bytes = 4096 * 4096 * 2 + 2 * 4096 * 2
    traffic, traffic_src = profile_traffic()
    roofline = {
        "bound": "mfma", "kernel": "ptb_kernel<GemmBody> (best-effort GEMM, persistent workers)",
        "achieved": tf_ptb, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
        "frac": tf_ptb / PEAK_BF16_TFLOPS,
        # L2-side bytes per launch, not measured in this run: read from the committed
        # rocprofv3 counter summary named in traffic_source (FETCH_SIZE, WRITE_SIZE, scaled)
        "traffic": traffic, "traffic_source": traffic_src,
        "traffic_unit": "bytes per launch (algorithmic: 100663296)",
        "avg_launch_ms": ms_ptb,
        "native": {"achieved": tf_nat, "frac": tf_nat / PEAK_BF16_TFLOPS, "avg_launch_ms": ms_nat},
        "transformed_over_native": tf_ptb / tf_nat,
        # what the matrix pipe sustains on this device at its power-managed clock: a
        # register-only loop of the same MFMAs on every compute unit, measured in this run
        "measured_ceiling": {"peak": ceiling, "unit": "TFLOP/s", "frac": tf_ptb / ceiling},
        "hi_pri_gemv": {"bound": "hbm", "achieved": gemv_bytes / (ms_gemv * 1e-3) / 1e9,
                        "peak": PEAK_HBM_GBS, "unit": "GB/s",
                        "frac": gemv_bytes / (ms_gemv * 1e-3) / 1e9 / PEAK_HBM_GBS,
                        "avg_launch_ms": ms_gemv},
    }

    dec_p99 = lambda r: pct(r["latency_us"][Wm:], 99) if len(r["latency_us"][Wm:]) >= MIN_P99_SAMPLES else None
    steps_run = (len(idx) / (2.0 * T)) * len(runs)
    out = {
        "metric": METRIC,
        "value": overhead,
        "unit": "% (hi-pri p99 latency overhead, co-located vs alone; host clock, scheduled "
                "arrival to completion observed)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": co["window_us"] / steps_run / 1e3,
        "repeats": len(co_runs),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "cfg1: best-effort bf16 GEMM 4096^3 (256x256 logical tiles, "
                               f"{choice['form']} {choice['param']} x {choice['chunk']}) + hi-pri bf16 GEMV "
                               f"4096x4096 every {args.period_us:.0f} us",
                   "step": f"{PERIODS_PER_STEP} high-priority periods (arrivals) co-located with the "
                           f"best-effort job, preceded by {PERIODS_PER_STEP} periods alone as their baseline "
                           "(blocks alternate inside one run; each block starts with 5 more arrivals that are left out)",
                   "arrivals_per_step": PERIODS_PER_STEP, "timed_arrivals_per_run": n_run,
                   "be_config": choice,
                   "period_us": args.period_us, "gpu_max_hw_queues": hwq, "streams": streams},
        "hi_pri_latency_us": host_side,
        "hi_pri_device_side_latency_us": dict(
            device_side, definition="completion observed minus the moment the request's launch "
                                    "calls had returned on the host: the GPU's share of the latency"),
        "p99_overhead_pct": overhead,
        "p99_overhead_pct_device_side": device_side["p99_overhead_pct"],
        "p50_overhead_pct": host_side["p50_overhead_pct"],
        "be_tput_retained_pct": retained,
        "be_tput": {"solo_kernels_per_s": tput_solo, "coloc_kernels_per_s": tput_co,
                    "solo_tflops": tput_solo * flops / 1e12, "coloc_tflops": tput_co * flops / 1e12},
        "preempt_latency_us": {"n": int(co["n_preempts"]),
                               "p50": pct(pre, 50) if len(pre) else None,
                               "p99": pct(pre, 99) if len(pre) >= MIN_P99_SAMPLES else None,
                               "max": float(pre.max()) if len(pre) else None},
        "decomposition_p99_us": {
            "ideal": host_side["solo_p99"], "full": host_side["coloc_p99"],
            "priority_native_be": dec_p99(nat), "no_scheduling": dec_p99(nos),
            "n": int(len(nat["latency_us"][Wm:]))},
        "transform_overhead_pct": (ms_ptb / ms_nat - 1.0) * 100.0,
        "roofline": roofline,
        "paper_context": "Tally on A100-40GB: 7.2% avg p99 overhead (TGS 188.9%), >=80% of TGS "
                         "system throughput; other hardware, context only",
        "coloc_wall_s": t_wall,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(g, gv)
    ctx.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
