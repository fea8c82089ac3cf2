#!/usr/bin/env python3
"""Benchmark of the FDA local-state + variance-check path on one MI355X.

A step is one pass of Algorithm 1 lines 6-9 over a synthetic [K, d] slab that is already
resident in HBM: fda_local_state, fda_estimate_variance, then fda_sync_xi (fda_sync and fda_update_xi)
predicated on the device-side decision (no host round trip inside a step).  The threshold
is set above the estimate, so in the timed steps the decision is "no synchronization" --
the case the method is built for -- and the metric is the cost of the state + check.  The
forced synchronization (fused mean + broadcast, then xi) is timed separately and reported
in the "sync" object.

Prints ONE JSON line.  `roofline` describes the streaming state kernel, timed live with HIP
events inside the library (fda_profile_*); `cpu_baseline` is the CPU oracle timed on a
bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published peak


def algorithmic_bytes(K, d, elem_bytes, variants):
    """Bytes one state pass must move: the slab once, w_t0 once, xi once if LinearFDA runs."""
    return K * d * elem_bytes + 4 * d + (4 * d if variants & 1 else 0)


def traffic_from_profile(workload, kernel="state_kernel"):
    """(HBM bytes per launch of a kernel, the file they come from): measured with rocprofv3 --pmc
    (FETCH_SIZE and WRITE_SIZE runs, scaled by a copy kernel) and committed as a summary for this
    workload -- not measured in this run.  (None, None) without such a summary."""
    rel = os.path.join("profiles", f"{kernel}_{workload}_traffic.txt")
    try:
        for line in open(os.path.join(ROOT, rel)):
            if line.startswith("traffic_bytes_per_launch="):
                return float(line.split("=", 1)[1]), rel
    except OSError:
        pass
    return None, None


def _block_state(job):
    """One coordinate block of the oracle's local state (a worker process of the all-cores leg)."""
    from threadpoolctl import threadpool_limits
    from oracle import fda_oracle as O
    a, b = job
    g = _CPU_JOB
    with threadpool_limits(limits=1):
        st = O.local_state(g["w"][:, a:b], g["dtype"], g["w0"][a:b], None if g["xi"] is None else g["xi"][a:b],
                           g["coef"], g["m"], scales=False, j0=a)
    return st["n"], st["p"], st["sk"]


_CPU_JOB = None


def cpu_baseline(config, over, variants, sample):
    """The CPU oracle, as it stands, on a bounded sample of the workload: first on ONE core (the process
    is pinned to one CPU and the numerical libraries are limited to one thread), then on all the cores
    this process may use, one coordinate block per core in worker processes (norms, projections and
    sketches of coordinate blocks add up: Section 3.1, linearity).  Only the method's own work is
    timed (local state + estimate; the oracle's tolerance scales are left out).  Runs before anything
    touches the GPU, because it forks."""
    global _CPU_JOB
    import multiprocessing as mp

    import numpy as np
    from threadpoolctl import threadpool_limits

    import fda_synth as S
    from oracle import fda_oracle as O

    c = dict(S.CONFIGS[config])
    c.update(over)
    ds = min(sample, c["d"])
    wls = S.make(config, device="cpu", seed=0, d=ds, **{k: v for k, v in over.items() if k != "d"})
    job = {"w": S.slab_to_numpy(wls.w), "dtype": wls.dtype, "w0": wls.w_t0.numpy(),
           "xi": wls.xi.numpy() if variants & 1 else None,
           "coef": wls.hash_coef if variants & 2 else None, "m": wls.m}
    K = wls.K
    allowed = sorted(os.sched_getaffinity(0))
    cores = min(len(allowed), 16)                   # a one-GPU machine grants 16 cores, whatever it shows
    # ---- one core
    os.sched_setaffinity(0, {allowed[0]})
    try:
        with threadpool_limits(limits=1):
            c0 = time.perf_counter()
            st = O.local_state(job["w"], job["dtype"], job["w0"], job["xi"], job["coef"], job["m"], scales=False)
            e1 = O.estimate_variance(st["n"], st["p"], st["sk"], wls.eps, 0.0)
            t_one = time.perf_counter() - c0
    finally:
        os.sched_setaffinity(0, set(allowed))
    # ---- all cores: one coordinate block per core
    _CPU_JOB = job
    cuts = [ds * q // cores for q in range(cores + 1)]
    jobs = [(a, b) for a, b in zip(cuts[:-1], cuts[1:]) if b > a]
    with mp.get_context("fork").Pool(cores) as pool:
        pool.map(_block_state, [(0, 1)] * cores)    # start the workers before the clock
        c0 = time.perf_counter()
        parts = pool.map(_block_state, jobs, chunksize=1)
        n = sum(q[0] for q in parts)
        pj = sum(q[1] for q in parts) if variants & 1 else None
        sk = sum(q[2] for q in parts) if variants & 2 else None
        e2 = O.estimate_variance(n, pj, sk, wls.eps, 0.0)
        t_all = time.perf_counter() - c0
    _CPU_JOB = None
    for key in ("mean_sqnorm", "h_linear", "h_sketch"):
        assert abs(e1[key] - e2[key]) <= 1e-9 * abs(e1["mean_sqnorm"]), key
    return {"value": K * ds / t_all, "unit": "worker-params/s", "cores": len(jobs), "kind": "oracle",
            "one_core_value": K * ds / t_one, "one_core_seconds": round(t_one, 2),
            "all_cores_seconds": round(t_all, 2), "cpus_visible": os.cpu_count(),
            "sample": f"fp64 numpy oracle (local state + estimate, without its tolerance scales) on a "
                      f"{K} x {ds} slab drawn on the CPU from the same recipe (same distributions and sketch, "
                      f"not the GPU's bits): pinned to one core {t_one:.1f} s; {len(jobs)} worker processes, one "
                      f"coordinate block each, {t_all:.1f} s"}


def run_calibration(args):
    """--lds-calibration / --stream-calibration: the rates of the chip the FDA kernels are compared with,
    from the library's own calibration kernels.  Prints one JSON line."""
    import torch

    import paper_2405_20988_amd as F
    F.load_library()
    torch.cuda.set_device(0)
    st = torch.cuda.current_stream().cuda_stream
    sink = torch.zeros(4, dtype=torch.int32, device="cuda:0")
    out = {}
    if args.lds_calibration:
        rates = {}
        ghz = None
        for op, opi in F.LDS_OPS.items():
            for pat, pi in F.LDS_PATTERNS.items():
                iters = 200 if op == "f32" else 2000
                r, ghz = F.fda_calib_lds_atomics(opi, pi, iters, sink.data_ptr(), st)
                rates[f"{op}/{pat}"] = round(r, 2)
        out["lds_atomic_adds_per_lane_per_clk_per_cu"] = rates      # read8 / read16: plain reads
        out["clock_ghz"] = ghz
        out["compute_units"] = torch.cuda.get_device_properties(0).multi_processor_count
    if args.stream_calibration:
        n = args.stream_calibration << 20
        src = torch.full((n // 4,), 1.0, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        cal = {"bytes": n}
        for hint, add in (("", 0), ("_nontemporal", 4)):
            ms_r = F.fda_calib_stream(0 + add, src.data_ptr(), sink.data_ptr(), n, 5, st)
            ms_w = F.fda_calib_stream(1 + add, None, dst.data_ptr(), n, 5, st)
            ms_c = F.fda_calib_stream(2 + add, src.data_ptr(), dst.data_ptr(), n, 5, st)
            cal.update({f"read{hint}_GBps": round(n / ms_r / 1e6, 1), f"fill{hint}_GBps": round(n / ms_w / 1e6, 1),
                        f"copy{hint}_GBps_read_plus_written": round(2 * n / ms_c / 1e6, 1),
                        f"read{hint}_ms": round(ms_r, 4), f"fill{hint}_ms": round(ms_w, 4),
                        f"copy{hint}_ms": round(ms_c, 4)})
        out["stream_calibration"] = cal
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="cfg5", help="cfg1..cfg5 (default: the largest, cfg5)")
    ap.add_argument("--variants", type=int, default=3, help="1 linear, 2 sketch, 3 both")
    ap.add_argument("--d", type=int, default=None, help="override d (for quick checks)")
    ap.add_argument("--l", type=int, default=None, help="override the sketch rows (sketch-size sweeps)")
    ap.add_argument("--m", type=int, default=None, help="override the sketch width (sketch-size sweeps)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--plain-table", action="store_true",
                    help="FDA_DESC_PLAIN_TABLE: every sketch row in its own slot of the tabulated hash "
                         "(the state pass without the placement against LDS collisions, for comparison)")
    ap.add_argument("--wbar", action="store_true",
                    help="mean-state mode: also emit the average model from the state pass and "
                         "synchronize with fda_sync_from_mean instead of fda_sync + fda_update_xi "
                         "(costs the state pass more than it saves unless synchronizations are frequent)")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MiB",
                    help="instead of the benchmark, run a plain device copy of this many MiB five "
                         "times (a kernel of known traffic, to scale rocprofv3's FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--lds-calibration", action="store_true",
                    help="instead of the benchmark: LDS atomic-add rates of this chip (library calibration kernels)")
    ap.add_argument("--stream-calibration", type=int, default=0, metavar="MiB",
                    help="instead of the benchmark: read / fill / copy rates over this many MiB with 16-byte "
                         "accesses (library calibration kernels)")
    ap.add_argument("--cpu-sample", type=int, default=6_000_000,
                    help="coordinates of the workload the CPU oracle is timed on")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (K workers are simulated as a [K,d] slab on one "
              "device; there are no collectives). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    over = {k: v for k, v in (("l", args.l), ("m", args.m)) if v is not None}
    calibrating = args.copy_calibration or args.lds_calibration or args.stream_calibration
    cpu = None
    if not args.no_cpu_baseline and not calibrating:
        # first, while nothing has touched the GPU yet (this leg forks worker processes)
        cpu_over = dict(over)
        if args.d is not None:
            cpu_over["d"] = args.d
        cpu = cpu_baseline(args.config, cpu_over, args.variants, args.cpu_sample)

    import numpy as np
    import torch

    import fda_synth as S
    import paper_2405_20988_amd as F

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(2)
    F.load_library()
    dev = "cuda:0"
    torch.cuda.set_device(0)

    if args.copy_calibration:
        n = args.copy_calibration << 20
        src = torch.full((n // 4,), 1.0, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_read": n, "copy_calibration_bytes_written": n,
                          "launches": 5}))
        return

    if args.lds_calibration or args.stream_calibration:
        run_calibration(args)
        return

    wl = S.make(args.config, device=dev, seed=0, d=args.d, **over)
    K, d = wl.K, wl.d
    esz = 4 if wl.dtype == "f32" else 2
    mon = F.FdaMonitor(K, d, wl.dtype, args.variants, wl.l, wl.m, wl.eps, wl.hash_coef, device=dev,
                       flags=F.FDA_DESC_PLAIN_TABLE if args.plain_table else 0)
    w_prev = wl.w_t0.clone()
    xi = wl.xi if args.variants & 1 else None
    pred = "sketch" if args.variants & 2 else "linear"

    # threshold above the current estimate: timed steps take the no-synchronization branch
    mon.local_state(wl.w, wl.w_t0, xi)
    est0 = mon.estimate_variance(0.0)
    h0 = est0.h_sketch if args.variants & 2 else est0.h_linear
    theta = 4.0 * max(h0, est0.mean_sqnorm)

    def step():
        mon.local_state(wl.w, wl.w_t0, xi)
        mon.estimate_variance(theta, want_host=False)
        if args.variants & 1:
            mon.sync_xi(wl.w, wl.w_t0, w_prev, wl.xi, pred=pred)
        else:
            mon.sync(wl.w, wl.w_t0, w_prev, pred=pred)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    F.fda_profile_enable(mon.ctx, True)
    F.fda_profile_read(mon.ctx, reset=True)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(args.steps):
        step()
        marks[i + 1].record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    kernel_ms, launches = F.fda_profile_read(mon.ctx, reset=True)
    F.fda_profile_enable(mon.ctx, False)
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
    est = mon.estimate_variance(theta)
    assert (est.sync_sketch if args.variants & 2 else est.sync_linear) == 0
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = K * d / (ms_per_step * 1e-3)

    # the same step as ONE call (fda_step) captured in a HIP graph and replayed: what a training loop that
    # replays its step pays, without the host's launch gaps -- reported beside `value`, never as it
    graph_info = None
    if args.variants & 2 or args.variants & 1:
        by = "sketch" if args.variants & 2 else "linear"
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            mon.step(wl.w, wl.w_t0, w_prev, wl.xi if args.variants & 1 else None, theta, decide_by=by)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            mon.step(wl.w, wl.w_t0, w_prev, wl.xi if args.variants & 1 else None, theta, decide_by=by)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        g0.record()
        for _ in range(args.steps):
            graph.replay()
        g1.record()
        torch.cuda.synchronize()
        est_g = mon.estimate_variance(theta)
        assert (est_g.sync_sketch if args.variants & 2 else est_g.sync_linear) == 0
        assert est_g.h_sketch == est.h_sketch and est_g.h_linear == est.h_linear
        graph_info = {"ms_per_step": round(g0.elapsed_time(g1) / args.steps, 4), "replays": args.steps,
                      "what": "fda_step (the same kernels, decision: no sync) captured once in a HIP graph"}
        del graph

    abytes = algorithmic_bytes(K, d, esz, args.variants)
    kern_ms_avg = kernel_ms / max(launches, 1)
    achieved = abytes / (kern_ms_avg * 1e-3) / 1e9
    workload = args.config if args.d is None else f"{args.config}-d{d}"
    if over:
        workload += f"-sketch{wl.l}x{wl.m}"
    traffic, traffic_source = traffic_from_profile(workload if args.variants == 3 else f"{workload}_v{args.variants}")
    roofline = {"bound": "hbm", "kernel": "state_kernel", "achieved": round(achieved, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": traffic, "traffic_source": traffic_source, "algorithmic_bytes": abytes,
                "kernel_ms": round(kern_ms_avg, 4), "launches": launches}
    if args.variants & 2:
        # what actually bounds this kernel: one LDS cell update per (worker, sketch row, coordinate).
        # With an even number of worker slots one returning 64-bit LDS addition updates the cells of
        # two workers; otherwise a returning 32-bit addition updates one.  The ceiling is measured
        # here, by the library's calibration kernel: such additions on random cells, per lane, clock
        # (the device's reported rate) and compute unit, times the cells an addition updates.
        props = torch.cuda.get_device_properties(0)
        sink = torch.zeros(4, dtype=torch.int32, device=dev)
        paired = mon.plan["worker_slots"] % 2 == 0
        op = "u64_rtn" if paired else "u32_rtn"
        rate, ghz = F.fda_calib_lds_atomics(F.LDS_OPS[op], F.LDS_PATTERNS["random"], 2000,
                                            sink.data_ptr(), torch.cuda.current_stream().cuda_stream)
        updates = float(wl.l) * K * d
        roofline["lds_cell_updates_per_clk_per_cu"] = round(
            updates / (kern_ms_avg * 1e-3) / props.multi_processor_count / (ghz * 1e9), 2)
        roofline["lds_cell_update_ceiling_per_clk_per_cu"] = round(rate * (2 if paired else 1), 2)
        roofline["lds_ceiling_source"] = (f"fda_calib_lds_atomics({op}, random cells) x {2 if paired else 1} cells per "
                                          "addition, measured in this run" +
                                          ("; the table's placed rows collide less than random cells do"
                                           if mon.plan.get("placed_row_group") else ""))
        roofline["clock_ghz"] = ghz

    # The same step with the average state computed directly (fda_mean_state: sketch of the mean
    # drift, by linearity) instead of the K per-worker states -- labelled separately, never `value`.
    w_bar = torch.empty_like(wl.w_t0)

    def mean_step():
        if not args.wbar:
            mon.mean_state(wl.w, wl.w_t0, xi)
            mon.estimate_variance_mean(theta, want_host=False)
            if args.variants & 1:
                mon.sync_xi(wl.w, wl.w_t0, w_prev, wl.xi, pred=pred)
            else:
                mon.sync(wl.w, wl.w_t0, w_prev, pred=pred)
        else:
            mon.mean_state(wl.w, wl.w_t0, xi, w_bar=w_bar)
            mon.estimate_variance_mean(theta, want_host=False)
            mon.sync_from_mean(wl.w, wl.w_t0, w_bar, w_prev=w_prev, xi=xi, pred=pred)

    for _ in range(args.warmup):
        mean_step()
    torch.cuda.synchronize()
    F.fda_profile_enable(mon.ctx, True)
    F.fda_profile_read(mon.ctx, reset=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        mean_step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    mkernel_ms, mlaunches = F.fda_profile_read(mon.ctx, reset=True)
    F.fda_profile_enable(mon.ctx, False)
    est_m = mon.estimate_variance_mean(theta)
    assert (est_m.sync_sketch if args.variants & 2 else est_m.sync_linear) == 0
    mean_ms = (t1 - t0) * 1e3 / args.steps
    mk = mkernel_ms / max(mlaunches, 1)
    mean_info = {"what": "same step with fda_mean_state (average state by linearity of the sketch, no "
                         "per-worker states" + ("; also emits the average model" if args.wbar else "") +
                         ") + fda_estimate_variance_mean + predicated " +
                         ("fda_sync_from_mean" if args.wbar else "fda_sync_xi"),
                 "ms_per_step": round(mean_ms, 4), "value": K * d / (mean_ms * 1e-3),
                 "unit": "worker-params/s", "kernel": "mean_state_kernel", "kernel_ms": round(mk, 4),
                 "achieved": round(abytes / (mk * 1e-3) / 1e9, 1), "peak": HBM_PEAK_GBS,
                 "frac": round(abytes / (mk * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                 "traffic": None if args.wbar else traffic_from_profile(workload, "mean_state_kernel")[0],
                 "traffic_source": None if args.wbar else traffic_from_profile(workload, "mean_state_kernel")[1],
                 "h_sketch": est_m.h_sketch, "h_linear": est_m.h_linear}

    # forced synchronization + xi refresh, timed separately (it rewrites the slab, so last)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = 3
    mon.sync(wl.w, wl.w_t0, w_prev, pred=None)
    torch.cuda.synchronize()
    ev0.record()
    for _ in range(reps):
        mon.sync(wl.w, wl.w_t0, w_prev, pred=None)
    ev1.record()
    torch.cuda.synchronize()
    sync_ms = ev0.elapsed_time(ev1) / reps
    sync_bytes = 2 * K * d * esz + 4 * d * (3 if w_prev is not None else 1)
    # after the forced synchronizations w_prev equals w_t0; a model change that is not zero makes
    # the refresh of xi do its real work
    w_prev.add_(torch.randn_like(w_prev) * 1e-3)
    torch.cuda.synchronize()
    ev0.record()
    for _ in range(reps):
        mon.update_xi(wl.w_t0, w_prev, wl.xi, pred=None)
    ev1.record()
    torch.cuda.synchronize()
    xi_ms = ev0.elapsed_time(ev1) / reps
    # both in one call, the norm taken inside the synchronization pass
    # (w_t0 is moved before each call, outside the timed part: after a synchronization the mean equals
    # w_t0, and a zero change would spare the scaling pass its reads)
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for e0, e1 in pairs:
        wl.w_t0.add_(1e-3)
        e0.record()
        mon.sync_xi(wl.w, wl.w_t0, w_prev, wl.xi, pred=None)
        e1.record()
    torch.cuda.synchronize()
    sync_xi_ms = sum(e0.elapsed_time(e1) for e0, e1 in pairs) / reps
    # the write-only synchronization from the average model fda_mean_state emitted (xi included)
    mon.mean_state(wl.w, wl.w_t0, xi, w_bar=w_bar)
    torch.cuda.synchronize()
    ev0.record()
    for _ in range(reps):
        mon.sync_from_mean(wl.w, wl.w_t0, w_bar, w_prev=w_prev, xi=wl.xi, pred=None)
    ev1.record()
    torch.cuda.synchronize()
    fused_ms = ev0.elapsed_time(ev1) / reps
    fused_bytes = K * d * esz + 4 * d * 5
    # what a run pays per step when it synchronizes every `period` steps (the synthetic runs of the
    # two configurations that have a step count synchronize about 5 times in 100 steps, resp. every
    # 4-5 steps); never part of `value`
    period = {"cfg2": 20.0, "cfg5": 4.5}.get(args.config)
    amortized = None
    if period is not None:
        amortized = {"sync_every_steps": period,
                     "ms_per_step_incl_syncs": round(ms_per_step + sync_xi_ms / period, 4),
                     "mean_state_mode_ms_per_step_incl_syncs": round(mean_ms + sync_xi_ms / period, 4)}
    # what this chip sustains for a plain copy with 16-byte accesses (read N, write N), the reference the
    # synchronization kernels' mix of reads and writes is compared with: measured here
    cal_n = min(K * d * esz, 2 << 30) // 16 * 16
    cal_src = torch.zeros(cal_n, dtype=torch.uint8, device=dev)
    cal_dst = torch.empty_like(cal_src)
    torch.cuda.synchronize()
    stream_now = torch.cuda.current_stream().cuda_stream
    copy_ms = F.fda_calib_stream(6, cal_src.data_ptr(), cal_dst.data_ptr(), cal_n, 3, stream_now)
    read_ms = F.fda_calib_stream(4, cal_src.data_ptr(), cal_dst.data_ptr(), cal_n, 3, stream_now)
    del cal_src, cal_dst
    sync_info = {"amortized": amortized,
                 "copy_kernel_GBps": round(2 * cal_n / copy_ms / 1e6, 1),
                 "read_kernel_GBps": round(cal_n / read_ms / 1e6, 1),
                 "calibration": f"fda_calib_stream (nontemporal copy / read) over {cal_n} bytes, measured in this run", "sync_from_mean_ms": round(fused_ms, 4),
                 "sync_from_mean_GBps": round(fused_bytes / fused_ms / 1e6, 1),
                 "sync_from_mean_algorithmic_bytes": fused_bytes,
                 "sync_ms": round(sync_ms, 4), "sync_GBps": round(sync_bytes / sync_ms / 1e6, 1),
                 "sync_algorithmic_bytes": sync_bytes, "update_xi_ms": round(xi_ms, 4),
                 "update_xi_GBps": round(20 * d / xi_ms / 1e6, 1),
                 "sync_xi_ms": round(sync_xi_ms, 4), "sync_xi_algorithmic_bytes": sync_bytes + 12 * d,
                 "sync_xi_GBps": round((sync_bytes + 12 * d) / sync_xi_ms / 1e6, 1)}

    out = {
        "metric": "worker-params/s (K*d per step) for local-state+variance check",
        "value": value, "unit": "worker-params/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "ms_per_step_median": round(per_step[len(per_step) // 2], 4), "ms_per_step_min": round(per_step[0], 4),
        "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None,
        # the arithmetic type: drifts, norms and projections in fp32 (fp64 across tiles), sketch cells
        # as exact integers of fp32-rounded terms; the slab's storage type is in config.slab_dtype
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": workload, "K": K, "d": d, "slab_dtype": wl.dtype,
                   "sketch": f"{wl.l}x{wl.m}", "variants": args.variants,
                   "slab_bytes": K * d * esz, "plan": mon.plan,
                   "step": "fda_local_state + fda_estimate_variance + predicated fda_sync_xi "
                           "(decision: no sync)"},
        "roofline": roofline,
        "graph_replay": graph_info,
        "mean_state_mode": mean_info,
        "sync": sync_info,
    }

    if cpu is not None:
        out["cpu_baseline"] = cpu
    print(json.dumps(out))
    mon.close()


if __name__ == "__main__":
    main()
