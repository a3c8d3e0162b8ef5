#!/usr/bin/env python3
"""Benchmark of the DC-ASGD server hot path on one MI355X.

A step is one worker arrival at the parameter server, all of it in HIP
kernels on torch's current stream:
    synthetic worker gradient at the worker's backup  ->  delay-compensated
    push (Eq. 4.1 / Eq. 18) fused with the worker's pull (backup refresh).
For the queued workload a step is one dcasgd_push_batch call over K arrivals
(K gradient launches + one fused launch); element-updates are counted per
arrival either way.  Inputs are resident in HBM before the timed region.

Prints ONE JSON line.  `value` is whole-path element-updates/s; `roofline`
describes the server-update kernel alone (HIP events around it, inside the
timed region); `cpu_baseline` times the CPU oracle on a bounded sample.

After the headline region (untouched by what follows) the default run adds:
a second short leg of the same workload in which the worker kernel leaves
nothing in the last-level cache, so that `roofline.frac_nothing_cached` is the
push against HBM alone; and one short leg per other configuration and for the
synchronous fold, reported under `all_configs`.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published peak
# plain (unpacked, non-FMA-counted) vector issue: 256 CU x 4 SIMD x 16 lanes x 2.4 GHz
VALU_PEAK_TLANE = 256 * 4 * 16 * 2.4e9 / 1e12


def algorithmic_bytes_per_update(wl, unfused: bool = False, bak_bf16: bool = False) -> float:
    """Bytes the method itself must move per element per applied push
    (fused push+pull): reads w, backup, gradient (+MeanSquare), writes w,
    backup (+MeanSquare).  Queue of K: w/MeanSquare once per queue."""
    g = 2 if wl.grad_bf16 else 4
    b = 2 if bak_bf16 else 4        # backup element, read once and written once per push
    adaptive = wl.mode == 1
    if wl.order == "sync":      # fold: w (+MeanSquare) once, K gradients, no backups
        return ((16 if adaptive else 8) + wl.K * g) / wl.K
    if wl.K > 1:
        per_queue = (16 if adaptive else 8) + wl.K * (g + b + b)
        return per_queue / wl.K
    # unfused: the separate pull reads w once more
    return (4 + b + g + 4 + b) + (8 if adaptive else 0) + (4 if unfused else 0)


def read_profile(name: str, key: str = "traffic_bytes_per_launch"):
    """A per-launch figure (HBM bytes, VALU instructions) from the committed
    rocprofv3 counter summary of this kernel and workload, if there is one."""
    path = os.path.join(ROOT, "profiles", "pmc_%s.txt" % name)
    try:
        m = re.search(r"^%s:\s*([0-9.eE+]+)" % key, open(path).read(), re.M)
        return float(m.group(1)) if m else None
    except OSError:
        return None


def read_probe(key: str, size: str):
    """A ceiling the stand-alone memory probe measured (GB/s), from its committed summary:
    `key` for the vector length `size` ("25m" or "138m")."""
    path = os.path.join(ROOT, "profiles", "membw_probe_mi355x.txt")
    try:
        m = re.search(r"^%s_%s:\s*([0-9.eE+]+)" % (key, size), open(path).read(), re.M)
        return float(m.group(1)) if m else None
    except OSError:
        return None


def device_clock_hz(lib, device_index: int):
    """Peak engine clock the HIP runtime reports for the device (hipDeviceGetAttribute,
    hipDeviceAttributeClockRate: the sixth enumerator of the public header, kilohertz),
    resolved through the already loaded library's dependency on the runtime; None if the
    runtime does not answer."""
    import ctypes
    try:
        fn = lib.hipDeviceGetAttribute
    except AttributeError:
        return None
    fn.restype, fn.argtypes = ctypes.c_int, [ctypes.POINTER(ctypes.c_int), ctypes.c_int, ctypes.c_int]
    khz = ctypes.c_int(0)
    if fn(ctypes.byref(khz), 5, int(device_index)) != 0 or khz.value <= 0:
        return None
    return khz.value * 1e3


def cpu_baseline(wl, target_s: float, bak_bf16: bool = False):
    """Time the oracle (as it stands) on a bounded sample of the workload:
    a leading slice of the parameter vector, the workload's arrival order
    (continued with the same generator if the sample needs more arrivals)."""
    import numpy as np
    import oracle
    cores = min(16, len(os.sched_getaffinity(0)))
    n = min(wl.d, 32 << 20)
    hd = wl.hdiag()[:n]
    ws = wl.wstar()[:n]

    def timed(T, threads):
        order = wl.replace(T=-(-T // wl.K) * wl.K).arrivals()[:T]
        sv = oracle.Server(np.zeros(n, dtype=np.float32), wl.M, wl.eta, wl.lambda0, wl.mode,
                           wl.ema_m, wl.eps)
        if bak_bf16:
            sv.set_backup_bf16()
        t0 = time.perf_counter()
        sv.run(order, hd, ws, wl.sigma, wl.seed, as_bf16=wl.grad_bf16, nthreads=threads)
        return time.perf_counter() - t0

    def timed_server_only(T):
        """push + pull per arrival on one thread, gradients formed beforehand (untimed)."""
        order = wl.replace(T=-(-T // wl.K) * wl.K).arrivals()[:T]
        sv = oracle.Server(np.zeros(n, dtype=np.float32), wl.M, wl.eta, wl.lambda0, wl.mode,
                           wl.ema_m, wl.eps)
        if bak_bf16:
            sv.set_backup_bf16()
        spent = 0.0
        for t, m in enumerate(order):
            g = oracle.synth_grad(sv.bak(int(m)), hd, ws, wl.sigma, wl.seed, t, as_bf16=wl.grad_bf16)
            t0 = time.perf_counter()
            sv.push(int(m), g)
            sv.pull(int(m))
            spent += time.perf_counter() - t0
        return spent

    def cpu_model():
        try:
            for line in open("/proc/cpuinfo"):
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
        except OSError:
            pass
        return "unknown"

    probe = 8
    dt = timed(probe, cores)
    T = int(max(probe, min(20000, target_s / max(dt / probe, 1e-9))))
    dt = timed(T, cores)
    # the oracle as specified is sequential: one thread, a quarter of the time budget
    T1 = int(max(1, min(T, 0.25 * target_s / max(dt / T * cores, 1e-9))))
    dt1 = timed(T1, 1)
    dts = timed_server_only(T1)
    return {"value": n * T / dt, "unit": "element-updates/s", "cores": cores, "kind": "oracle",
            "cpu": cpu_model(), "host_threads_available": len(os.sched_getaffinity(0)),
            "server_only_one_core": {"value": n * T1 / dts, "unit": "element-updates/s",
                                     "sample": "%d arrivals, push + pull only (the gradient is "
                                               "formed outside the timed calls), 1 thread, %.1f s"
                                               % (T1, dts)},
            "sample": "first %d of %d elements, %d arrivals in the workload's order, "
                      "gradient+push+pull per arrival, %d threads over element chunks, %.1f s"
                      % (n, wl.d, T, cores, dt),
            "one_core": {"value": n * T1 / dt1, "unit": "element-updates/s",
                         "sample": "%d arrivals, 1 thread, %.1f s" % (T1, dt1)}}


def measure(args, workload: str, n_steps: int, n_warm: int, *, uncached_worker: bool = False,
            arrivals_iid: bool = False, extras: bool = False) -> dict:
    """Time n_steps steps of one workload (after n_warm untimed ones) and return the report:
    the keys of the JSON line, `roofline` for the server-update kernel included.
    uncached_worker: the worker kernel reads its snapshot and writes its gradient
    non-temporally, so the push finds nothing in the last-level cache.
    arrivals_iid (queued workloads): the queue is filled by independent uniform arrivals
    instead of distinct workers; it is then delivered in pieces that hold distinct workers,
    because a repeated worker's second gradient needs the snapshot its first push leaves.
    extras: also run the optional paths the command line asks for."""
    import numpy as np
    import torch
    from paper_1609_08326_amd import binding as B
    from paper_1609_08326_amd import workloads as W

    wl = W.get(workload)
    own_mode = wl.mode
    if args.variant == "c":
        wl = wl.replace(name=wl.name + "+c", mode=W.MODE_C, lambda0=0.04, ema_m=0.0, eps=0.0)
    elif args.variant == "a":
        wl = wl.replace(name=wl.name + "+a", mode=W.MODE_A, lambda0=2.0, ema_m=0.95, eps=1e-7)
    sync = wl.order == "sync"
    batched = wl.K > 1 and not sync
    K = wl.K
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    order_wl = wl.replace(T=(n_steps + n_warm) * K)
    if arrivals_iid and batched:
        order_wl = order_wl.replace(order="iid")
    arrivals = order_wl.arrivals()

    hd = torch.from_numpy(wl.hdiag()).to(dev)
    ws = torch.from_numpy(wl.wstar()).to(dev)
    w = torch.from_numpy(wl.w0()).to(dev)
    sv = B.Server(w, wl.M, wl.eta, wl.lambda0, wl.mode, wl.ema_m, wl.eps,
                  grad_bf16=wl.grad_bf16, pull_on_push=not batched and not args.unfused,
                  bak_bf16=args.bak_bf16)
    if args.threads or args.items or args.max_blocks or args.streaming >= 0:
        sv.set_launch(args.threads, args.items, args.max_blocks,
                      args.streaming if args.streaming >= 0 else 2)
    gdt = torch.bfloat16 if wl.grad_bf16 else torch.float32
    gbuf = [torch.empty(wl.d, dtype=gdt, device=dev) for _ in range(K)]

    # Server-update launches carry their own start/stop HIP events (attached to
    # the kernel by the library), so their distance is the kernel's duration.
    use_events = not args.no_events
    # (launch-bound 1 MB workloads: the extra host work of an event-carrying
    # launch would dominate, so they are timed by stream events instead)
    kernel_events = use_events and wl.d * 4 >= (16 << 20)
    stream_events = use_events and (args.stream_events or not kernel_events)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(n_steps)] \
        if stream_events else None
    pieces_launched = [0]

    def pieces_of(ms_):
        """Consecutive runs of a queue that hold distinct workers."""
        start = 0
        while start < len(ms_):
            end = start + 1
            while end < len(ms_) and ms_[end] not in ms_[start:end]:
                end += 1
            yield start, end
            start = end

    def step(i: int, rec) -> None:
        base = i * K
        ms_ = [int(m) for m in arrivals[base:base + K]]
        if rec:
            rec[0].record()
        if batched and arrivals_iid:
            for start, end in pieces_of(ms_):
                for j in range(start, end):
                    B.synth_grad(sv.snapshot(ms_[j]), hd, ws, wl.sigma, wl.seed, base + j, gbuf[j],
                                 threads=args.synth_threads, items=args.synth_items,
                                 uncached=uncached_worker)
                sv.push_batch(ms_[start:end], gbuf[start:end])
                pieces_launched[0] += 1
            if rec:
                rec[1].record()
                rec[2].record()
            return
        for j, m in enumerate(ms_):
            B.synth_grad(sv.w if sync else sv.snapshot(m), hd, ws, wl.sigma, wl.seed, base + j,
                         gbuf[j], threads=args.synth_threads, items=args.synth_items,
                         uncached=uncached_worker)
        if rec:
            rec[1].record()
        if sync:
            sv.sync_fold(gbuf, wl.eta * K)
        elif batched:
            sv.push_batch(ms_, gbuf)
        else:
            sv.push(ms_[0], gbuf[0])
            if args.unfused:
                sv.pull(ms_[0])
        if rec:
            rec[2].record()

    for i in range(n_warm):
        step(i, None)
    torch.cuda.synchronize()
    pieces_launched[0] = 0

    def timed_region():
        if kernel_events:
            sv.timing(True)
        t_start = time.perf_counter()
        for i in range(n_steps):
            step(n_warm + i, ev[i] if stream_events else None)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t_start
        each = None
        try:
            if kernel_events:
                each = sv.timing_read_each()
                ms, launches = float(each.sum(dtype="float64")), int(each.size)
            else:
                ms, launches = 0.0, 0
        except B.DcasgdError:
            ms, launches = 0.0, 0
        sv.timing(False)
        return dt, ms, launches, each

    elapsed, kernel_ms, kernel_launches, kernel_each = timed_region()
    if kernel_events and (kernel_launches == 0 or not kernel_ms > 0.0):
        # the runtime gave no times for launch-attached events: measure again
        # with stream events around the kernels instead
        kernel_events, stream_events = False, True
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(n_steps)]
        pieces_launched[0] = 0
        elapsed, kernel_ms, kernel_launches, kernel_each = timed_region()

    updates = wl.d * K * n_steps
    value = updates / elapsed
    unfused = args.unfused and K == 1 and not sync
    bpu = algorithmic_bytes_per_update(wl, unfused, args.bak_bf16)
    kname = ("sync_fold_J%d" % K if sync else "push_batch_K%d" % K if batched
             else "push_then_pull" if unfused else "push_fused")
    if wl.mode != own_mode:
        kname += "_" + args.variant      # another kernel than the workload's own: its own profile
    if args.bak_bf16 and not sync:
        kname += "_bak16"
    out = {
        "metric": "element-updates/sec",
        "value": value,
        "unit": "element-updates/s",
        "n_gpus": 1,
        "steps": n_steps,
        "warmup": n_warm,
        "ms_per_step": 1e3 * elapsed / n_steps,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if not wl.grad_bf16 else "f32 (bf16 gradients)",
        "data": "synthetic",
        "config": {"workload": wl.name, "d": wl.d, "M": wl.M, "K": K,
                   "variant": "DC-ASGD-a" if wl.mode == 1 else "DC-ASGD-c",
                   "snapshots": "bf16" if args.bak_bf16 else "f32",
                   "arrivals": ("independent uniform draws; a queue is delivered in pieces of "
                                "distinct workers" if arrivals_iid and batched else
                                {"round_robin": "round robin", "iid": "independent uniform draws",
                                 "queues": "per queue a random choice of K distinct workers (one "
                                           "gradient in flight per worker, Algorithm 1)",
                                 "sync": "none (all gradients taken at the current model)"}[wl.order]),
                   "worker_kernel": ("leaves nothing in the last-level cache" if uncached_worker else
                                     "leaves its snapshot and gradient cacheable"),
                   "step": ("synth_grad x%d + synchronous fold" if sync else
                            "synth_grad x%d + fused push+pull") % K},
    }
    if use_events:
        if kernel_events:
            push_ms = kernel_ms / n_steps        # server-update kernel time per step
        else:
            push_ms = sum(e[1].elapsed_time(e[2]) for e in ev) / n_steps
            kernel_launches = n_steps
        launch_bytes = bpu * wl.d * K
        achieved = launch_bytes / (push_ms * 1e-3) / 1e9
        pname = "%s_%s" % (kname, wl.name.split("_")[0])
        out["roofline"] = {"bound": "hbm", "kernel": kname, "achieved": achieved,
                           "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                           "traffic": read_profile(pname),
                           "traffic_source": "profiles/pmc_%s.txt (rocprofv3 FETCH_SIZE and "
                                             "WRITE_SIZE of this kernel and workload, committed; "
                                             "not measured in this run)" % pname,
                           "avg_launch_ms": push_ms,
                           "algorithmic_bytes_per_launch": launch_bytes,
                           "bytes_per_element_update": bpu}
        valu = read_profile(pname, "valu_instr_per_launch")
        if batched and arrivals_iid:
            valu = None                  # the committed counters are of whole, unsplit queues
        # the same vector-issue peak at the engine clock and unit count this device reports
        props = torch.cuda.get_device_properties(dev)
        clock_hz = device_clock_hz(B.load(), dev.index or 0)
        device_peak = props.multi_processor_count * 4 * 16 * clock_hz / 1e12 if clock_hz else None
        if valu:
            # vector issue: measured wavefront VALU instructions per launch x 64 lanes / time
            lane_rate = valu * 64 / (push_ms * 1e-3) / 1e12
            out["roofline"]["alu_achieved_Tlane_per_s"] = lane_rate
            out["roofline"]["alu_peak_Tlane_per_s"] = VALU_PEAK_TLANE
            out["roofline"]["alu_frac"] = lane_rate / VALU_PEAK_TLANE
            out["roofline"]["valu_instr_per_element_update"] = valu * 64 / (wl.d * K)
            if device_peak:
                out["roofline"]["alu_peak_at_device_reported_clock"] = {
                    "compute_units": props.multi_processor_count, "clock_GHz": clock_hz / 1e9,
                    "peak_Tlane_per_s": device_peak, "frac": lane_rate / device_peak}
        if sync and valu:
            # the fold moves 5 B per update and is bound by vector issue instead
            hbm = out["roofline"]
            out["roofline"] = {"bound": "alu", "kernel": kname, "achieved": lane_rate,
                               "peak": VALU_PEAK_TLANE, "unit": "T lane-instr/s",
                               "frac": lane_rate / VALU_PEAK_TLANE,
                               "traffic": hbm["traffic"], "traffic_source": hbm["traffic_source"],
                               "avg_launch_ms": push_ms,
                               "hbm_achieved_GBs": achieved, "hbm_frac": achieved / HBM_PEAK_GBS,
                               "valu_instr_per_element_update": valu * 64 / (wl.d * K),
                               "alu_peak_at_device_reported_clock":
                                   hbm.get("alu_peak_at_device_reported_clock"),
                               "algorithmic_bytes_per_launch": launch_bytes,
                               "bytes_per_element_update": bpu}
        out["server_update_only"] = {"value": wl.d * K / (push_ms * 1e-3),
                                     "unit": "element-updates/s"}
        if kernel_events and kernel_each is not None and kernel_each.size >= n_steps \
                and kernel_each.size % n_steps == 0:
            # spread over the region: server-kernel time of each step (its launches added up)
            per_step = kernel_each.reshape(n_steps, -1).sum(axis=1, dtype="float64")
            p10, p50, p90 = (float(x) for x in np.percentile(per_step, [10, 50, 90]))
            out["roofline"]["launch_ms_p10_median_p90"] = [p10, p50, p90]
        out["roofline"]["launches_timed"] = kernel_launches
        out["roofline"]["timed_by"] = ("HIP events attached to each launch" if kernel_events
                                       else "HIP stream events around each launch")
        if batched and arrivals_iid:
            out["roofline"]["launches_per_queue"] = pieces_launched[0] / n_steps
        out["worker_and_gaps_ms_per_step"] = 1e3 * elapsed / n_steps - push_ms
        if stream_events:
            synth_ms = sum(e[0].elapsed_time(e[1]) for e in ev) / n_steps
            synth_bytes = (8 + (2 if args.bak_bf16 else 4) + (2 if wl.grad_bf16 else 4)) * wl.d * K
            out["stream_event_intervals"] = {
                "worker_ms_per_step": synth_ms,
                "server_ms_per_step": sum(e[1].elapsed_time(e[2]) for e in ev) / n_steps,
                "worker_achieved_GBs": synth_bytes / (synth_ms * 1e-3) / 1e9}
    if not extras:
        out["_wl"] = wl
        return out
    if args.fused_worker and K == 1:
        # same arrivals, one launch per arrival: the gradient never leaves registers
        torch.cuda.synchronize()
        for i in range(n_warm):
            sv.push_synth(int(arrivals[i]), hd, ws, wl.sigma, wl.seed)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(n_steps):
            sv.push_synth(int(arrivals[n_warm + i]), hd, ws, wl.sigma, wl.seed)
        torch.cuda.synchronize()
        fe = time.perf_counter() - t0
        fbytes = (32 + (0 if wl.mode == 1 else -8) - (4 if args.bak_bf16 else 0)) * wl.d
        out["fused_worker_path"] = {"value": wl.d * n_steps / fe, "unit": "element-updates/s",
                                    "ms_per_step": 1e3 * fe / n_steps,
                                    "algorithmic_GBs": fbytes * n_steps / fe / 1e9,
                                    "bytes_per_element_update": fbytes / wl.d,
                                    "note": "synthetic workload only: worker gradient formed in "
                                            "registers inside the push kernel"}
    if args.native_loop and K == 1 and not sync:
        # the same arrivals through the library's own event loop (one C call; one launch per
        # block of 64 arrivals, the parameters staying in registers over the block)
        torch.cuda.synchronize()
        sv.run_synth(arrivals[:n_warm], hd, ws, wl.sigma, wl.seed)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        sv.run_synth(arrivals[n_warm:n_warm + n_steps], hd, ws, wl.sigma, wl.seed)
        torch.cuda.synchronize()
        ne = time.perf_counter() - t0
        # per arrival and parameter: the pusher's backup read and written; w, MeanSquare, h, w*
        # read and w, MeanSquare written once per block of 64
        b = 2 if args.bak_bf16 else 4
        nbytes = 2 * b + ((16 if wl.mode == 1 else 12) + (8 if wl.mode == 1 else 4)) / 64.0
        out["native_loop_path"] = {"value": wl.d * n_steps / ne, "unit": "element-updates/s",
                                   "ms_per_step": 1e3 * ne / n_steps,
                                   "bytes_per_element_update": nbytes,
                                   "algorithmic_GBs": nbytes * wl.d * n_steps / ne / 1e9,
                                   "note": "synthetic workload only: dcasgd_run_synth, worker "
                                           "fused into the push, 64 arrivals per launch with w, "
                                           "MeanSquare, h and w* held in registers"}
        valu = read_profile("run_synth_blocks_%s" % wl.name.split("_")[0], "valu_instr_per_launch")
        if valu and not args.bak_bf16 and not args.variant:
            # counted over launches of 64 arrivals; wall clock of the whole call here
            per_update = valu * 64 / (wl.d * 64.0)
            lane_rate = per_update * wl.d * n_steps / ne / 1e12
            out["native_loop_path"].update({
                # 1 MB vectors give each SIMD two waves: the chains' latency, not issue, bounds them
                "bound": "alu" if wl.d * 4 >= (16 << 20) else "instruction latency (two waves per SIMD)",
                "valu_instr_per_element_update": per_update,
                "alu_achieved_Tlane_per_s": lane_rate, "alu_peak_Tlane_per_s": VALU_PEAK_TLANE,
                "alu_frac": lane_rate / VALU_PEAK_TLANE,
                "alu_note": "the peak counts one wave instruction per SIMD every four cycles, "
                            "which is what float32 add, multiply, fma, selects and integer "
                            "multiplies take; adds, shifts, logic and moves on integers issue "
                            "about twice as fast and sqrt/rcp/rsq half as fast "
                            "(profiles/membw_probe_mi355x.txt, 'issue'), so a mix rich in the "
                            "former can read above 1"})
    if args.ordered and sync:
        # norms + ranking + fold over the ranked list: three launches per fold
        fws = B.Server.fold_workspace(dev)

        def ordered_step(i: int) -> None:
            for j in range(K):
                B.synth_grad(sv.w, hd, ws, wl.sigma, wl.seed, i * K + j, gbuf[j],
                             threads=args.synth_threads, items=args.synth_items)
            sv.sync_fold(gbuf, wl.eta * K, workspace=fws)

        base_i = n_warm + n_steps
        for i in range(n_warm):
            ordered_step(base_i + i)
        torch.cuda.synchronize()
        if kernel_events:
            sv.timing(True)
        t0 = time.perf_counter()
        for i in range(n_steps):
            ordered_step(base_i + n_warm + i)
        torch.cuda.synchronize()
        oe = time.perf_counter() - t0
        o_ms, o_launches = sv.timing_read() if kernel_events else (0.0, 0)
        sv.timing(False)
        gbytes = (2 if wl.grad_bf16 else 4) * wl.d * K
        rep = {"value": updates / oe, "unit": "element-updates/s",
               "ms_per_step": 1e3 * oe / n_steps,
               "note": "squared norms, ranking and fold: three launches, no host round trip"}
        if o_launches:
            extra = o_ms / n_steps - out["roofline"]["avg_launch_ms"]
            rep.update({"server_ms_per_fold": o_ms / n_steps, "launches_timed": o_launches,
                        "norms_and_ranking_ms": extra,
                        "norm_pass_algorithmic_GBs": gbytes / (extra * 1e-3) / 1e9})
        out["ordered_fold_path"] = rep
    if args.graph > 0 and K == 1 and not sync:
        # The push counter moves to device memory, so the captured launches keep
        # drawing fresh noise on every replay; the block of arrivals repeats.
        G = args.graph
        block = [int(m) for m in arrivals[:G]]
        side = torch.cuda.Stream()
        torch.cuda.synchronize()

        def run_block():
            for m in block:
                if args.fused_worker:
                    sv.push_synth(m, hd, ws, wl.sigma, wl.seed)
                else:
                    sv.worker_grad(m, hd, ws, wl.sigma, wl.seed, gbuf[0])
                    sv.push(m, gbuf[0])

        with torch.cuda.stream(side):
            sv.bind_counter()
            run_block()
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            run_block()
        replays = max(1, -(-n_steps // G))
        for _ in range(max(1, n_warm // G)):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(replays):
            graph.replay()
        torch.cuda.synchronize()
        ge = time.perf_counter() - t0
        out["graph_replay_path"] = {"value": wl.d * G * replays / ge, "unit": "element-updates/s",
                                    "us_per_arrival": 1e6 * ge / (G * replays),
                                    "arrivals_per_graph": G, "replays": replays,
                                    "note": ("worker fused into the push, " if args.fused_worker
                                             else "worker gradient + fused push+pull per arrival, ")
                                            + "launches replayed from one HIP graph"}
    out["_wl"] = wl
    return out


def leg_summary(rep: dict) -> dict:
    """The figures of one extra leg that go under `all_configs`."""
    r = rep.get("roofline", {})
    d = {"workload": rep["config"]["workload"], "arrivals": rep["config"]["arrivals"],
         "steps": rep["steps"], "warmup": rep["warmup"],
         "value": rep["value"], "unit": rep["unit"], "ms_per_step": rep["ms_per_step"]}
    if r:
        d.update({"kernel": r["kernel"], "avg_launch_ms": r["avg_launch_ms"],
                  "bytes_per_element_update": r["bytes_per_element_update"],
                  "server_update_only": rep["server_update_only"]["value"],
                  "timed_by": r["timed_by"]})
        for k in ("alu_frac", "valu_instr_per_element_update", "launches_per_queue",
                  "launch_ms_p10_median_p90"):
            if k in r:
                d[k] = r[k]
        if r["bound"] == "alu":
            d.update({"bound": "alu", "frac": r["frac"], "hbm_frac": r["hbm_frac"],
                      "hbm_achieved_GBs": r["hbm_achieved_GBs"]})
        elif rep["config"]["d"] * 4 < (16 << 20):
            # 1 MB vectors: a launch takes longer to issue than to run; no roofline applies
            d.update({"bound": "launch latency", "frac": None, "achieved_GBs": r["achieved"]})
        else:
            d.update({"bound": "hbm", "frac": r["frac"], "achieved_GBs": r["achieved"]})
            if r["kernel"] == "push_fused" and rep["config"]["variant"] == "DC-ASGD-a":
                # the probe's figure for the same 4-read/3-write mix at the nearer vector length
                ceiling = read_probe("practical_ceiling_4r3w_GBs",
                                     "25m" if rep["config"]["d"] < 60_000_000 else "138m")
                if ceiling:
                    d["practical_ceiling_GBs"] = ceiling
                    d["frac_of_practical"] = r["achieved"] / ceiling
    for k in ("native_loop_path", "fused_worker_path", "ordered_fold_path", "graph_replay_path"):
        if k in rep:
            d[k] = {kk: vv for kk, vv in rep[k].items() if kk != "note"}
    d["variant"] = rep["config"]["variant"]
    d["snapshots"] = rep["config"]["snapshots"]
    return d


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg2")
    ap.add_argument("--threads", type=int, default=0)
    ap.add_argument("--items", type=int, default=0)
    ap.add_argument("--max-blocks", type=int, default=0)
    ap.add_argument("--streaming", type=int, default=-1, help="0..3 (see dcasgd_set_launch)")
    ap.add_argument("--synth-threads", type=int, default=0)
    ap.add_argument("--synth-items", type=int, default=0)
    ap.add_argument("--fused-worker", action="store_true",
                    help="also time the worker+push fusion (dcasgd_push_synth) and report it "
                         "under 'fused_worker_path'; K=1 workloads only")
    ap.add_argument("--variant", choices=["a", "c"], default=None,
                    help="override the workload's variant (c: constant lambda 0.04, a: adaptive "
                         "lambda0 2, m 0.95, eps 1e-7) to time the other kernel at the same size")
    ap.add_argument("--unfused", action="store_true",
                    help="K=1 workloads: push and pull as two launches (24 + 8 bytes per update "
                         "in the adaptive variant) instead of the fused one")
    ap.add_argument("--graph", type=int, default=0, metavar="G",
                    help="also capture a block of G arrivals (worker gradient + push each) into a "
                         "HIP graph and time its replays, reported under 'graph_replay_path'; "
                         "meant for the launch-bound 1 MB workloads, K=1 only")
    ap.add_argument("--no-events", action="store_true",
                    help="no per-kernel events at all (whole-path timing only)")
    ap.add_argument("--stream-events", action="store_true",
                    help="additionally record stream events between the kernels of a step and "
                         "report their intervals (adds a dispatch gap per event)")
    ap.add_argument("--bak-bf16", action="store_true",
                    help="snapshots handed out and kept as bfloat16 (a storage variant; the "
                         "default measures the float32 backups of the configurations)")
    ap.add_argument("--native-loop", action="store_true",
                    help="additionally time the same arrivals through dcasgd_run_synth")
    ap.add_argument("--ordered", action="store_true",
                    help="fold workload: after the timed region, time the same steps again "
                         "with the gradients ranked by norm on the device before each fold")
    ap.add_argument("--uncached-worker", action="store_true",
                    help="the worker kernel leaves nothing in the last-level cache (the headline "
                         "leaves its snapshot and gradient cacheable)")
    ap.add_argument("--iid-queues", action="store_true",
                    help="queued workload: fill the queues by independent uniform arrivals")
    ap.add_argument("--legs", default="default",
                    help="'default': after the headline region also the nothing-cached leg and "
                         "one leg per other configuration and further kernel (reported under "
                         "all_configs) when the workload is the headline one and no variant flag "
                         "is given; 'none': headline only; or a comma list of cfg0,cfg1,cfg2nc,cfg3,"
                         "cfg3iid,cfg4,fold,cfg2_variant_c,cfg2_bf16_snapshots,cfg2_fused_worker,"
                         "fold_ordered")
    ap.add_argument("--cpu-seconds", type=float, default=15.0,
                    help="CPU oracle sample length; 0 skips the baseline")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the path shards by index range, "
              "one GPU holds one shard); --gpus %d is not supported" % args.gpus, file=sys.stderr)
        return 2

    n_steps, n_warm = args.steps, args.warmup
    out = measure(args, args.workload, n_steps, n_warm, uncached_worker=args.uncached_worker,
                  arrivals_iid=args.iid_queues, extras=True)
    wl = out.pop("_wl")

    plain = not (args.variant or args.unfused or args.bak_bf16 or args.uncached_worker or
                 args.iid_queues or args.no_events or args.threads or args.items or
                 args.max_blocks or args.streaming >= 0)
    if args.legs == "default":
        legs = ["cfg2nc", "cfg3", "cfg3iid", "cfg4", "fold", "cfg0", "cfg1",
                "cfg2_variant_c", "cfg2_bf16_snapshots", "cfg2_fused_worker", "fold_ordered"] \
            if plain and wl.name.startswith("cfg2") else []
    elif args.legs == "none":
        legs = []
    else:
        legs = [x for x in args.legs.split(",") if x]

    def leg_args(**kw):
        a = argparse.Namespace(**vars(args))
        a.fused_worker = a.ordered = a.native_loop = False
        a.graph = 0
        for k, v in kw.items():
            setattr(a, k, v)
        return a

    all_configs = {}
    for leg in legs:
        small = leg in ("cfg0", "cfg1")
        # the launch-bound 1 MB configurations need more arrivals for a stable figure
        ls, lw = (max(n_steps, 400), max(n_warm, 50)) if small else (min(n_steps, 40), min(n_warm, 5))
        if leg == "cfg2nc":
            rep = measure(leg_args(), "cfg2", min(n_steps, 100), min(n_warm, 10),
                          uncached_worker=True)
            if "roofline" in out and "roofline" in rep:
                r, nc = out["roofline"], rep["roofline"]
                ceiling = read_probe("practical_ceiling_4r3w_GBs", "25m")
                r["achieved_nothing_cached"] = nc["achieved"]
                r["frac_nothing_cached"] = nc["frac"]
                r["avg_launch_ms_nothing_cached"] = nc["avg_launch_ms"]
                r["practical_ceiling_GBs"] = ceiling
                r["probe_sustained_GBs"] = read_probe("sustained_4r3w_GBs", "25m")
                r["practical_ceiling_source"] = ("profiles/membw_probe_mi355x.txt: plain 4-read/"
                                                 "3-write streaming kernels with nothing cacheable, "
                                                 "same vector length: the best figure any variant "
                                                 "reached, and the rate the library's shape sustains "
                                                 "over two seconds (committed; not measured in this "
                                                 "run)")
                if ceiling:
                    r["frac_of_practical"] = nc["achieved"] / ceiling
                r["which_is_hbm_only"] = (
                    "frac counts algorithmic bytes against the HBM peak in the workload as it runs: "
                    "the worker kernel has just read the snapshot and written the gradient, both "
                    "fit the 256 MB last-level cache, and the push finds them there - that figure "
                    "is HBM plus last-level cache. frac_nothing_cached is the same kernel with the "
                    "worker's accesses non-temporal: every byte comes from and goes to HBM; it is "
                    "the figure to hold against an HBM-bandwidth target.")
            rep.pop("_wl", None)
            continue
        # further kernels at the headline size: the constant-lambda push, bfloat16 snapshots,
        # the worker fused into the push, and the fold ranked by norm on the device
        special = {"cfg2_variant_c": ("cfg2", dict(variant="c")),
                   "cfg2_bf16_snapshots": ("cfg2", dict(bak_bf16=True)),
                   "cfg2_fused_worker": ("cfg2", dict(fused_worker=True, native_loop=True)),
                   "fold_ordered": ("fold", dict(ordered=True))}
        if leg in special:
            name, overrides = special[leg]
            rep = measure(leg_args(**overrides), name, ls, lw, extras=True)
            rep.pop("_wl", None)
            all_configs[leg] = leg_summary(rep)
            continue
        name = {"cfg3iid": "cfg3"}.get(leg, leg)
        rep = measure(leg_args(native_loop=small, graph=64 if small else 0), name, ls, lw,
                      arrivals_iid=(leg == "cfg3iid"),
                      extras=small)
        rep.pop("_wl", None)
        all_configs[leg] = leg_summary(rep)
    if all_configs:
        all_configs["cfg2"] = leg_summary(out)
        out["all_configs"] = dict(sorted(all_configs.items()))

    if args.cpu_seconds > 0 and wl.order != "sync":
        out["cpu_baseline"] = cpu_baseline(wl, args.cpu_seconds, args.bak_bf16)
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
