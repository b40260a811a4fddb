#!/usr/bin/env python3
"""Benchmark of the emulated lane-aware all-reduce on one MI355X.

One "step" is one whole all-reduce (every launch of the schedule) over P resident rank buffers.
Prints ONE JSON line: whole-job HBM GB/s (algorithmic bytes of the schedule / time), the roofline
of the dominant kernel (per-launch duration from HIP events recorded on the launch stream inside
the timed region), and the CPU oracle timed on the host cores as a reported baseline.
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

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published

# HBM-side bytes per launch of a step, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this
# file (FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0, the factors calibrated on the ring's plain-copy launches
# of known size; profiles/seg_reduce_kernel_c2_lane_pmc.md).  Keyed by (config, algo, flags, stage).
MEASURED_TRAFFIC = {
    ("c2", "lane", 0, "S1"): 1342274596,
    ("c2", "lane", 0, "S2"): 268528640 + 268435456,
    ("c2", "lane", 0, "S3"): 268525917 + 806258048,
    # profiles/seg_reduce_kernel_c3_c4_c5.md
    ("c3", "lane_multiproc", 0, "S1"): 2147902929 + 134217728,
    ("c3", "lane_multiproc", 0, "S3"): 134673303 + 2015343919,
    ("c4", "lane_multiproc", 0, "S1"): 4295180870 + 536934330,
    ("c4", "lane_multiproc", 0, "S3"): 537058385 + 3758096384,
    ("c5", "lane_multiproc", 0, "S1"): 4296550633 + 134217728,
    ("c5", "lane_multiproc", 0, "S3"): 135180544 + 4164127663,
}

CONFIGS = {
    "c1": dict(topo=(2, 4, 1), algo="lane", n=1 << 16, dist="uniform_pm1", dtype="float32",
               name="C1 tiny: 2 nodes x 4 GPUs x 1 proc = 8 ranks, 65,536 fp32 per rank (cache-resident)"),
    "c2": dict(topo=(4, 4, 1), algo="lane", n=1 << 24, dist="normal", dtype="float32",
               name="C2: 4 nodes x 4 GPUs x 1 proc = 16 ranks, fp32 SUM, 16 Mi elements (64 MiB) per rank, N(0,1)"),
    "c3": dict(topo=(8, 4, 4), algo="lane_multiproc", n=1 << 22, dist="uniform_pm1", dtype="float32",
               name="C3: 8 nodes x 4 GPUs x 4 procs = 128 ranks, fp32 SUM, 4 Mi elements (16 MiB) per rank"),
    "c4": dict(topo=(2, 4, 2), algo="lane_multiproc", n=1 << 27, dist="normal_bf16", dtype="bfloat16",
               name="C4: 2 nodes x 4 GPUs x 2 procs = 16 ranks, bf16 in / fp32 acc, 128 Mi elements (256 MiB) per rank"),
    "c5": dict(topo=(32, 4, 8), algo="lane_multiproc", n=1 << 20, dist="uniform_pm1", dtype="float32",
               name="C5: 32 nodes x 4 GPUs x 8 procs = 1024 ranks, fp32 SUM, 1 Mi elements (4 MiB) per rank"),
    # the size the paper's 8-node runs are quoted on, in the shared-buffer model (one buffer per GPU,
    # 16 processes per GPU on slices of it): 32 buffers of 512 MiB
    "paper8": dict(topo=(8, 4, 16), algo="lane_multiproc", n=1 << 27, dist="uniform_pm1", dtype="float32", flags=8,
                   name="paper size: 8 nodes x 4 GPUs, 2^27 fp32 (512 MiB) per GPU buffer, 16 processes per GPU "
                        "sharing it (multi-lane approach; --algo ring = standard approach)"),
}
DTYPE_TAG = {"float32": "f32", "int32": "i32", "bfloat16": "bf16 in, f32 accumulate"}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="c2", choices=sorted(CONFIGS))
    ap.add_argument("--algo", default=None, choices=["ring", "lane", "lane_multiproc"])
    ap.add_argument("--n", type=int, default=None, help="elements per rank buffer, instead of the configuration's")
    ap.add_argument("--flags", type=int, default=0, help="LA_SCHED_* bits: 1 = point-to-point gather, 2 = staged")
    ap.add_argument("--unroll", type=int, default=None)
    ap.add_argument("--cache-policy", type=int, default=None)
    ap.add_argument("--block", type=int, default=None, help="lanes per workgroup for every step: 256 or 1024")
    ap.add_argument("--skew", type=int, default=0, help="extra bytes between consecutive rank buffers")
    ap.add_argument("--flush-cache", action="store_true",
                    help="overwrite a 1 GiB scratch buffer before every timed all-reduce, so that nothing "
                         "the previous one wrote is left in the last-level cache (the flush is outside "
                         "the per-launch events; ms_per_step then comes from the events)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-ring", action="store_true", help="skip the ring comparison leg of C2")
    return ap.parse_args()


def device_buffers(x, skew_bytes):
    """One device tensor per rank.  With skew, all come from one slab at a stride of
    n*e + skew bytes, so the distance between operands of a segment is not a power of two."""
    import numpy as np
    import torch

    P, n = x.shape
    tdt = {np.dtype(np.float32): torch.float32, np.dtype(np.int32): torch.int32, np.dtype(np.uint16): torch.bfloat16}[x.dtype]

    def up(row):
        if row.dtype == np.uint16:
            return torch.from_numpy(row.view(np.int16)).view(torch.bfloat16)
        return torch.from_numpy(row)

    if skew_bytes == 0:
        return [up(x[r]).cuda() for r in range(P)], None
    e = x.dtype.itemsize
    stride = n + skew_bytes // e
    slab = torch.empty(P * stride, dtype=tdt, device="cuda")
    bufs = [slab[r * stride: r * stride + n] for r in range(P)]
    for r in range(P):
        bufs[r].copy_(up(x[r]))
    return bufs, slab


def plain_copy_ceiling(torch, dominant_gbs):
    """What a plain device-to-device copy of 1 GiB (torch's own copy kernel, 2 GiB of traffic,
    nothing cache-resident) reaches on this GPU, measured here: the second reference, beside the
    published peak, for the dominant kernel's rate."""
    a = torch.empty(1 << 28, dtype=torch.float32, device="cuda").uniform_(-1, 1)
    b = torch.empty_like(a)
    for _ in range(2):
        b.copy_(a)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = 10
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        b.copy_(a)
    e1.record()
    torch.cuda.synchronize()
    gbs = 2 * a.numel() * 4 * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del a, b
    torch.cuda.empty_cache()
    return {"plain_copy_GBps": round(gbs, 1), "what": "torch device copy of 1 GiB (read + write bytes)",
            "dominant_kernel_over_plain_copy": round(dominant_gbs / gbs, 3)}


INSTRUMENT_EVERY = 4


def time_schedule(la, torch, sched, bufs, steps, warmup, flush=None):
    """W warm-up all-reduces, then K timed ones.  Every fourth timed all-reduce (all of them with
    a cache flush) is issued launch by launch with an event after every launch; the others go
    through la_allreduce_emulated, the entry point an application calls.  An event record costs
    the stream several microseconds, so instrumenting every launch of every step would make the
    whole-job figure measure the instrumentation (6 % on a 0.4 ms all-reduce)."""
    stream = torch.cuda.current_stream()
    ptrs = la.ptr_array([b.data_ptr() for b in bufs])
    ns = sched.num_steps
    for _ in range(warmup):
        la.la_allreduce_emulated(sched, ptrs, sched.n, sched.dtype, la.LA_SUM, stream.cuda_stream)
    every = 1 if flush is not None else INSTRUMENT_EVERY
    marked = [k for k in range(steps) if k % every == 0]
    ev = {k: [torch.cuda.Event(enable_timing=True) for _ in range(ns + 1)] for k in marked}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        if flush is not None:
            flush.add_(1.0)
        if k in ev:
            ev[k][0].record(stream)
            for s in range(ns):
                la.la_schedule_run_step(sched, s, ptrs, stream.cuda_stream)
                ev[k][s + 1].record(stream)
        else:
            la.la_allreduce_emulated(sched, ptrs, sched.n, sched.dtype, la.LA_SUM, stream.cuda_stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    per_step_ms = [sum(ev[k][s].elapsed_time(ev[k][s + 1]) for k in marked) / len(marked) for s in range(ns)]
    wall_ms = (t1 - t0) / steps * 1e3
    if flush is not None:  # the wall clock contains the flushes: use the event-to-event time of the launches
        wall_ms = sum(per_step_ms)
    # the same K all-reduces through the one-call entry point, no events in between
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    for _ in range(steps):
        la.la_allreduce_emulated(sched, ptrs, sched.n, sched.dtype, la.LA_SUM, stream.cuda_stream)
    torch.cuda.synchronize()
    t3 = time.perf_counter()
    return wall_ms, per_step_ms, (t3 - t2) / steps * 1e3


def cpu_baseline(cfg, algo, total_bytes_full, shared=False):
    """The oracle as it stands, on the host cores, on a bounded sample of the workload."""
    import oracle
    from paper_2508_13397_amd import synth

    N, G, Q = cfg["topo"]
    P = N * G if shared else N * G * Q
    threads = min(oracle.max_threads(), os.cpu_count() or 1, 16)
    oracle.set_threads(threads)
    n = cfg["n"]
    sample_n = max(n // 16, 1024)
    x = synth.make_inputs(P, sample_n, cfg["dist"])
    t0 = time.perf_counter()
    oracle.allreduce(algo, N, G, Q, x, in_place=True, shared=shared)
    dt = time.perf_counter() - t0
    frac = sample_n / n
    if dt / frac < 25.0 and sample_n < n:  # the full workload fits the time budget: time that instead
        x = synth.make_inputs(P, n, cfg["dist"])
        sample_n, frac = n, 1.0
        runs, spent = [], 0.0
        while len(runs) < 3 and spent < 12.0:  # repeat a short run for a steadier figure
            t0 = time.perf_counter()
            oracle.allreduce(algo, N, G, Q, x, in_place=True, shared=shared)
            runs.append(time.perf_counter() - t0)
            spent += runs[-1]
        dt = sum(runs) / len(runs)
    gbs = total_bytes_full * frac / dt / 1e9
    return {"value": round(gbs, 3), "unit": "GB/s", "cores": threads, "kind": "oracle",
            "sample": f"{algo} schedule, same topology, {sample_n} of {n} elements per rank, "
                      f"{dt:.2f} s wall; GB/s = algorithmic bytes of the GPU schedule for that sample / time",
            "seconds": round(dt, 3)}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU: the P virtual ranks all live in one MI355X's HBM; "
              f"--gpus {args.gpus} is not supported.", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    import paper_2508_13397_amd as la
    from paper_2508_13397_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    la.lib()
    torch.cuda.set_device(0)
    cfg = dict(CONFIGS[args.config])
    if args.n is not None:
        cfg["n"] = args.n
        cfg["name"] += f" [n overridden: {args.n}]"
    algo = args.algo or cfg["algo"]
    if args.unroll is not None:
        la.la_tuning_set("unroll", args.unroll)
    if args.cache_policy is not None:
        la.la_tuning_set("cache_policy", args.cache_policy)
    if args.block is not None:
        la.la_tuning_set("block", args.block)
    N, G, Q = cfg["topo"]
    args.flags |= cfg.get("flags", 0)
    shared = bool(args.flags & la.LA_SCHED_SHARED_BUFFERS)
    P, n = (N * G if shared else N * G * Q), cfg["n"]   # number of buffers
    e = la.ELEM_SIZE[la.DTYPES[cfg["dtype"]]]

    x = synth.make_inputs(P, n, cfg["dist"], workers=16)
    bufs, slab = device_buffers(x, args.skew)
    del x
    topo = la.la_topology_create(N, G, Q)
    sched = la.la_schedule_build(topo, algo, n, cfg["dtype"], args.flags)
    info = sched.steps()
    step_bytes = [s["bytes_read"] + s["bytes_written"] for s in info]
    total_bytes = sum(step_bytes)

    flush = torch.zeros(1 << 28, dtype=torch.float32, device="cuda") if args.flush_cache else None
    ms, per_step_ms, ms_onecall = time_schedule(la, torch, sched, bufs, args.steps, args.warmup, flush)

    # the dominant kernel: the launch (or family of identical launches) with the most time
    fam = {}
    for i, s in enumerate(info):
        key = (s["stage_name"], s["fan_in"], s["fan_out"])
        f = fam.setdefault(key, {"ms": 0.0, "bytes": 0, "launches": 0})
        f["ms"] += per_step_ms[i]
        f["bytes"] += step_bytes[i]
        f["launches"] += 1
    dom_key = max(fam, key=lambda k: fam[k]["ms"])
    dom = fam[dom_key]
    dom_gbs = dom["bytes"] / (dom["ms"] * 1e-3) / 1e9
    kernels = [{"stage": k[0], "fan_in": k[1], "fan_out": k[2], "launches": v["launches"],
                "bytes_per_launch": v["bytes"] // v["launches"], "avg_ms": round(v["ms"] / v["launches"], 5),
                "GBps": round(v["bytes"] / (v["ms"] * 1e-3) / 1e9, 1),
                "frac_of_peak": round(v["bytes"] / (v["ms"] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)} for k, v in fam.items()]

    out = {
        "metric": "segmented-reduce HBM GB/s (% of peak) + emulated allreduce bytes/s per virtual rank",
        "value": round(total_bytes / (ms * 1e-3) / 1e9, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": DTYPE_TAG[cfg["dtype"]],
        "data": "synthetic",
        "config": {"workload": cfg["name"], "config_id": args.config, "algo": algo, "schedule_flags": args.flags,
                   "virtual_ranks": N * G * Q, "buffers": P, "elements_per_rank": n, "launches_per_allreduce": len(info),
                   "unroll": la.la_tuning_get("unroll"), "cache_policy": la.la_tuning_get("cache_policy"),
                   "skew_bytes": args.skew, "flush_cache_between_allreduces": bool(args.flush_cache),
                   "steps_with_per_launch_events": len(range(0, args.steps, 1 if args.flush_cache else INSTRUMENT_EVERY))},
        "pct_of_hbm_peak": round(total_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS * 100, 2),
        "algorithmic_bytes_per_allreduce": total_bytes,
        "allreduce_bytes_per_s_per_rank": round(n * e / (ms * 1e-3), 1),
        "bus_bandwidth_bytes_per_s": round(n * e / (ms * 1e-3) * 2 * (P - 1) / P, 1),
        "ms_per_step_single_call_no_events": round(ms_onecall, 5),
        "kernels": kernels,
        "roofline": {"bound": "hbm", "achieved": round(dom_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(dom_gbs / HBM_PEAK_GBS, 4),
                     "traffic": MEASURED_TRAFFIC.get((args.config, algo, args.flags, dom_key[0])),
                     "kernel": f"seg_reduce_kernel, stage {dom_key[0]} (k={dom_key[1]}, m={dom_key[2]})",
                     "bytes_per_launch": dom["bytes"] // dom["launches"],
                     "avg_launch_ms": round(dom["ms"] / dom["launches"], 5)},
    }

    if args.config == "c2" and algo == "lane" and not args.no_ring:
        # the comparison the workload names: the flat ring over the same 16 ranks
        ring = la.la_schedule_build(topo, "ring", n, cfg["dtype"], args.flags)
        rbytes = sum(s["bytes_read"] + s["bytes_written"] for s in ring.steps())
        rk = max(3, args.steps // 4)
        rms, rsteps, _ = time_schedule(la, torch, ring, bufs, rk, 1)
        out["ring_comparison"] = {"ms_per_allreduce": round(rms, 5), "launches": ring.num_steps, "steps_timed": rk,
                                  "GBps": round(rbytes / (rms * 1e-3) / 1e9, 1),
                                  "allreduce_bytes_per_s_per_rank": round(n * e / (rms * 1e-3), 1),
                                  "lane_speedup_over_ring": round(rms / ms, 3)}
    if not args.no_ring:
        out["achievable"] = plain_copy_ceiling(torch, dom_gbs)
    if algo in ("lane", "lane_multiproc") and (args.flags & ~la.LA_SCHED_SHARED_BUFFERS) == 0 and not args.no_ring:
        # the same all-reduce with both all-gathers folded into the last reduce's store
        fz = la.la_schedule_build(topo, algo, n, cfg["dtype"], args.flags | la.LA_SCHED_FUSED_GATHER)
        fbytes = sum(s["bytes_read"] + s["bytes_written"] for s in fz.steps())
        fk = max(3, args.steps // 2)
        fms, _, _ = time_schedule(la, torch, fz, bufs, fk, 1)
        out["fused_gather_variant"] = {"ms_per_allreduce": round(fms, 5), "launches": fz.num_steps, "steps_timed": fk,
                                       "algorithmic_bytes": fbytes, "GBps": round(fbytes / (fms * 1e-3) / 1e9, 1),
                                       "allreduce_bytes_per_s_per_rank": round(n * e / (fms * 1e-3), 1)}
        # and the whole of Algorithm 2 as one two-level reduce launch
        one = la.la_schedule_build(topo, algo, n, cfg["dtype"], args.flags | la.LA_SCHED_SINGLE_LAUNCH)
        obytes = sum(s["bytes_read"] + s["bytes_written"] for s in one.steps())
        oms, _, _ = time_schedule(la, torch, one, bufs, fk, 1)
        out["single_launch_variant"] = {"ms_per_allreduce": round(oms, 5), "launches": one.num_steps, "steps_timed": fk,
                                        "algorithmic_bytes": obytes, "GBps": round(obytes / (oms * 1e-3) / 1e9, 1),
                                        "allreduce_bytes_per_s_per_rank": round(n * e / (oms * 1e-3), 1)}
    del bufs, slab
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, algo, total_bytes, shared)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
