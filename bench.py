#!/usr/bin/env python3
"""Benchmark of the emulated lane-aware all-reduce on one MI355X.

One "step" is one whole all-reduce (every launch of the schedule) over P resident rank buffers.
The headline workload is the largest fp32 configuration (C5: 1024 virtual ranks, 4 GiB resident,
far beyond the 256 MB last-level cache, so its rates are DRAM rates).  Prints ONE JSON line:
whole-job HBM GB/s (algorithmic bytes of the schedule / time), the roofline of the dominant kernel
(median per-launch duration from HIP events recorded on the launch stream, over a second pass of
at least 20 instrumented all-reduces, warm and from a flushed cache), one record per other
configuration (C2 lane, C2 ring, C3, C4) with the same figures, ceilings measured with the
library's own kernels on plain streaming shapes, and the CPU oracle timed on the host cores
(one thread and all cores) as a reported baseline.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "seg_reduce_kernel_pmc_traffic.md")
INSTRUMENTED = 20      # all-reduces of the second, per-launch-instrumented pass (at least)

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
               name="C5: 32 nodes x 4 GPUs x 8 procs = 1024 ranks, lane_multiproc, fp32 SUM, 1 Mi elements (4 MiB) per rank, "
                    "4 GiB resident, uniform [-1,1)"),
    # the size the paper's 8-node runs are quoted on, in the shared-buffer model (one buffer per GPU,
    # 16 processes per GPU on slices of it): 32 buffers of 512 MiB
    "paper8": dict(topo=(8, 4, 16), algo="lane_multiproc", n=1 << 27, dist="uniform_pm1", dtype="float32", flags=8,
                   name="paper size: 8 nodes x 4 GPUs, 2^27 fp32 (512 MiB) per GPU buffer, 16 processes per GPU "
                        "sharing it (multi-lane approach; --algo ring = standard approach)"),
}
# the other configurations reported beside the headline: (record id, configuration, algorithm)
SIDE_CONFIGS = (("c2-lane", "c2", "lane"), ("c2-ring", "c2", "ring"), ("c3", "c3", "lane_multiproc"),
                ("c4", "c4", "lane_multiproc"))
DTYPE_TAG = {"float32": "f32", "int32": "i32", "bfloat16": "bf16 in, f32 accumulate"}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="c5", choices=sorted(CONFIGS))
    ap.add_argument("--algo", default=None, choices=["ring", "lane", "lane_multiproc"])
    ap.add_argument("--n", type=int, default=None, help="elements per rank buffer, instead of the configuration's")
    ap.add_argument("--flags", type=int, default=0, help="LA_SCHED_* bits: 1 = point-to-point gather, 2 = staged, ...")
    ap.add_argument("--unroll", type=int, default=None)
    ap.add_argument("--cache-policy", type=int, default=None)
    ap.add_argument("--block", type=int, default=None, help="lanes per workgroup for every step: 256 or 1024")
    ap.add_argument("--skew", type=int, default=0, help="extra bytes between consecutive rank buffers")
    ap.add_argument("--flush-cache", action="store_true",
                    help="the headline figures themselves are taken with a 1 GiB scratch buffer rewritten before "
                         "every all-reduce (ms_per_step then comes from the per-launch events); without it the "
                         "flushed figures are still reported beside the steady-state ones")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-configs", action="store_true", help="skip the records of the other configurations")
    ap.add_argument("--no-variants", "--no-ring", dest="no_variants", action="store_true",
                    help="skip the schedule variants and the ceilings timed beside the headline")
    ap.add_argument("--headline-only", action="store_true",
                    help="the headline workload alone: no other configurations, variants, ceilings or CPU baseline "
                         "(the command the rocprofv3 summaries are taken with)")
    return ap.parse_args()


def host_buffers_to_device(x, skew_bytes):
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


def device_buffers_drawn_on_the_gpu(torch, cfg, P):
    """The side configurations: the same shapes and distributions, drawn by torch's seeded device
    generator instead of the host recipe (the kernels are HBM-bound: values do not move the time)."""
    gen = torch.Generator(device="cuda")
    gen.manual_seed(250813397)
    n, dist = cfg["n"], cfg["dist"]
    bufs = []
    for _ in range(P):
        if dist == "normal":
            b = torch.empty(n, dtype=torch.float32, device="cuda").normal_(0.0, 1.0, generator=gen)
        elif dist == "normal_bf16":
            b = torch.empty(n, dtype=torch.float32, device="cuda").normal_(0.0, 0.1, generator=gen).to(torch.bfloat16)
        elif dist == "uniform_pm1":
            b = torch.empty(n, dtype=torch.float32, device="cuda").uniform_(-1.0, 1.0, generator=gen)
        else:
            raise ValueError(dist)
        bufs.append(b)
    return bufs


def launch_units(la, sched):
    """The launches of one all-reduce as the library makes them: one per step, except that a run of
    steps which the library fuses without being asked (the ring forms) is ONE launch.  Each unit:
    dict(first, count, stage_name, fan_in, fan_out, bytes (as executed), table_bytes (as the step
    tables count them: a fused launch takes a chunk that the same lane has just stored from its
    registers instead of loading it again))."""
    info = sched.steps()
    runs = {}
    if la.la_tuning_get("fuse") != 0:
        for r in range(la.la_schedule_fusion_runs(sched)):
            f = la.la_schedule_fusion_table(sched, r)
            if f["automatic"] or la.la_tuning_get("fuse") == 1:
                runs[f["first_step"]] = f
    units, i = [], 0
    while i < len(info):
        if i in runs:
            f = runs[i]
            part = info[i:i + f["num_steps"]]
            names = []
            for s in part:
                if s["stage_name"] not in names:
                    names.append(s["stage_name"])
            units.append(dict(first=i, count=f["num_steps"], stage_name="+".join(names) + f" (one fused launch of {f['num_steps']} steps)",
                              fan_in=max(s["fan_in"] for s in part), fan_out=max(s["fan_out"] for s in part),
                              bytes=f["bytes_read"] + f["bytes_written"],
                              table_bytes=sum(s["bytes_read"] + s["bytes_written"] for s in part), fused=True))
            i += f["num_steps"]
        else:
            s = info[i]
            b = s["bytes_read"] + s["bytes_written"]
            units.append(dict(first=i, count=1, stage_name=s["stage_name"], fan_in=s["fan_in"], fan_out=s["fan_out"], bytes=b,
                              table_bytes=b, fused=False))
            i += 1
    return units


def time_schedule(la, torch, sched, bufs, steps, warmup, flush=None, instrumented=INSTRUMENTED, one_call=True):
    """W warm-up all-reduces; K timed ones through la_allreduce_emulated, the entry point an
    application calls (wall clock around the region, synchronised on both sides); then a second pass
    of `instrumented` all-reduces issued launch by launch with an event recorded on the launch stream
    after every launch: the per-launch durations are medians over that pass.  (An event record costs
    the stream several microseconds, so the whole-job figure is never taken from the instrumented
    pass.)  With a flush buffer, that buffer (1 GiB) is rewritten before every all-reduce of the
    instrumented pass, and the whole-job time is the median over as many all-reduces issued through the one-call entry
    point, each after a flush, between two events.  Returns (ms per all-reduce, ms per launch unit, runs, units)."""
    stream = torch.cuda.current_stream()
    ptrs = la.ptr_array([b.data_ptr() for b in bufs])
    units = launch_units(la, sched)
    fused_before = la.la_tuning_get("fused_launches")
    for _ in range(warmup):
        la.la_allreduce_emulated(sched, ptrs, sched.n, sched.dtype, la.LA_SUM, stream.cuda_stream)
    if warmup and any(u["fused"] for u in units) and la.la_tuning_get("fused_launches") == fused_before:
        # the buffers did not allow the fused launch (addresses that disagree modulo 16 bytes): every step is a launch
        la.la_tuning_set("fuse", 0)
        units = launch_units(la, sched)
    wall_ms = None
    if one_call:
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            la.la_allreduce_emulated(sched, ptrs, sched.n, sched.dtype, la.LA_SUM, stream.cuda_stream)
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) / steps * 1e3
    runs = max(instrumented, 1)
    nu = len(units)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(nu + 1)] for _ in range(runs)]
    torch.cuda.synchronize()
    for k in range(runs):
        if flush is not None:
            flush.add_(1.0)
        ev[k][0].record(stream)
        for i, u in enumerate(units):
            la.la_schedule_run_steps(sched, u["first"], u["count"], ptrs, la.LA_SUM, stream.cuda_stream)
            ev[k][i + 1].record(stream)
    torch.cuda.synchronize()
    per_unit_ms = [statistics.median(ev[k][i].elapsed_time(ev[k][i + 1]) for k in range(runs)) for i in range(nu)]
    if flush is not None:
        # whole all-reduces from a flushed cache, through the one-call entry point: two events around each
        pair = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(runs)]
        for a, b in pair:
            flush.add_(1.0)
            a.record(stream)
            la.la_allreduce_emulated(sched, ptrs, sched.n, sched.dtype, la.LA_SUM, stream.cuda_stream)
            b.record(stream)
        torch.cuda.synchronize()
        wall_ms = statistics.median(a.elapsed_time(b) for a, b in pair)
    return wall_ms, per_unit_ms, runs, units


def families(units, per_unit_ms):
    """Launches of one shape (stage, fan-in, fan-out) are one kernel family."""
    fam = {}
    for u, ms in zip(units, per_unit_ms):
        key = (u["stage_name"], u["fan_in"], u["fan_out"])
        f = fam.setdefault(key, {"ms": 0.0, "bytes": 0, "launches": 0})
        f["ms"] += ms
        f["bytes"] += u["bytes"]
        f["launches"] += 1
    return fam


def gbps(nbytes, ms):
    return nbytes / (ms * 1e-3) / 1e9


def kernel_records(fam, fam_cold=None):
    out = []
    for k, v in fam.items():
        rec = {"stage": k[0], "fan_in": k[1], "fan_out": k[2], "launches": v["launches"],
               "bytes_per_launch": v["bytes"] // v["launches"], "median_ms": round(v["ms"] / v["launches"], 5),
               "GBps": round(gbps(v["bytes"], v["ms"]), 1), "frac_of_peak": round(gbps(v["bytes"], v["ms"]) / HBM_PEAK_GBS, 4)}
        if fam_cold is not None:
            c = fam_cold[k]
            rec["median_ms_cold"] = round(c["ms"] / c["launches"], 5)
            rec["frac_of_peak_cold"] = round(gbps(c["bytes"], c["ms"]) / HBM_PEAK_GBS, 4)
        out.append(rec)
    return out


def recorded_traffic(config_id, algo, stage):
    """HBM-side bytes per launch of a step as recorded by the committed rocprofv3 --pmc runs
    (FETCH_SIZE and WRITE_SIZE, each scaled by what the same counter reads for a plain copy of known
    size): a row `| config | algo | stage | ... | traffic bytes |` of the summary file.  Not measured
    in this run; None when the file has no such row."""
    try:
        with open(TRAFFIC_FILE) as f:
            for line in f:
                cells = [c.strip() for c in line.strip().strip("|").split("|")]
                if len(cells) >= 4 and cells[0] == config_id and cells[1] == algo and cells[2] == stage:
                    return int(re.sub(r"[^0-9]", "", cells[-1]))
    except (OSError, ValueError):
        pass
    return None


def measure_config(la, torch, cfg, algo, flags, bufs, steps, warmup, flush):
    """Steady-state and flushed-cache figures of one schedule on resident buffers."""
    N, G, Q = cfg["topo"]
    topo = la.la_topology_create(N, G, Q)
    sched = la.la_schedule_build(topo, algo, cfg["n"], cfg["dtype"], flags)
    info = sched.steps()
    fuse_knob = la.la_tuning_get("fuse")
    try:
        wall_ms, per_ms, runs, units = time_schedule(la, torch, sched, bufs, steps, warmup)
        cold_wall_ms, cold_ms, _, _ = time_schedule(la, torch, sched, bufs, 0, 1, flush=flush, one_call=False)
    finally:
        la.la_tuning_set("fuse", fuse_knob)
    total = sum(u["bytes"] for u in units)              # as executed
    table_total = sum(u["table_bytes"] for u in units)  # as the step tables count them
    fam, fam_cold = families(units, per_ms), families(units, cold_ms)
    dom = max(fam, key=lambda k: fam[k]["ms"])
    return dict(sched=sched, info=info, units=units, total=total, table_total=table_total, wall_ms=wall_ms, per_ms=per_ms,
                cold_ms=cold_ms, cold_wall_ms=cold_wall_ms, fam=fam, fam_cold=fam_cold, dom=dom, runs=runs)


def side_record(rid, cfg, algo, m, e):
    n, P = cfg["n"], len(m["bufs"])
    fam, cold, dom = m["fam"], m["fam_cold"], m["dom"]
    cold_total = m["cold_wall_ms"]
    return {"id": rid, "workload": cfg["name"], "algo": algo, "dtype": DTYPE_TAG[cfg["dtype"]],
            "steps_per_allreduce": len(m["info"]), "launches_per_allreduce": len(m["units"]),
            "algorithmic_bytes_per_allreduce": m["total"], "step_table_bytes_per_allreduce": m["table_total"],
            "ms_per_allreduce": round(m["wall_ms"], 5), "GBps": round(gbps(m["total"], m["wall_ms"]), 1),
            "frac_of_peak": round(gbps(m["total"], m["wall_ms"]) / HBM_PEAK_GBS, 4),
            "ms_per_allreduce_cold": round(cold_total, 5), "GBps_cold": round(gbps(m["total"], cold_total), 1),
            "frac_cold": round(gbps(m["total"], cold_total) / HBM_PEAK_GBS, 4),
            "allreduce_bytes_per_s_per_rank": round(n * e / (m["wall_ms"] * 1e-3), 1),
            "dominant_kernel": {"stage": dom[0], "fan_in": dom[1], "fan_out": dom[2],
                                "GBps": round(gbps(fam[dom]["bytes"], fam[dom]["ms"]), 1),
                                "frac": round(gbps(fam[dom]["bytes"], fam[dom]["ms"]) / HBM_PEAK_GBS, 4),
                                "frac_cold": round(gbps(cold[dom]["bytes"], cold[dom]["ms"]) / HBM_PEAK_GBS, 4),
                                "traffic": recorded_traffic(rid.split("-")[0], algo, dom[0])},
            "kernels": kernel_records(fam, cold),
            "launches_timed_per_kernel": m["runs"],
            "note": ("1 GiB resident: in the steady-state loop part of the reads is served by the 256 MB last-level "
                     "cache; frac_cold is the DRAM-rate figure" if rid.startswith("c2") else
                     "2 to 4 GiB resident: DRAM rates in both columns")}


def ceilings(la, torch, dom_gbs):
    """What plain streaming shapes reach with the library's own kernel on a 4 GiB working set
    (nothing cache-resident), measured here: a stream copy (one source, one destination: the copy
    step of an out-of-place schedule over one rank), a two-operand in-place add (la_reduce_segments
    with one source: 2 reads + 1 write per element, the shape of STREAM's add / triad), and an
    eight-operand in-place reduce (8 reads + 1 write).  Medians of 10 event-timed launches."""
    stream = torch.cuda.current_stream()
    n = 1 << 29  # 2 GiB of fp32 per buffer
    out = {}

    def timed(fn, nbytes):
        for _ in range(2):
            fn()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(11)]
        torch.cuda.synchronize()
        ev[0].record(stream)
        for i in range(10):
            fn()
            ev[i + 1].record(stream)
        torch.cuda.synchronize()
        return round(gbps(nbytes, statistics.median(ev[i].elapsed_time(ev[i + 1]) for i in range(10))), 1)

    a = torch.empty(n, dtype=torch.float32, device="cuda").uniform_(-1, 1)
    b = torch.empty(n, dtype=torch.float32, device="cuda").uniform_(-1, 1)
    one = la.la_schedule_build(la.la_topology_create(1, 1, 1), "lane", n, "float32", la.LA_SCHED_OUT_OF_PLACE)
    send, recv = la.ptr_array([a.data_ptr()]), la.ptr_array([b.data_ptr()])
    out["stream_copy_GBps"] = timed(lambda: la.la_allreduce_emulated_out_of_place(
        one, send, recv, n, "float32", la.LA_SUM, stream.cuda_stream), 2 * n * 4)
    out["add_2_operands_in_place_GBps"] = timed(lambda: la.la_reduce_segments(
        b.data_ptr(), [a.data_ptr()], [0], n, "float32", la.LA_SUM, stream.cuda_stream), 3 * n * 4)
    del a, b, one
    torch.cuda.empty_cache()
    m = 1 << 26  # 9 buffers of 256 MiB... the reduce reads 8 and writes 1: 2.25 GiB per launch; two sets alternate
    sets = [[torch.empty(m, dtype=torch.float32, device="cuda").uniform_(-1, 1) for _ in range(8)] for _ in range(2)]
    state = {"i": 0}

    def reduce8():
        s = sets[state["i"] & 1]
        state["i"] += 1
        la.la_reduce_segments(s[0].data_ptr(), [t.data_ptr() for t in s[1:]], [0], m, "float32", la.LA_SUM, stream.cuda_stream)

    out["reduce_8_operands_in_place_GBps"] = timed(reduce8, 9 * m * 4)
    del sets
    torch.cuda.empty_cache()
    m32 = 1 << 25  # 32 buffers of 128 MiB: 4 GiB; 32 reads + 1 write per element, the dominant kernel's mix
    wide = [torch.empty(m32, dtype=torch.float32, device="cuda").uniform_(-1, 1) for _ in range(32)]
    out["reduce_32_operands_in_place_GBps"] = timed(lambda: la.la_reduce_segments(
        wide[0].data_ptr(), [t.data_ptr() for t in wide[1:]], [0], m32, "float32", la.LA_SUM, stream.cuda_stream), 33 * m32 * 4)
    del wide
    torch.cuda.empty_cache()
    out["what"] = ("the library's own kernel on plain shapes, 4 GiB working sets, medians of 10 launches: stream copy "
                   "(2 GiB -> 2 GiB), b += a (2 reads + 1 write per element), 8-operand in-place reduce over two "
                   "alternating sets of 2 GiB, 32-operand in-place reduce over 4 GiB (one contiguous segment, the read / write "
                   "mix of C5's S1)")
    best = max(v for k, v in out.items() if k.endswith("GBps"))
    out["dominant_kernel_over_best_ceiling"] = round(dom_gbs / best, 3)
    out["best_ceiling_frac_of_peak"] = round(best / HBM_PEAK_GBS, 4)
    return out


def cpu_baseline(cfg, algo, total_bytes_full, shared=False, budget_s=12.0):
    """The oracle as it stands on the host cores, on a bounded sample of the workload: one thread,
    then all the cores the box gives (at most 16).  The sample is the same topology with fewer
    elements per rank, sized so that each leg takes a few seconds."""
    import oracle
    from paper_2508_13397_amd import synth

    N, G, Q = cfg["topo"]
    P = N * G if shared else N * G * Q
    n = cfg["n"]
    cores = min(oracle.max_threads(), os.cpu_count() or 1, 16)

    def leg(threads, sample_n):
        oracle.set_threads(threads)
        x = synth.make_inputs(P, sample_n, cfg["dist"])
        t0 = time.perf_counter()
        oracle.allreduce(algo, N, G, Q, x, in_place=True, shared=shared)
        return time.perf_counter() - t0

    # a probe on 1/64 of the workload sizes both samples
    probe_n = max(n // 64, 1024)
    t_probe_1 = leg(1, probe_n)
    per_elem_1 = t_probe_1 / probe_n
    n1 = int(min(n, max(probe_n, budget_s / per_elem_1)))
    t1 = leg(1, n1)
    t_probe_all = leg(cores, probe_n)
    n_all = int(min(n, max(probe_n, budget_s / (t_probe_all / probe_n))))
    t_all = leg(cores, n_all)
    g1 = total_bytes_full * (n1 / n) / t1 / 1e9
    g_all = total_bytes_full * (n_all / n) / t_all / 1e9
    return {"value": round(g_all, 3), "unit": "GB/s", "cores": cores, "kind": "oracle",
            "sample": f"{algo} schedule, same topology, {n_all} of {n} elements per rank on {cores} threads in {t_all:.2f} s; "
                      f"GB/s = algorithmic bytes of the GPU schedule for that sample / time",
            "seconds": round(t_all, 3),
            "single_thread": {"value": round(g1, 3), "unit": "GB/s", "cores": 1, "seconds": round(t1, 3),
                              "sample": f"{n1} of {n} elements per rank on one thread"}}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU: the P virtual ranks all live in one MI355X's HBM; "
              f"--gpus {args.gpus} is not supported.", file=sys.stderr)
        sys.exit(2)
    import torch

    import paper_2508_13397_amd as la
    from paper_2508_13397_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    la.lib()
    torch.cuda.set_device(0)
    if args.headline_only:
        args.no_configs = args.no_variants = args.no_cpu_baseline = True
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
    flush = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")

    # ---- the headline workload, on buffers drawn by the seeded host recipe
    x = synth.make_inputs(P, n, cfg["dist"], workers=16)
    bufs, slab = host_buffers_to_device(x, args.skew)
    del x
    m = measure_config(la, torch, cfg, algo, args.flags, bufs, args.steps, args.warmup, flush)
    sched, info, total_bytes = m["sched"], m["info"], m["total"]
    fam, fam_cold, dom_key = m["fam"], m["fam_cold"], m["dom"]
    ms = m["cold_wall_ms"] if args.flush_cache else m["wall_ms"]
    dom = fam_cold[dom_key] if args.flush_cache else fam[dom_key]
    dom_gbs = gbps(dom["bytes"], dom["ms"])
    dom_cold_gbs = gbps(fam_cold[dom_key]["bytes"], fam_cold[dom_key]["ms"])
    ptr_list = [b.data_ptr() for b in bufs]
    launch_segments = [la.la_schedule_launch_segments(sched, i, ptr_list)["count"] for i in range(len(info))] \
        if sched.staging_elems == 0 else [None] * len(info)

    out = {
        "metric": "segmented-reduce HBM GB/s (% of peak) + emulated allreduce bytes/s per virtual rank",
        "value": round(gbps(total_bytes, ms), 2),
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
                   "virtual_ranks": N * G * Q, "buffers": P, "elements_per_rank": n, "steps_per_allreduce": len(info),
                   "launches_per_allreduce": len(m["units"]),
                   "unroll": la.la_tuning_get("unroll"), "cache_policy": la.la_tuning_get("cache_policy"),
                   "skew_bytes": args.skew, "flush_cache_between_allreduces": bool(args.flush_cache),
                   "instrumented_allreduces": m["runs"]},
        "pct_of_hbm_peak": round(gbps(total_bytes, ms) / HBM_PEAK_GBS * 100, 2),
        "pct_of_hbm_peak_cold": round(gbps(total_bytes, m["cold_wall_ms"]) / HBM_PEAK_GBS * 100, 2),
        "ms_per_step_cold": round(m["cold_wall_ms"], 5),
        "algorithmic_bytes_per_allreduce": total_bytes,
        "step_table_bytes_per_allreduce": m["table_total"],
        "allreduce_bytes_per_s_per_rank": round(n * e / (ms * 1e-3), 1),
        "bus_bandwidth_bytes_per_s": round(n * e / (ms * 1e-3) * 2 * (P - 1) / P, 1),
        "schedule_report": [{"step": i, "stage": s["stage_name"], "segments": s["num_segments"],
                             "launch_segments": launch_segments[i], "segment_elements_max": s["seg_len_max"],
                             "fan_in": s["fan_in"], "fan_out": s["fan_out"]} for i, s in enumerate(info)],
        "kernels": kernel_records(fam, fam_cold),
        "roofline": {"bound": "hbm", "achieved": round(dom_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(dom_gbs / HBM_PEAK_GBS, 4),
                     "traffic": recorded_traffic(args.config, algo, dom_key[0]) if args.flags == cfg.get("flags", 0) else None,
                     "traffic_source": "recorded: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs summarised in "
                                       "profiles/seg_reduce_kernel_pmc_traffic.md, not measured in this run",
                     "kernel": f"seg_reduce_kernel, stage {dom_key[0]} (k={dom_key[1]}, m={dom_key[2]})",
                     "bytes_per_launch": dom["bytes"] // dom["launches"],
                     "median_launch_ms": round(dom["ms"] / dom["launches"], 5),
                     "launches_timed": m["runs"] * dom["launches"],
                     "achieved_cold": round(dom_cold_gbs, 1), "frac_cold": round(dom_cold_gbs / HBM_PEAK_GBS, 4)},
    }

    if not args.no_variants and algo in ("lane", "lane_multiproc") and (args.flags & ~la.LA_SCHED_SHARED_BUFFERS) == 0:
        topo = la.la_topology_create(N, G, Q)
        for name, bit in (("fused_gather_variant", la.LA_SCHED_FUSED_GATHER), ("single_launch_variant", la.LA_SCHED_SINGLE_LAUNCH)):
            v = la.la_schedule_build(topo, algo, n, cfg["dtype"], args.flags | bit)
            vbytes = sum(s["bytes_read"] + s["bytes_written"] for s in v.steps())
            vms, _, _, _ = time_schedule(la, torch, v, bufs, max(3, args.steps // 2), 1, instrumented=1)
            out[name] = {"ms_per_allreduce": round(vms, 5), "launches": v.num_steps, "algorithmic_bytes": vbytes,
                         "GBps": round(gbps(vbytes, vms), 1), "allreduce_bytes_per_s_per_rank": round(n * e / (vms * 1e-3), 1)}
            del v
    del bufs, slab, sched, m
    torch.cuda.empty_cache()

    if not args.no_configs:
        records = []
        for rid, cid, salgo in SIDE_CONFIGS:
            if cid == args.config and salgo == algo:
                continue
            scfg = CONFIGS[cid]
            sN, sG, sQ = scfg["topo"]
            sbufs = device_buffers_drawn_on_the_gpu(torch, scfg, sN * sG * sQ)
            sm = measure_config(la, torch, scfg, salgo, 0, sbufs, args.steps, args.warmup, flush)
            sm["bufs"] = sbufs
            records.append(side_record(rid, scfg, salgo, sm, la.ELEM_SIZE[la.DTYPES[scfg["dtype"]]]))
            del sbufs, sm
            torch.cuda.empty_cache()
        out["configs"] = records
    if not args.no_variants:
        out["achievable"] = ceilings(la, torch, dom_gbs)
    del flush
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, algo, total_bytes, shared)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
