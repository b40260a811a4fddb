"""Host logic that decides how a step is launched (no GPU): la_schedule_launch_plan against the
rules it documents, on addresses that are never dereferenced.

What is checked is what a kernel launch relies on: enough workgroups for every segment under the
tiling the plan names, edge workgroups exactly when some segment has elements outside its whole
16-byte vectors, and the launch shapes of the five benchmark configurations (the ones the committed
rocprofv3 summaries name)."""
import numpy as np
import pytest

import paper_2508_13397_amd as la

BASE = 0x7F0000000000  # a 2 MiB aligned fake device address
EDGE_LANES = 128
ALIGN_MIN_TILES = 8
SMALL_SCHEDULE_BYTES = 96 << 20
ESIZE = {"int32": 4, "float32": 4, "bfloat16": 2, "float16": 2, "float64": 8}


def fake_buffers(count, n, esize, shift_elems=0, skew=None):
    stride = ((n + 65536) * esize + (1 << 21) - 1) >> 21 << 21
    return [BASE + r * stride + (shift_elems if skew is None else skew[r]) * esize for r in range(count)]


def segment_geometry(launch, esize):
    """Per launch segment: (whole vectors, head + tail elements, address of the first whole vector
    in destination 0 or None when the operands disagree modulo 16 bytes)."""
    vec = 16 // esize
    out = []
    for g in range(launch["count"]):
        addrs = [int(a) for a in launch["src_addr"][g]]
        dsts = [int(a) for a in launch["dst_addr"][g]]
        ln = int(launch["seg_len"][g])
        every = addrs + dsts
        if any((a ^ every[0]) & 15 for a in every):
            out.append((ln // vec, ln % vec, None))
            continue
        align = 16 if any((a ^ every[0]) & 127 for a in every) else 128
        head = min(((align - every[0] % align) % align) // esize, ln)
        body = ln - head
        out.append((body // vec, head + body % vec, dsts[0] + head * esize))
    return out


def check_merge(sched, step, bufs, esize, launch):
    """The launch segments are runs of consecutive table segments: every source list continues the
    previous one's, the destination sets do too, and a run ends exactly where that stops."""
    tab = sched.step_table(step)
    k, m = tab["fan_in"], tab["fan_out"]
    runs, cur = [], None
    for g in range(tab["num_segments"]):
        src = [bufs[b] + int(o) * esize for b, o in zip(tab["src_buf"][g], tab["src_off"][g])]
        dst = [bufs[b] + int(o) * esize for b, o in zip(tab["dst_buf"][g], tab["dst_off"][g])]
        ln = int(tab["seg_len"][g])
        if cur is not None:
            shift = cur["len"] * esize
            if src == [a + shift for a in cur["src"]] and sorted(dst) == sorted(a + shift for a in cur["dst"]):
                cur["len"] += ln
                continue
        cur = dict(src=src, dst=dst, len=ln)
        runs.append(cur)
    assert launch["count"] == len(runs), (step, launch["count"], len(runs))
    for g, r in enumerate(runs):
        assert int(launch["seg_len"][g]) == r["len"]
        assert [int(a) for a in launch["src_addr"][g]] == r["src"]
        assert [int(a) for a in launch["dst_addr"][g]] == r["dst"]  # the first segment's order is kept
    assert sum(int(x) for x in launch["seg_len"]) == sum(int(x) for x in tab["seg_len"])
    assert (k, m) == (launch["src_addr"].shape[1], launch["dst_addr"].shape[1])


def check_plan(sched, bufs, esize, sendbufs=None):
    for step in range(sched.num_steps):
        plan = la.la_schedule_launch_plan(sched, step, bufs, sendbufs=sendbufs)
        launch = la.la_schedule_launch_segments(sched, step, bufs, sendbufs=sendbufs)
        if sendbufs is None and sched.staging_elems == 0:
            check_merge(sched, step, bufs, esize, launch)
        S = launch["count"]
        tile = plan["block"] * plan["unroll"]
        assert plan["block"] in (256, 1024) and plan["unroll"] in (1, 2, 4, 8) and 0 <= plan["cache_policy"] <= 7
        assert plan["unroll"] < 8 or plan["block"] == 1024
        geo = segment_geometry(launch, esize)
        longest = max(max(nvec, 1 if edge and first is None else 0) for nvec, edge, first in geo)
        need, leads = 1, []
        for nvec, edge, first in geo:
            lead = 0
            if plan["tiling"] == 1 and first is not None:
                lead = (first % (tile * 16)) // 16
                leads.append(lead)
            need = max(need, -(-(lead + nvec) // tile))
        assert plan["tiles_per_segment"] == need, (step, plan, need)
        if plan["tiling"] == 1:
            assert longest >= ALIGN_MIN_TILES * tile and any(leads), (step, plan)
        elif plan["tiling"] == 2:
            assert longest < ALIGN_MIN_TILES * tile, (step, plan)
        else:
            assert plan["tiling"] == 0 and longest >= ALIGN_MIN_TILES * tile, (step, plan)
            assert all(first is None or first % (tile * 16) == 0 for nvec, edge, first in geo), (step, plan)
        any_edge = any(edge for nvec, edge, first in geo)
        per_block = plan["block"] // EDGE_LANES
        assert plan["edge_workgroups"] == (-(-S // per_block) if any_edge else 0), (step, plan)
        assert plan["workgroups"] == plan["edge_workgroups"] + S * plan["tiles_per_segment"]
        assert all(edge < EDGE_LANES for nvec, edge, first in geo)


@pytest.mark.parametrize("cfg,expect", [
    (((2, 4, 1), "lane", 1 << 16, "float32"), [(256, 1, 6), (256, 1, 7), (256, 1, 4)]),  # small: one workgroup size for all steps
    (((4, 4, 1), "lane", 1 << 24, "float32"), [(1024, 8, 6), (1024, 1, 7), (256, 1, 4)]),  # S1 streams 1 GiB of inputs
    (((8, 4, 4), "lane_multiproc", 1 << 22, "float32"), [(1024, 4, 6), (256, 4, 7), (1024, 8, 4)]),
    (((2, 4, 2), "lane_multiproc", 1 << 27, "bfloat16"), [(1024, 8, 3), (1024, 1, 7), (1024, 8, 7)]),
    (((32, 4, 8), "lane_multiproc", 1 << 20, "float32"), [(1024, 4, 6), (256, 4, 7), (1024, 8, 4)]),  # S2: 32 merged segments of 128 KiB
])
def test_launch_shapes_of_the_benchmark_configurations(cfg, expect):
    topo, algo, n, dtype = cfg
    sched = la.la_schedule_build(la.la_topology_create(*topo), algo, n, dtype)
    bufs = fake_buffers(sched.num_buffers, n, ESIZE[dtype])
    check_plan(sched, bufs, ESIZE[dtype])
    plans = [la.la_schedule_launch_plan(sched, i, bufs) for i in range(sched.num_steps)]
    assert all(p["edge_workgroups"] == 0 for p in plans)  # whole tensors of a power-of-two length
    if expect is not None:
        assert [(p["block"], p["unroll"], p["cache_policy"]) for p in plans] == expect


def test_plans_for_random_lengths_offsets_and_flags():
    rng = np.random.default_rng(7)
    topos = [(2, 2, 1), (2, 2, 2), (1, 3, 1), (3, 1, 2), (4, 4, 1), (8, 4, 4), (1, 1, 1), (2, 4, 2)]
    algos = ["ring", "lane", "lane_multiproc", "rabenseifner", "recursive_doubling"]
    flag_sets = [0, la.LA_SCHED_P2P_GATHER, la.LA_SCHED_INNER_RING, la.LA_SCHED_FUSED_GATHER, la.LA_SCHED_SINGLE_LAUNCH,
                 la.LA_SCHED_ONLY_REDUCE_SCATTER]
    seen = set()
    for case in range(160):
        topo = topos[int(rng.integers(len(topos)))]
        algo = algos[int(rng.integers(len(algos)))]
        flags = flag_sets[int(rng.integers(len(flag_sets)))]
        if algo in ("ring", "rabenseifner", "recursive_doubling"):
            flags &= la.LA_SCHED_ONLY_REDUCE_SCATTER if algo != "recursive_doubling" else 0
        if algo in ("rabenseifner", "recursive_doubling") and (topo[0] * topo[1] * topo[2]) & (topo[0] * topo[1] * topo[2] - 1):
            algo = "ring"  # those two need a power-of-two number of ranks
            flags = 0
        dtype = ["float32", "bfloat16", "float64", "int32"][int(rng.integers(4))]
        n = int(rng.integers(1, 40)) if case % 8 == 0 else int(2 ** rng.uniform(8, 25))
        e = ESIZE[dtype]
        sched = la.la_schedule_build(la.la_topology_create(*topo), algo, n, dtype, flags)
        P = sched.num_buffers
        kind = case % 4
        if kind == 0:
            bufs = fake_buffers(P, n, e)
        elif kind == 1:
            bufs = fake_buffers(P, n, e, shift_elems=int(rng.integers(0, 50000)))
        elif kind == 2:
            bufs = fake_buffers(P, n, e, shift_elems=int(rng.integers(0, 64)) * 1024)
        else:  # every buffer at its own odd offset: operands disagree modulo 16 bytes
            bufs = fake_buffers(P, n, e, skew=[int(x) for x in rng.integers(0, 9, size=P)])
        check_plan(sched, bufs, e)
        plans = [la.la_schedule_launch_plan(sched, i, bufs) for i in range(sched.num_steps)]
        seen.update(p["tiling"] for p in plans)
        if P * n * e <= SMALL_SCHEDULE_BYTES:  # one workgroup size for every step of a small schedule
            assert all(p["block"] == 256 for p in plans), (case, plans)
    assert seen == {0, 1, 2}


def test_plan_follows_the_tuning_knobs_and_rejects_bad_arguments():
    sched = la.la_schedule_build(la.la_topology_create(2, 2, 1), "lane", 3000001, "float32")
    bufs = fake_buffers(4, 3000001, 4)
    try:
        la.la_tuning_set("block", 256)
        la.la_tuning_set("unroll", 2)
        la.la_tuning_set("cache_policy", 5)
        for i in range(sched.num_steps):
            p = la.la_schedule_launch_plan(sched, i, bufs)
            assert (p["block"], p["unroll"], p["cache_policy"]) == (256, 2, 5)
        check_plan(sched, bufs, 4)
    finally:
        la.la_tuning_set("block", 0)
        la.la_tuning_set("unroll", 0)
        la.la_tuning_set("cache_policy", -1)
    with pytest.raises(la.LaError):
        la.la_schedule_launch_plan(sched, sched.num_steps, bufs)
    with pytest.raises(la.LaError):
        la.la_schedule_launch_plan(sched, 0, [bufs[0]] * 4)  # one pointer passed four times
    with pytest.raises(la.LaError):
        la.la_schedule_launch_plan(sched, 0, [b + 2 for b in bufs])  # not aligned to the element size
    staged = la.la_schedule_build(la.la_topology_create(2, 2, 1), "lane", 4096, "float32", la.LA_SCHED_STAGED)
    with pytest.raises(la.LaError):
        la.la_schedule_launch_plan(staged, 0, fake_buffers(4, 4096, 4))  # no staging address
    assert la.la_schedule_launch_plan(staged, 0, fake_buffers(4, 4096, 4), staging=BASE - (1 << 30))["workgroups"] > 0


def test_plan_of_an_out_of_place_schedule_needs_both_buffer_sets():
    n = 700001
    sched = la.la_schedule_build(la.la_topology_create(2, 2, 2), "lane_multiproc", n, "bfloat16", la.LA_SCHED_OUT_OF_PLACE)
    recv = fake_buffers(8, n, 2)
    send = [a + (1 << 36) + 6 for a in recv]  # another region, at an odd element offset
    with pytest.raises(la.LaError):
        la.la_schedule_launch_plan(sched, 0, recv)
    plans = [la.la_schedule_launch_plan(sched, i, recv, sendbufs=send) for i in range(sched.num_steps)]
    assert all(p["workgroups"] > 0 for p in plans)
    # the first step reads the send buffers, whose addresses disagree with the receive buffers modulo 16 bytes:
    # no common vector phase, so the elements that do not fill a vector go to edge workgroups
    assert plans[0]["edge_workgroups"] > 0
    in_place = la.la_schedule_build(la.la_topology_create(2, 2, 2), "lane_multiproc", n, "bfloat16")
    with pytest.raises(la.LaError):
        la.la_schedule_launch_plan(in_place, 0, recv, sendbufs=send)


def test_pieces_of_a_part_are_launched_as_one_segment():
    """The inter-node step of config 5 has 1024 table segments (32 parts x 32 pieces of 4 KiB, fan-in
    and fan-out 32); the pieces of a part read the same 32 buffers back to back and store to the same 32
    buffers, so the launch has 32 segments of 128 KiB.  With fused all-gathers likewise (fan-out 1024),
    and the one-launch form is a single segment: every table segment has the same 1024 sources and
    destinations.  The logical tables are unchanged, and the knob restores one launch segment per table segment."""
    topo, n = (32, 4, 8), 1 << 20
    for flags, step, table_segments, launch_segments in ((0, 1, 1024, 32), (la.LA_SCHED_FUSED_GATHER, 1, 1024, 32),
                                                         (la.LA_SCHED_SINGLE_LAUNCH, 0, 1024, 1), (0, 0, 1024, 1024),
                                                         (0, 2, 1024, 1024)):
        sched = la.la_schedule_build(la.la_topology_create(*topo), "lane_multiproc", n, "float32", flags)
        bufs = fake_buffers(sched.num_buffers, n, 4)
        assert sched.step_info(step)["num_segments"] == table_segments
        launch = la.la_schedule_launch_segments(sched, step, bufs)
        assert launch["count"] == launch_segments, (flags, step, launch["count"])
        check_merge(sched, step, bufs, 4, launch)
        try:
            la.la_tuning_set("merge", 0)
            assert la.la_schedule_launch_segments(sched, step, bufs)["count"] == table_segments
        finally:
            la.la_tuning_set("merge", 1)
    # buffers that do not follow each other's layout (every rank at its own odd offset) merge all the same:
    # the condition is on the addresses of consecutive table segments, which move together
    sched = la.la_schedule_build(la.la_topology_create(3, 2, 2), "lane_multiproc", 100003, "int32")
    bufs = fake_buffers(sched.num_buffers, 100003, 4, skew=[r % 5 for r in range(12)])
    for step in range(sched.num_steps):
        check_merge(sched, step, bufs, 4, la.la_schedule_launch_segments(sched, step, bufs))
    assert la.la_schedule_launch_segments(sched, 1, bufs)["count"] == 4  # 4 parts x 3 pieces
