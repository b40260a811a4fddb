"""The column analysis behind the one-launch execution of runs of steps (no GPU).

A run is a maximal sequence of consecutive steps with at most two sources and destinations per
segment.  la_schedule_fusion_table cuts the element axis into chains that never exchange data and
lists, per chain, the (step, segment) pairs of the run that cover it.  A numpy interpreter executes
the schedule with every run done chain by chain, in REVERSE chain order and each chain start to end
before the next begins, which is only correct if the chains are in fact independent and their
operations complete and ordered (the steps outside runs are executed table by table); the result
must equal the CPU oracle bit for bit.  It also checks what the kernel relies on: chains tile the
elements the run touches without overlap, every operation covers its chain entirely, operations of
a chain follow step order, a source marked as loadable ahead of time has not been written by an
earlier operation of its chain, and a source marked as forwarded is what the previous operation of
the chain stored."""
import itertools

import numpy as np
import pytest

import paper_2508_13397_amd as la
from paper_2508_13397_amd import synth
from test_schedule_tables import oracle_name, sum_in_order


def inputs_for(kind, B, n):
    if kind == "i32":
        return np.random.default_rng(n).integers(-(1 << 31), 1 << 31, size=(B, n), dtype=np.int64).astype(np.int32), "int32"
    if kind == "f32":
        return synth.order_sensitive_f32(B, n), "float32"
    return synth.to_bf16_bits(synth.order_sensitive_f32(B, n) * np.float32(2.0 ** -20)), "bfloat16"


def run_one_step(t, state):
    old = [b.copy() for b in state]
    for g in range(t["num_segments"]):
        ln = int(t["seg_len"][g])
        ops = [old[int(b)][int(o):int(o) + ln] for b, o in zip(t["src_buf"][g], t["src_off"][g])]
        res = sum_in_order(ops, t["group"])
        for b, o in zip(t["dst_buf"][g], t["dst_off"][g]):
            state[int(b)][int(o):int(o) + ln] = res


def run_chains_of(sched, f, tables, state):
    """one run, chain by chain (modifies state in place)"""
    C = len(f["chain_lo"])
    covered = np.zeros(sched.n, dtype=np.int32)
    steps = range(f["first_step"], f["first_step"] + f["num_steps"])
    longest = 0
    for c in reversed(range(C)):
        lo, ln = int(f["chain_lo"][c]), int(f["chain_len"][c])
        assert ln > 0
        covered[lo:lo + ln] += 1
        written, last_step, last_dsts = set(), -1, None
        a, b = int(f["chain_first_op"][c]), int(f["chain_first_op"][c + 1])
        assert b > a
        longest = max(longest, b - a)
        for o in range(a, b):
            step, g = int(f["op_step"][o]), int(f["op_segment"][o])
            assert step in steps and step >= last_step  # step order (several segments of one step may cover a chain)
            last_step = step
            t = tables[step]
            assert t["fan_in"] <= 2 and t["fan_out"] <= 2
            seg_lo, seg_len = int(t["dst_off"][g][0]), int(t["seg_len"][g])
            assert all(int(x) == seg_lo for x in t["src_off"][g]) and all(int(x) == seg_lo for x in t["dst_off"][g])
            assert seg_lo <= lo and lo + ln <= seg_lo + seg_len  # the operation covers the whole chain
            srcs = [int(x) for x in t["src_buf"][g]]
            pf, fw = int(f["op_prefetch_source"][o]), int(f["op_forward_source"][o])
            if pf >= 0:
                assert srcs[pf] not in written
            for ti, sbuf in enumerate(srcs):
                if sbuf not in written:
                    assert 0 <= pf <= ti  # the first original input is the one marked
            if fw >= 0:
                assert last_dsts is not None and srcs[fw] in last_dsts
            elif last_dsts is not None:
                assert not any(sbuf in last_dsts for sbuf in srcs)
            ops = [state[sbuf][lo:lo + ln] for sbuf in srcs]
            res = sum_in_order(ops, None)
            last_dsts = [int(d) for d in t["dst_buf"][g]]
            for d in last_dsts:
                state[d][lo:lo + ln] = res
                written.add(d)
    # the chains tile what the run touches, exactly once
    touched = np.zeros(sched.n, dtype=bool)
    for i in steps:
        t = tables[i]
        for g in range(t["num_segments"]):
            o, ln = int(t["dst_off"][g][0]), int(t["seg_len"][g])
            touched[o:o + ln] = True
    assert np.array_equal(covered, touched.astype(np.int32))
    # every (step, segment) of the run appears, and is covered entirely by its chains
    per_seg = {}
    for c in range(C):
        for o in range(int(f["chain_first_op"][c]), int(f["chain_first_op"][c + 1])):
            key = (int(f["op_step"][o]), int(f["op_segment"][o]))
            per_seg[key] = per_seg.get(key, 0) + int(f["chain_len"][c])
    for i in steps:
        for g in range(tables[i]["num_segments"]):
            assert per_seg.get((i, g), 0) == int(tables[i]["seg_len"][g]), (i, g)
    assert f["automatic"] == (f["num_steps"] >= 4 and longest < 8 * f["num_steps"])


def run_chains(sched, state):
    """The whole schedule: runs chain by chain, the other steps table by table.  Returns the runs."""
    tables = [sched.step_table(i) for i in range(sched.num_steps)]
    runs = [la.la_schedule_fusion_table(sched, r) for r in range(la.la_schedule_fusion_runs(sched))]
    # runs are maximal, disjoint, in order, and hold exactly the steps with at most two sources and destinations
    narrow = [t["fan_in"] <= 2 and t["fan_out"] <= 2 and t["group"] == t["fan_in"]
              and int(t["src_buf"].max()) != sched.num_buffers and int(t["dst_buf"].max()) != sched.num_buffers for t in tables]
    expect, i = [], 0
    while i < len(tables):
        j = i
        while j < len(tables) and narrow[j]:
            j += 1
        if j - i >= 2:
            expect.append((i, j - i))
        i = max(j, i + 1)
    assert [(f["first_step"], f["num_steps"]) for f in runs] == expect
    start = {f["first_step"]: f for f in runs}
    i = 0
    while i < sched.num_steps:
        if i in start:
            run_chains_of(sched, start[i], tables, state)
            i += start[i]["num_steps"]
        else:
            run_one_step(tables[i], state)
            i += 1
    return runs


FLAGS = (0, la.LA_SCHED_P2P_GATHER, la.LA_SCHED_INNER_RING, la.LA_SCHED_FUSED_GATHER, la.LA_SCHED_INNER_RING | la.LA_SCHED_P2P_GATHER)


@pytest.mark.parametrize("algo", ["ring", "lane", "lane_multiproc"])
@pytest.mark.parametrize("flags", FLAGS)
def test_chains_reproduce_the_oracle_in_any_chain_order(oracle, algo, flags):
    if algo == "ring" and flags & la.LA_SCHED_FUSED_GATHER:
        pytest.skip("the ring has no all-gather to fuse")
    for (N, G, Q) in itertools.product((1, 2, 3), repeat=3):
        if N * G * Q == 1:
            continue
        topo = la.la_topology_create(N, G, Q)
        for n, kind in ((1, "i32"), (5, "f32"), (17, "bf16"), (36, "f32"), (40, "i32"), (97, "bf16")):
            x, dt = inputs_for(kind, N * G * Q, n)
            sched = la.la_schedule_build(topo, algo, n, dt, flags)
            if sched.num_steps == 0:
                continue
            state = [x[r].copy() for r in range(x.shape[0])]
            run_chains(sched, state)
            ref = oracle.allreduce(oracle_name(algo, flags), N, G, Q, x)
            assert np.array_equal(np.stack(state).view(np.uint8), ref.view(np.uint8)), (algo, flags, N, G, Q, n, kind)


@pytest.mark.parametrize("algo", ["recursive_doubling", "rabenseifner"])
def test_chains_of_the_small_message_algorithms(oracle, algo):
    for topo3 in ((2, 1, 1), (2, 2, 1), (2, 2, 2), (1, 4, 4)):
        P = topo3[0] * topo3[1] * topo3[2]
        for n, kind in ((1, "i32"), (13, "f32"), (64, "bf16"), (1001, "f32")):
            x, dt = inputs_for(kind, P, n)
            sched = la.la_schedule_build(la.la_topology_create(*topo3), algo, n, dt)
            state = [x[r].copy() for r in range(P)]
            run_chains(sched, state)
            ref = oracle.allreduce(algo, *topo3, x)
            assert np.array_equal(np.stack(state).view(np.uint8), ref.view(np.uint8)), (algo, topo3, n, kind)


def test_chains_of_shared_buffer_and_out_of_place_schedules(oracle):
    SH, OOP = la.LA_SCHED_SHARED_BUFFERS, la.LA_SCHED_OUT_OF_PLACE
    for algo, topo3, n in (("ring", (2, 2, 3), 50), ("lane_multiproc", (3, 2, 2), 77), ("lane", (2, 3, 2), 31)):
        N, G, Q = topo3
        B = N * G
        x, dt = inputs_for("f32", B, n)
        sched = la.la_schedule_build(la.la_topology_create(*topo3), algo, n, dt, SH)
        state = [x[b].copy() for b in range(B)]
        run_chains(sched, state)
        if algo == "lane":  # one process per GPU does the whole buffer
            ref = oracle.allreduce("lane_multiproc", N, G, 1, x, shared=True)
        else:
            ref = oracle.allreduce(algo, N, G, Q, x, shared=True)
        assert np.array_equal(np.stack(state).view(np.uint8), ref.view(np.uint8)), (algo, topo3)
    for algo, topo3, n in (("ring", (2, 2, 1), 23), ("lane_multiproc", (2, 2, 2), 100), ("lane", (1, 1, 1), 9)):
        N, G, Q = topo3
        P = N * G * Q
        x, dt = inputs_for("bf16", P, n)
        sched = la.la_schedule_build(la.la_topology_create(*topo3), algo, n, dt, OOP)
        junk = np.full(n, 0x5A5A, dtype=np.uint16)
        state = [junk.copy() for _ in range(P)] + [np.zeros(1, dtype=np.uint16)] + [x[r].copy() for r in range(P)]
        run_chains(sched, state)
        ref = oracle.allreduce(algo, N, G, Q, x)
        assert np.array_equal(np.stack(state[:P]).view(np.uint8), ref.view(np.uint8)), (algo, topo3)
        assert np.array_equal(np.stack(state[P + 1:]), x)  # the send buffers are never written


def test_chain_shapes():
    # Algorithm 1 over P ranks: one run of 2(P - 1) steps, one chain per chunk, 2(P - 1) operations each; the
    # reduce steps load the rank's own copy of the chunk ahead of time (an original input) and take the
    # incoming partial sum from registers; the gather copies pass on what the chain itself produced
    P, n = 8, 8 * 1000
    sched = la.la_schedule_build(la.la_topology_create(2, 2, 2), "ring", n, "float32")
    assert la.la_schedule_fusion_runs(sched) == 1
    f = la.la_schedule_fusion_table(sched, 0)
    assert (f["first_step"], f["num_steps"], f["automatic"]) == (0, 2 * (P - 1), True)
    assert len(f["chain_lo"]) == P and list(f["chain_len"]) == [1000] * P
    assert [int(b - a) for a, b in zip(f["chain_first_op"][:-1], f["chain_first_op"][1:])] == [2 * (P - 1)] * P
    for c in range(P):
        a = int(f["chain_first_op"][c])
        pf = [int(v) for v in f["op_prefetch_source"][a:a + 2 * (P - 1)]]
        fw = [int(v) for v in f["op_forward_source"][a:a + 2 * (P - 1)]]
        assert pf[:P - 1] == [0] * (P - 1) and pf[P - 1:] == [-1] * (P - 1)
        assert fw == [-1] + [1] * (P - 2) + [0] * (P - 1)
    # config 5 with the ring as the inter-node stage: S1, one run of 62 ring steps, S3
    sched = la.la_schedule_build(la.la_topology_create(32, 4, 8), "lane_multiproc", 1 << 20, "float32", la.LA_SCHED_INNER_RING)
    assert la.la_schedule_fusion_runs(sched) == 1
    f = la.la_schedule_fusion_table(sched, 0)
    assert (f["first_step"], f["num_steps"], f["automatic"]) == (1, 62, True)
    assert len(f["chain_lo"]) == 1024 and set(int(v) for v in f["chain_len"]) == {1024}
    assert set(int(b - a) for a, b in zip(f["chain_first_op"][:-1], f["chain_first_op"][1:])) == {62}
    # the default three-stage schedule of config 2 has no run (fan-in 4, fan-out 3 and 4) ...
    assert la.la_schedule_fusion_runs(la.la_schedule_build(la.la_topology_create(4, 4, 1), "lane", 1 << 24, "float32")) == 0
    # ... recursive doubling is one run whose chain (the whole buffer) sees every pair of every round: not automatic
    sched = la.la_schedule_build(la.la_topology_create(4, 4, 1), "recursive_doubling", 4096, "float32")
    f = la.la_schedule_fusion_table(sched, 0)
    assert (f["first_step"], f["num_steps"], f["automatic"]) == (0, 4, False) and len(f["chain_lo"]) == 1
    # Rabenseifner: one run of 2 log2 P steps, automatic
    sched = la.la_schedule_build(la.la_topology_create(4, 4, 1), "rabenseifner", 4096, "float32")
    f = la.la_schedule_fusion_table(sched, 0)
    assert (f["first_step"], f["num_steps"], f["automatic"]) == (0, 8, True) and len(f["chain_lo"]) == 16


def test_schedules_without_runs_and_bad_arguments():
    topo = la.la_topology_create(2, 2, 2)
    for algo, flags in (("lane_multiproc", la.LA_SCHED_STAGED), ("lane_multiproc", la.LA_SCHED_SINGLE_LAUNCH),
                        ("lane_multiproc", 0)):
        sched = la.la_schedule_build(topo, algo, 4096, "float32", flags)
        assert la.la_schedule_fusion_runs(sched) == 0, (algo, flags)
        with pytest.raises(la.LaError) as e:
            la.la_schedule_fusion_table(sched, 0)
        assert e.value.status == la.LA_ERR_INVALID_ARG
    # a staged ring packs every incoming chunk into the staging area (other offsets: no run), but its
    # gather loop copies rank buffer to rank buffer: one run of P - 1 steps after the 2(P - 1) pack and reduce steps
    sched = la.la_schedule_build(topo, "ring", 4096, "float32", la.LA_SCHED_STAGED)
    assert la.la_schedule_fusion_runs(sched) == 1
    f = la.la_schedule_fusion_table(sched, 0)
    assert (f["first_step"], f["num_steps"]) == (14, 7)
    assert la.lib().la_schedule_fusion_runs(None) == -1
    assert la.lib().la_schedule_fusion_info(None, 0, None, None, None, None, None, None, None) == la.LA_ERR_INVALID_ARG
