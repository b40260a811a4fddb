"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs.  Bit-exact for int32; bit-exact for fp32 / bf16 because the oracle adds in the same
per-segment order; and within the stated tolerance of the exact sum."""
import ctypes
import itertools

import numpy as np
import pytest

import paper_2508_13397_amd as la
from paper_2508_13397_amd import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

TOL_F32, TOL_BF16 = 1e-5, 8e-3  # max |got - exact| / sum_p |in_p|, stated by the benchmark spec
FLAG_SETS = (la.LA_SCHED_DEFAULT, la.LA_SCHED_P2P_GATHER, la.LA_SCHED_STAGED,
             la.LA_SCHED_P2P_GATHER | la.LA_SCHED_STAGED, la.LA_SCHED_INNER_RING,
             la.LA_SCHED_INNER_RING | la.LA_SCHED_STAGED)


def oracle_name(algo, flags):
    """the oracle's name of what a schedule built with these flags computes"""
    return algo + "_ring" if (flags & la.LA_SCHED_INNER_RING) and algo != "ring" else algo
ALGOS = ("ring", "lane", "lane_multiproc")
NAME = {np.dtype(np.int32): "int32", np.dtype(np.float32): "float32", np.dtype(np.uint16): "bfloat16",
        np.dtype(np.float16): "float16", np.dtype(np.float64): "float64"}


@pytest.fixture(scope="module", autouse=True)
def need_gpu():
    if not torch.cuda.is_available():
        pytest.fail("these tests need a GPU (run with -m 'not gpu' elsewhere)")
    la.lib()  # the HIP library must be there: no fallback


def to_dev(row: np.ndarray):
    if row.dtype == np.uint16:
        return torch.from_numpy(row.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(row).cuda()


def to_host(t) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def bits(a: np.ndarray) -> np.ndarray:
    return a.view(np.uint8)


def gpu_allreduce(topo, algo, x, flags=la.LA_SCHED_DEFAULT, stream=None, op="sum"):
    N, G, Q = topo
    t = la.la_topology_create(N, G, Q)
    sched = la.la_schedule_build(t, algo, x.shape[1], NAME[x.dtype], flags)
    bufs = [to_dev(x[r]) for r in range(x.shape[0])]
    la.allreduce_tensors(sched, bufs, stream, op)
    torch.cuda.synchronize()
    return np.stack([to_host(b) for b in bufs])


def make(P, n, kind, seed=0):
    if kind == "i32":
        return synth.make_inputs(P, n, "int_pm1000", seed=synth.BASE_SEED + seed)
    if kind == "i32wrap":
        return np.random.default_rng(seed).integers(-(1 << 31), 1 << 31, size=(P, n), dtype=np.int64).astype(np.int32)
    if kind == "f32":
        return synth.make_inputs(P, n, "uniform_pm1", seed=synth.BASE_SEED + seed)
    if kind == "f32order":
        return synth.order_sensitive_f32(P, n)
    if kind == "bf16":
        return synth.make_inputs(P, n, "normal_bf16", seed=synth.BASE_SEED + seed)
    raise ValueError(kind)


def check_tolerance(oracle, x, got0):
    exact = oracle.definition_sum(x)
    if x.dtype == np.uint16:
        mag = np.abs((x.astype(np.uint32) << 16).view(np.float32).astype(np.float64)).sum(axis=0)
        val = (got0.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
        tol = TOL_BF16
    else:
        mag = np.abs(x.astype(np.float64)).sum(axis=0)
        val = got0.astype(np.float64)
        tol = TOL_F32
    err = np.abs(val - exact)
    assert np.all(err <= tol * mag), f"max err/mag = {np.max(err / np.maximum(mag, 1e-300)):.3e}"


def test_c_abi_consumer_without_python_or_torch():
    """tests/consumer/consumer.exe (built by build()) allocates with HIP, calls the library
    through the C header alone and checks int32 all-reduces of seven schedules against the
    definition."""
    import os
    import subprocess

    exe = os.path.join(os.path.dirname(os.path.abspath(__file__)), "consumer", "consumer.exe")
    assert os.path.exists(exe), "run __graft_entry__.build() first: tests/consumer/consumer.exe is missing"
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and r.stdout.strip().endswith("all ok"), (r.returncode, r.stdout[-1500:], r.stderr[-1500:])


def test_package_used_before_torch_is_imported():
    """A fresh process that loads the library (a tuning call) before it imports torch still finds
    the GPU: the binding makes both share one HIP runtime.  An int32 all-reduce there equals the
    plain sum."""
    import os
    import subprocess
    import sys

    code = (
        "import sys\n"
        "import paper_2508_13397_amd as la\n"
        "assert 'torch' not in sys.modules\n"
        "la.la_tuning_get('merge')\n"
        "import torch\n"
        "topo = la.la_topology_create(2, 2, 1)\n"
        "sched = la.la_schedule_build(topo, la.LA_ALGO_LANE, 1000, la.LA_I32)\n"
        "bufs = [torch.full((1000,), r + 1, dtype=torch.int32, device='cuda:0') for r in range(4)]\n"
        "la.la_allreduce_emulated(sched, [b.data_ptr() for b in bufs], 1000, la.LA_I32, la.LA_SUM, torch.cuda.current_stream().cuda_stream)\n"
        "torch.cuda.synchronize()\n"
        "assert all(bool((b == 10).all()) for b in bufs)\n"
        "print('ok')\n")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=300, cwd=root)
    assert r.returncode == 0 and r.stdout.strip().endswith("ok"), (r.returncode, r.stdout[-1500:], r.stderr[-1500:])


# ------------------------------------------------------------------------------ config 1
# ------------------------------------------------------------------------------ config 1

@pytest.mark.parametrize("kind", ["i32", "f32"])
def test_config1_tiny_lane(oracle, kind):
    topo, n = (2, 4, 1), 65536
    x = make(8, n, kind)
    got = gpu_allreduce(topo, "lane", x)
    ref = oracle.allreduce("lane", *topo, x)
    assert np.array_equal(bits(got), bits(ref))
    if kind == "i32":
        assert np.array_equal(got[5], oracle.definition_sum(x))
    else:
        check_tolerance(oracle, x, got[0])


# ------------------------------------------------------------------------------ sweep of small cases

@pytest.mark.parametrize("algo", ALGOS)
@pytest.mark.parametrize("flags", FLAG_SETS)
def test_small_topologies_ragged_sizes_all_dtypes(oracle, algo, flags):
    cases = [((2, 2, 2), 100003), ((3, 2, 1), 40961), ((1, 3, 2), 7), ((2, 1, 3), 12289), ((1, 1, 1), 100),
             ((2, 3, 2), 5), ((4, 2, 2), 262147)]
    for (topo, n), kind in itertools.product(cases, ("i32wrap", "f32order", "bf16")):
        P = topo[0] * topo[1] * topo[2]
        x = make(P, n, kind, seed=n)
        print("case", algo, flags, topo, n, kind, flush=True)
        got = gpu_allreduce(topo, algo, x, flags)
        ref = oracle.allreduce(oracle_name(algo, flags), *topo, x)
        assert np.array_equal(bits(got), bits(ref)), (algo, flags, topo, n, kind)
        if kind == "i32wrap":
            assert np.array_equal(got[0], oracle.definition_sum(x))


@pytest.mark.parametrize("unroll,nt,block", [(u, nt, b) for u in (1, 2, 4) for nt in range(8) for b in (256, 1024)]
                         + [(8, nt, 1024) for nt in range(8)] + [(8, 3, 256), (0, -1, 0)])
def test_every_launch_shape_gives_the_same_bits(oracle, unroll, nt, block):
    try:
        la.la_tuning_set("unroll", unroll)
        la.la_tuning_set("cache_policy", nt)
        la.la_tuning_set("block", block)
        for algo, kind, n in (("lane_multiproc", "f32order", 50021), ("ring", "bf16", 33333), ("lane", "i32wrap", 9001)):
            x = make(12, n, kind, seed=unroll)
            got = gpu_allreduce((3, 2, 2), algo, x)
            ref = oracle.allreduce(algo, 3, 2, 2, x)
            assert np.array_equal(bits(got), bits(ref)), (algo, kind)
    finally:
        la.la_tuning_set("unroll", 0)
        la.la_tuning_set("cache_policy", -1)
        la.la_tuning_set("block", 0)


@pytest.mark.parametrize("kind", ["f32order", "bf16", "i32wrap"])
def test_largest_tiles_whole_and_ragged(oracle, kind):
    """128 KiB tiles (8 vectors per lane, 1024 lanes): segments of many whole tiles plus a tail"""
    try:
        la.la_tuning_set("unroll", 8)
        la.la_tuning_set("block", 1024)
        for algo, topo, n in (("lane", (2, 2, 1), 1000003), ("lane_multiproc", (2, 2, 2), 1500007), ("ring", (1, 2, 1), 300001)):
            P = topo[0] * topo[1] * topo[2]
            x = make(P, n, kind, seed=n)
            got = gpu_allreduce(topo, algo, x)
            ref = oracle.allreduce(algo, *topo, x)
            assert np.array_equal(bits(got), bits(ref)), (algo, kind)
    finally:
        la.la_tuning_set("unroll", 0)
        la.la_tuning_set("block", 0)


# ------------------------------------------------------------------------------ alignment

@pytest.mark.parametrize("kind", ["i32wrap", "f32order", "bf16"])
@pytest.mark.parametrize("offsets", ["same_odd", "mixed"])
def test_buffers_not_aligned_to_16_bytes(oracle, kind, offsets):
    topo, n = (2, 2, 2), 30011
    P = 8
    x = make(P, n, kind, seed=3)
    pad = 16
    shift = [3] * P if offsets == "same_odd" else [(r * 5) % 7 for r in range(P)]
    big = []
    for r in range(P):  # the payload sits at an odd element offset inside a zeroed allocation
        host = np.zeros(n + 2 * pad, x.dtype)
        host[shift[r]:shift[r] + n] = x[r]
        big.append(to_dev(host))
    views = [big[r][shift[r]:shift[r] + n] for r in range(P)]
    t = la.la_topology_create(*topo)
    for algo in ALGOS:
        for r in range(P):
            views[r].copy_(to_dev(x[r]))
        sched = la.la_schedule_build(t, algo, n, NAME[x.dtype])
        la.allreduce_tensors(sched, views)
        torch.cuda.synchronize()
        got = np.stack([to_host(v) for v in views])
        ref = oracle.allreduce(algo, *topo, x)
        assert np.array_equal(bits(got), bits(ref)), algo
        for r in range(P):  # nothing outside the payload was touched
            h = to_host(big[r])
            assert not h[:shift[r]].any() and not h[shift[r] + n:].any()


@pytest.mark.parametrize("kind", ["i32wrap", "f32order", "bf16"])
@pytest.mark.parametrize("shape", [(0, 0), (1024, 8), (1024, 4), (256, 4)])
def test_long_segments_that_start_between_tile_boundaries(oracle, kind, shape):
    """Segments of 8 and more tiles at arbitrary offsets: the launch cuts its tiles at absolute multiples
    of the tile size, with a short first tile per segment.  Same bits as the oracle, guards untouched."""
    block, unroll = shape
    cases = (("lane", (2, 2, 1), 2400011, 5), ("lane_multiproc", (2, 2, 2), 2500009, 0), ("ring", (1, 4, 1), 4700021, 9),
             ("lane_multiproc", (3, 2, 2), 3100003, 4100))
    try:
        la.la_tuning_set("unroll", unroll)
        la.la_tuning_set("block", block)
        for algo, topo, n, shift in cases:
            P = topo[0] * topo[1] * topo[2]
            x = make(P, n, kind, seed=n)
            pad = 8192
            big = []
            for r in range(P):
                host = np.zeros(n + 2 * pad, x.dtype)
                host[shift:shift + n] = x[r]
                big.append(to_dev(host))
            views = [big[r][shift:shift + n] for r in range(P)]
            t = la.la_topology_create(*topo)
            sched = la.la_schedule_build(t, algo, n, NAME[x.dtype])
            la.allreduce_tensors(sched, views)
            torch.cuda.synchronize()
            got = np.stack([to_host(v) for v in views])
            ref = oracle.allreduce(algo, *topo, x)
            assert np.array_equal(bits(got), bits(ref)), (algo, kind, shape)
            for r in range(P):
                h = to_host(big[r])
                assert not h[:shift].any() and not h[shift + n:].any(), (algo, kind, shape, r)
    finally:
        la.la_tuning_set("unroll", 0)
        la.la_tuning_set("block", 0)


def test_random_lengths_shifts_and_shapes_cover_every_tiling(oracle):
    """Seeded sweep of buffer lengths, view offsets and launch shapes, so that segments of under one to
    several hundred tiles start anywhere relative to the tile boundaries in memory (plain, equal and
    aligned tilings, with and without heads and tails).  int32 with wrap-around: bit-exact, guards untouched."""
    rng = np.random.default_rng(20250813)
    topos = [("lane", (2, 2, 1)), ("lane_multiproc", (2, 2, 2)), ("ring", (1, 3, 1)), ("lane_multiproc", (3, 1, 2)),
             ("rabenseifner", (2, 2, 1)), ("lane", (1, 4, 1))]
    shapes = [(0, 0), (256, 1), (256, 4), (1024, 1), (1024, 8)]
    try:
        for case in range(48):
            algo, topo = topos[int(rng.integers(len(topos)))]
            block, unroll = shapes[int(rng.integers(len(shapes)))]
            n = int(rng.integers(20_000, 2_500_000))
            shift = int(rng.integers(0, 40_000)) if case % 3 else int(rng.integers(0, 64)) * 1024
            P = topo[0] * topo[1] * topo[2]
            x = make(P, n, "i32wrap", seed=case)
            tag = (case, algo, topo, n, shift, block, unroll)
            la.la_tuning_set("unroll", unroll)
            la.la_tuning_set("block", block)
            big = []
            for r in range(P):
                host = np.zeros(n + shift + 4096, x.dtype)
                host[shift:shift + n] = x[r]
                big.append(to_dev(host))
            views = [big[r][shift:shift + n] for r in range(P)]
            sched = la.la_schedule_build(la.la_topology_create(*topo), algo, n, "int32")
            la.allreduce_tensors(sched, views)
            torch.cuda.synchronize()
            ref = oracle.allreduce(algo, *topo, x)
            for r in range(P):
                h = to_host(big[r])
                assert np.array_equal(h[shift:shift + n], ref[r]), tag + (r,)
                assert not h[:shift].any() and not h[shift + n:].any(), tag + (r,)
    finally:
        la.la_tuning_set("unroll", 0)
        la.la_tuning_set("block", 0)


@pytest.mark.parametrize("kind", ["i32wrap", "f32order", "bf16", "f16", "f64"])
def test_longest_heads_and_tails_of_every_element_size(oracle, kind):
    """Views that start one element past a 128-byte boundary: every segment whose start keeps that phase has the
    longest possible head (127 bytes of elements), and lengths are chosen so that tails of every length occur.
    The elements outside the whole vectors are done by the edge workgroups, up to 70 lanes per segment."""
    esize = {"i32wrap": 4, "f32order": 4, "bf16": 2, "f16": 2, "f64": 8}[kind]
    per_line = 128 // esize
    topo, P = (2, 2, 2), 8
    t = la.la_topology_create(*topo)
    for n in (8 * per_line * 3 + 1, 8 * per_line * 40 + per_line - 1, 8 * per_line * 40 + 16 // esize - 1, 1, per_line, 70001):
        if kind in ("f16", "f64"):
            x = wide_inputs(P, n, kind, seed=n)
        else:
            x = make(P, n, kind, seed=n)
        shift = per_line + 1  # one element past a line boundary of a 256-byte aligned allocation
        big = []
        for r in range(P):
            host = np.zeros(n + 4 * per_line, x.dtype)
            host[shift:shift + n] = x[r]
            big.append(to_dev(host))
        views = [big[r][shift:shift + n] for r in range(P)]
        for algo, flags in (("lane_multiproc", 0), ("ring", 0), ("lane_multiproc", la.LA_SCHED_SINGLE_LAUNCH)):
            for r in range(P):
                views[r].copy_(to_dev(x[r]))
            sched = la.la_schedule_build(t, algo, n, NAME[x.dtype], flags)
            la.allreduce_tensors(sched, views)
            torch.cuda.synchronize()
            got = np.stack([to_host(v) for v in views])
            ref = oracle.allreduce(algo, *topo, x)
            assert np.array_equal(bits(got), bits(ref)), (kind, n, algo, flags)
            for r in range(P):
                h = to_host(big[r])
                assert not h[:shift].any() and not h[shift + n:].any(), (kind, n, algo, flags, r)


# ------------------------------------------------------------------------------ special values

def test_fp32_special_values_and_denormals(oracle):
    topo, n = (2, 2, 1), 4096
    x = synth.make_inputs(4, n, "uniform_pm1")
    tiny = np.float32(1e-41)  # subnormal
    x[:, 0:64] = tiny * np.arange(1, 65, dtype=np.float32)
    x[0, 64:70] = [np.inf, -np.inf, np.inf, 3e38, -3e38, 0.0]
    x[1, 64:70] = [1.0, 1.0, -np.inf, 3e38, -3e38, -0.0]
    x[2, 64:70] = [np.inf, 1.0, 0.0, 3e38, -3e38, 0.0]
    x[3, 70] = np.nan
    for algo in ALGOS:
        got = gpu_allreduce(topo, algo, x)
        ref = oracle.allreduce(algo, *topo, x)
        nan = np.isnan(ref)
        assert np.array_equal(np.isnan(got), nan)
        assert np.array_equal(got.view(np.uint32)[~nan], ref.view(np.uint32)[~nan])
        assert got[0, 0] != 0.0  # subnormal sums are kept, not flushed


def test_bf16_ties_and_overflow(oracle):
    topo = (2, 2, 1)
    vals = np.array([[1.0, 2.0 ** -8, 1.0, 3 * 2.0 ** -8], [3.0e38, 3.0e38, 3.0e38, 3.0e38],
                     [1.0, 2.0 ** -9, 2.0 ** -9, 0.0], [-1.0, -(2.0 ** -8), -1.0, -3 * 2.0 ** -8]], dtype=np.float32)
    n = 64
    x = np.zeros((4, n), dtype=np.uint16)
    for c in range(vals.shape[0]):
        for r in range(4):
            x[r, c::4] = synth.to_bf16_bits(vals[c, r:r + 1])[0]
    for algo in ALGOS:
        got = gpu_allreduce(topo, algo, x)
        ref = oracle.allreduce(algo, *topo, x)
        assert np.array_equal(got, ref), algo


# ------------------------------------------------------------------------------ intermediate states

@pytest.mark.parametrize("algo", ["lane", "lane_multiproc"])
def test_lane_steps_match_oracle_rounds(oracle, algo):
    topo, n = (3, 2, 2), 24013
    P = 12
    x = make(P, n, "f32order", seed=1)
    t = la.la_topology_create(*topo)
    sched = la.la_schedule_build(t, algo, n, "float32", la.LA_SCHED_P2P_GATHER)
    assert sched.num_steps == 4
    bufs = [to_dev(x[r]) for r in range(P)]
    ptrs = [b.data_ptr() for b in bufs]
    for step in range(4):
        la.la_schedule_run_step(sched, step, ptrs, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        got = np.stack([to_host(b) for b in bufs])
        ref = oracle.allreduce(algo, *topo, x, max_rounds=step + 1)
        assert np.array_equal(bits(got), bits(ref)), step


def test_ring_steps_match_oracle_rounds(oracle):
    topo, n = (2, 3, 1), 10007
    P = 6
    x = make(P, n, "f32order", seed=2)
    sched = la.la_schedule_build(la.la_topology_create(*topo), "ring", n, "float32")
    bufs = [to_dev(x[r]) for r in range(P)]
    ptrs = [b.data_ptr() for b in bufs]
    for step in range(sched.num_steps):
        la.la_schedule_run_step(sched, step, ptrs, 0)
        torch.cuda.synchronize()
        got = np.stack([to_host(b) for b in bufs])
        ref = oracle.allreduce("ring", *topo, x, max_rounds=step + 1)
        assert np.array_equal(bits(got), bits(ref)), step


@pytest.mark.parametrize("op", ["prod", "max", "min"])
@pytest.mark.parametrize("algo,flags", [("lane_multiproc", la.LA_SCHED_P2P_GATHER), ("ring", 0),
                                        ("lane", la.LA_SCHED_INNER_RING)])
def test_steps_with_other_operations_match_oracle_rounds(oracle, algo, flags, op):
    """la_schedule_run_steps takes the operation: every step by itself, and the steps in pairs, against
    the oracle stopped after as many rounds (product, maximum, minimum; fp32 and bf16)."""
    topo, n = (3, 2, 2), 9001
    for kind in ("f32order", "bf16"):
        x = make(12, n, kind, seed=8)
        if op == "prod" and kind == "f32order":
            x = (np.sign(x) * (1.0 + (np.abs(x) % 1.0) * 0.25)).astype(np.float32)  # keep 12-fold products finite
        sched = la.la_schedule_build(la.la_topology_create(*topo), algo, n, NAME[x.dtype], flags)
        for stride in (1, 2):
            bufs = [to_dev(x[r]) for r in range(12)]
            ptrs = [b.data_ptr() for b in bufs]
            for first in range(0, sched.num_steps, stride):
                count = min(stride, sched.num_steps - first)
                print("run_steps", algo, flags, op, kind, first, count, flush=True)
                la.la_schedule_run_steps(sched, first, count, ptrs, la.OPS[op], torch.cuda.current_stream().cuda_stream)
                torch.cuda.synchronize()
                got = np.stack([to_host(b) for b in bufs])
                ref = oracle.allreduce(oracle_name(algo, flags), *topo, x, max_rounds=first + count, op=op)
                assert np.array_equal(bits(got), bits(ref)), (first, count)
    with pytest.raises(la.LaError):
        la.la_schedule_run_steps(sched, sched.num_steps, 1, ptrs)
    with pytest.raises(la.LaError):
        la.la_schedule_run_steps(sched, 0, 1, ptrs, 17)
    la.la_schedule_run_steps(sched, sched.num_steps, 0, ptrs)  # an empty range is no work


def test_copies_move_signalling_nans_unchanged(oracle):
    """A copy or broadcast step moves bits: a signalling NaN of a 16-bit type must arrive as it was
    sent (widening and narrowing it would set its quiet bit), as the gather rounds of the oracle move
    what they carry unchanged.  Reached where original inputs are copied: the out-of-place form on one
    rank (a single copy step), and the all-gather half, which distributes ranges no reduce has touched."""
    n = 4099
    for dtype, snan in ((np.uint16, [0x7F81, 0xFF81, 0x7FA0]), (np.float16, [0x7D01, 0xFD01, 0x7C01])):
        x = make(1, n, "bf16", seed=1) if dtype == np.uint16 else wide_inputs(1, n, "f16", 1)
        raw = x.view(np.uint16)
        raw[0, 5:5 + len(snan)] = snan
        raw[0, n - 1] = snan[0]
        name = NAME[x.dtype]
        sched = la.la_schedule_build(la.la_topology_create(1, 1, 1), "lane", n, name, la.LA_SCHED_OUT_OF_PLACE)
        send = to_dev(x[0]) if dtype == np.uint16 else torch.from_numpy(x[0]).cuda()
        recv = torch.zeros_like(send)
        la.la_allreduce_emulated_out_of_place(sched, [send.data_ptr()], [recv.data_ptr()], n, name)
        torch.cuda.synchronize()
        got = to_host(recv).view(np.uint16)
        assert sched.num_steps == 1 and sched.step_info(0)["kind"] == la.LA_STEP_COPY
        assert np.array_equal(got, raw[0]), name
        # the all-gather half of a ring and of a lane schedule on 2 x 2 x 1 ranks: every rank's owned range holds
        # signalling NaNs; afterwards every rank holds them all, bit for bit
        for algo in ("ring", "lane"):
            P = 4
            ag = la.la_schedule_build(la.la_topology_create(2, 2, 1), algo, n, name, la.LA_SCHED_ONLY_ALLGATHER)
            y = np.zeros((P, n), dtype=np.uint16)
            want = np.zeros(n, dtype=np.uint16)
            for r in range(P):
                for off, ln in ag.owned_ranges(r):
                    y[r, off:off + ln] = np.resize(np.array(snan, dtype=np.uint16) + r, ln)
                    want[off:off + ln] = y[r, off:off + ln]
            bufs = [torch.from_numpy(y[r].view(np.int16)).cuda().view(torch.bfloat16 if dtype == np.uint16 else torch.float16)
                    for r in range(P)]
            la.allreduce_tensors(ag, bufs)
            torch.cuda.synchronize()
            for r in range(P):
                assert np.array_equal(bufs[r].view(torch.int16).cpu().numpy().view(np.uint16), want), (name, algo, r)


# ------------------------------------------------------------------------------ streams, rebinding, repetition

def test_side_stream_rebinding_and_repeated_calls(oracle):
    topo, n = (2, 2, 2), 70001
    P = 8
    x = make(P, n, "f32", seed=9)
    t = la.la_topology_create(*topo)
    sched = la.la_schedule_build(t, "lane_multiproc", n, "float32")
    side = torch.cuda.Stream()
    a = [to_dev(x[r]) for r in range(P)]
    b = [to_dev(x[(r + 1) % P]) for r in range(P)]
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        la.allreduce_tensors(sched, a)          # binds to a
        la.allreduce_tensors(sched, a)          # same buffers: second all-reduce of the results
        la.allreduce_tensors(sched, b)          # other buffers: rebinding
    side.synchronize()
    once = oracle.allreduce("lane_multiproc", *topo, x)
    twice = oracle.allreduce("lane_multiproc", *topo, once)
    assert np.array_equal(bits(np.stack([to_host(v) for v in a])), bits(twice))
    rolled = np.stack([x[(r + 1) % P] for r in range(P)])
    assert np.array_equal(bits(np.stack([to_host(v) for v in b])), bits(oracle.allreduce("lane_multiproc", *topo, rolled)))


@pytest.mark.parametrize("flags", [0, la.LA_SCHED_STAGED])
def test_one_schedule_many_buffer_sets(oracle, flags):
    """A schedule remembers the last few buffer sets it ran on (one, when it owns a staging area):
    alternate between three sets, then cycle through ten so that remembered ones are recycled."""
    topo, n = (2, 2, 2), 30011
    P = 8
    sched = la.la_schedule_build(la.la_topology_create(*topo), "lane_multiproc", n, "float32", flags)
    xs = [make(P, n, "f32order", seed=100 + i) for i in range(10)]
    refs = [oracle.allreduce("lane_multiproc", *topo, x) for x in xs]
    sets = [[to_dev(x[r]) for r in range(P)] for x in xs]
    state = list(xs)
    for rnd in range(3):
        for i in (0, 1, 2, 0, 2, 1):
            la.allreduce_tensors(sched, sets[i])
            state[i] = oracle.allreduce("lane_multiproc", *topo, state[i])
    for rnd in range(2):
        for i in range(10):
            la.allreduce_tensors(sched, sets[i])
            state[i] = oracle.allreduce("lane_multiproc", *topo, state[i])
    torch.cuda.synchronize()
    assert np.array_equal(bits(state[9]), bits(oracle.allreduce("lane_multiproc", *topo, refs[9])))
    for i in range(10):
        got = np.stack([to_host(b) for b in sets[i]])
        assert np.array_equal(bits(got), bits(state[i])), i


def test_two_host_threads_with_their_own_schedules_and_streams(oracle):
    """Handles are independent: two host threads, each with its own schedule, buffers and stream,
    call the library at the same time (ctypes releases the interpreter lock during the call);
    la_reduce_segments calls from both share the library's pinned upload pool."""
    import threading

    # graph replay is forced on, so both threads record and replay graphs, and every iteration
    # allocates new buffers, so both rebind (table upload) and record again all the time
    cases = [("lane_multiproc", (4, 2, 2), 90001, "f32order", la.LA_SCHED_INNER_RING), ("ring", (3, 2, 1), 50021, "bf16", 0)]
    inputs = [make(t[0] * t[1] * t[2], n, kind, seed=n) for _, t, n, kind, _ in cases]
    results, errors = [None, None], []

    def work(i):
        try:
            algo, topo, n, _, flags = cases[i]
            x = inputs[i]
            stream = torch.cuda.Stream()
            sched = la.la_schedule_build(la.la_topology_create(*topo), algo, n, NAME[x.dtype], flags)
            outs, keep = [], []
            for _ in range(20):
                with torch.cuda.stream(stream):
                    bufs = [to_dev(x[r]) for r in range(x.shape[0])]
                    la.allreduce_tensors(sched, bufs, stream)
                    extra = torch.zeros(1024, dtype=torch.float32, device="cuda")
                    ones = torch.ones(1024, dtype=torch.float32, device="cuda")
                    la.la_reduce_segments(extra.data_ptr(), [ones.data_ptr()] * 1, [0, 512], 512, "float32", la.LA_SUM,
                                          stream.cuda_stream)
                stream.synchronize()
                assert torch.equal(extra, ones)
                outs.append(np.stack([to_host(b) for b in bufs]))
                keep.append(bufs)  # the next iteration gets other addresses
            results[i] = outs
        except Exception as exc:  # reported by the main thread
            errors.append((i, repr(exc)))

    la.la_tuning_set("graph", 1)
    try:
        threads = [threading.Thread(target=work, args=(i,)) for i in range(2)]
        for th in threads:
            th.start()
        for th in threads:
            th.join()
    finally:
        la.la_tuning_set("graph", -1)
    assert not errors, errors
    for i, (algo, topo, n, _, flags) in enumerate(cases):
        ref = oracle.allreduce(oracle_name(algo, flags), *topo, inputs[i])
        for got in results[i]:
            assert np.array_equal(bits(got), bits(ref)), (algo, topo)


@pytest.mark.parametrize("algo,flags,topo", [("ring", 0, (4, 2, 2)), ("lane_multiproc", la.LA_SCHED_INNER_RING, (6, 2, 2))])
def test_graph_replays_match_step_by_step_launches(oracle, algo, flags, topo):
    """Schedules with many launches are replayed as one HIP graph.  Replay it several times, with
    other GPU work and synchronisations in between, and check every replay against the oracle and
    against the step-by-step path."""
    N, G, Q = topo
    P, n = N * G * Q, 60013
    x = make(P, n, "f32order", seed=5)
    t = la.la_topology_create(N, G, Q)
    sched = la.la_schedule_build(t, algo, n, "float32", flags)
    auto = sched.num_steps >= 16  # the automatic mode takes the graph path from 16 launches on
    bufs = [to_dev(x[r]) for r in range(P)]
    eager = [to_dev(x[r]) for r in range(P)]
    esched = la.la_schedule_build(t, algo, n, "float32", flags)
    ref = x
    scratch = torch.zeros(1 << 20, device="cuda")
    try:
        la.la_tuning_set("fuse", 0)  # the ring steps would otherwise go out as one fused launch, not as a graph
        for replay in range(4):
            la.la_tuning_set("graph", -1 if auto else 1)
            la.allreduce_tensors(sched, bufs)              # graph replay
            scratch.add_(1.0)                               # unrelated eager work in between
            torch.cuda.synchronize()
            la.la_tuning_set("graph", 0)
            la.allreduce_tensors(esched, eager)            # launch by launch
            torch.cuda.synchronize()
            ref = oracle.allreduce(oracle_name(algo, flags), N, G, Q, ref)
            got = np.stack([to_host(b) for b in bufs])
            assert np.array_equal(bits(got), bits(ref)), replay
            assert np.array_equal(bits(np.stack([to_host(b) for b in eager])), bits(ref)), replay
            assert float(scratch[0]) == replay + 1
        # rebinding to other buffers drops the recorded graph and records a new one
        la.la_tuning_set("graph", 1)
        other = [to_dev(x[r]) for r in range(P)]
        la.allreduce_tensors(sched, other)
        torch.cuda.synchronize()
        assert np.array_equal(bits(np.stack([to_host(b) for b in other])), bits(oracle.allreduce(oracle_name(algo, flags), N, G, Q, x)))
    finally:
        la.la_tuning_set("graph", -1)
        la.la_tuning_set("fuse", -1)


@pytest.mark.parametrize("algo,topo", [("lane_multiproc", (2, 2, 2)), ("ring", (3, 2, 1))])
def test_repeat_calls_can_be_captured_in_a_callers_graph(oracle, algo, topo):
    """A call on a buffer set the schedule already ran on makes kernel launches and nothing else
    (no allocation, copy, memset, event or synchronisation), so a caller can record it into a graph
    of their own: three launches for the lane schedule, one fused launch for the ring.  The graph
    restores the inputs and runs the all-reduce; every replay, with eager work and synchronisations
    in between, must give the oracle's bits."""
    N, G, Q = topo
    P, n = N * G * Q, 40003
    x = make(P, n, "f32order", seed=9)
    ref = oracle.allreduce(algo, N, G, Q, x)
    sched = la.la_schedule_build(la.la_topology_create(N, G, Q), algo, n, "float32")
    bufs = [to_dev(x[r]) for r in range(P)]
    src = [b.clone() for b in bufs]
    scratch = torch.zeros(1 << 20, device="cuda")
    la.allreduce_tensors(sched, bufs)  # binds the schedule to these buffers (one upload), outside the graph
    torch.cuda.synchronize()
    assert np.array_equal(bits(np.stack([to_host(b) for b in bufs])), bits(ref))
    launches_before = la.la_tuning_get("fused_launches")
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for b, s0 in zip(bufs, src):
            b.copy_(s0)
        la.allreduce_tensors(sched, bufs)  # on torch's current stream: the capturing one
    assert la.la_tuning_get("fused_launches") - launches_before == (1 if algo == "ring" else 0)
    for replay in range(3):
        for b in bufs:
            b.fill_(float(replay))  # whatever is there is overwritten by the graph's first nodes
        scratch.add_(1.0)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(bits(np.stack([to_host(b) for b in bufs])), bits(ref)), replay
        assert np.array_equal(bits(np.stack([to_host(b) for b in src])), bits(x))
    assert float(scratch[0]) == 3.0


# ------------------------------------------------------------------------------ operations and wide types

def wide_inputs(P, n, kind, seed):
    rng = np.random.default_rng(seed)
    if kind == "f16":
        x = (rng.standard_normal((P, n)) * np.exp2(rng.integers(-16, 4, size=(P, n)))).astype(np.float16)  # normals and subnormals
        special = np.array([0.0, -0.0, 65504.0, -65504.0, 6e-8, -6e-8, 1.0, 1.0 + 2.0 ** -10], dtype=np.float16)
        x[:, : min(8, n)] = special[: min(8, n)]
        return x
    if kind == "f64":
        return rng.standard_normal((P, n)) * np.exp2(rng.integers(-40, 40, size=(P, n)))
    raise ValueError(kind)


@pytest.mark.parametrize("op", ["sum", "prod", "max", "min"])
@pytest.mark.parametrize("algo,flags", [(a, 0) for a in ALGOS] + [("lane_multiproc", la.LA_SCHED_SINGLE_LAUNCH),
                                                                  ("lane", la.LA_SCHED_FUSED_GATHER)])
def test_operations_all_dtypes(oracle, algo, flags, op):
    topo, P = (2, 3, 2), 12
    for n, kind in itertools.product((5, 40009), ("i32wrap", "f32order", "bf16", "f16", "f64")):
        x = wide_inputs(P, n, kind, n) if kind in ("f16", "f64") else make(P, n, kind, seed=n)
        if op == "prod" and kind == "i32wrap":
            x[:, ::2] = np.random.default_rng(n).integers(-5, 6, size=x[:, ::2].shape)   # some products that do not wrap
        if op in ("max", "min") and x.dtype in (np.float32, np.float64, np.float16):
            x[0, 1], x[1, 1], x[3, 2], x[5, 3], x[6, 3] = np.nan, 1.0, np.nan, 0.0, -0.0
            x[:5, 4], x[5:, 4] = -0.0, 0.0
        print("op case", algo, flags, op, n, kind, flush=True)
        got = gpu_allreduce(topo, algo, x, flags, op=op)
        ref = oracle.allreduce(algo, *topo, x, op=op)
        fl = x.dtype in (np.float32, np.float64, np.float16)
        nan = np.isnan(ref) if fl else np.zeros(ref.shape, bool)
        if fl:
            assert np.array_equal(np.isnan(got), nan)
        u = {2: np.uint16, 4: np.uint32, 8: np.uint64}[x.dtype.itemsize]
        assert np.array_equal(got.view(u)[~nan], ref.view(u)[~nan]), (algo, op, n, kind)


@pytest.mark.parametrize("kind", ["f16", "f64"])
@pytest.mark.parametrize("flags", [la.LA_SCHED_DEFAULT, la.LA_SCHED_STAGED | la.LA_SCHED_P2P_GATHER, la.LA_SCHED_INNER_RING])
def test_wide_types_ragged_and_misaligned(oracle, kind, flags):
    topo, P, n = (2, 2, 2), 8, 30011
    x = wide_inputs(P, n, kind, 3)
    for shift in (0, 1):
        big = [to_dev(np.concatenate([np.zeros(4, x.dtype), x[r], np.zeros(4, x.dtype)])) for r in range(P)]
        views = [b[shift + 3: shift + 3 + n] for b in big]   # odd element offsets, the same for all
        for r in range(P):
            views[r].copy_(to_dev(x[r]))
        sched = la.la_schedule_build(la.la_topology_create(*topo), "lane_multiproc", n, NAME[x.dtype], flags)
        la.allreduce_tensors(sched, views)
        torch.cuda.synchronize()
        got = np.stack([to_host(v) for v in views])
        ref = oracle.allreduce(oracle_name("lane_multiproc", flags), *topo, x)
        assert np.array_equal(bits(got), bits(ref)), (kind, flags, shift)


def test_reduce_segments_operations(oracle):
    n = 50000
    for kind, op in itertools.product(("i32wrap", "f32order", "f16", "f64"), ("prod", "max", "min")):
        x = wide_inputs(4, n, kind, 1) if kind in ("f16", "f64") else make(4, n, kind, seed=2)
        dst = to_dev(x[0])
        srcs = [to_dev(x[t]) for t in (1, 2, 3)]
        offs = [3, 20001, 40000]
        la.la_reduce_segments(dst.data_ptr(), [s.data_ptr() for s in srcs], offs, 7777, NAME[x.dtype], la.OPS[op])
        torch.cuda.synchronize()
        ref = oracle.reduce_segments(x[0], [x[1], x[2], x[3]], offs, 7777, op=op)
        assert np.array_equal(bits(to_host(dst)), bits(ref)), (kind, op)


def test_many_gpus_per_node_fan_in_beyond_64(oracle):
    # an MI300A node in CPX mode exposes 24 logical GPUs; with 3 processes each the S1 fan-in is 72
    topo, n = (2, 24, 3), 150001
    P = 144
    x = make(P, n, "f32order", seed=8)
    for algo in ("lane", "lane_multiproc"):
        got = gpu_allreduce(topo, algo, x)
        ref = oracle.allreduce(algo, *topo, x)
        assert np.array_equal(bits(got), bits(ref)), algo


# ------------------------------------------------------------------------------ Background-section algorithms

@pytest.mark.parametrize("algo", ["recursive_doubling", "rabenseifner"])
@pytest.mark.parametrize("extra", [0, la.LA_SCHED_STAGED])
def test_small_message_algorithms(oracle, algo, extra):
    for (topo, n), kind in itertools.product([((2, 2, 2), 100003), ((1, 1, 1), 50), ((4, 4, 1), 7), ((2, 4, 4), 65536), ((1, 2, 1), 4099)],
                                             ("i32wrap", "f32order", "bf16")):
        P = topo[0] * topo[1] * topo[2]
        x = make(P, n, kind, seed=n)
        print("small-message case", algo, extra, topo, n, kind, flush=True)
        got = gpu_allreduce(topo, algo, x, extra)
        ref = oracle.allreduce(algo, *topo, x)
        assert np.array_equal(bits(got), bits(ref)), (algo, extra, topo, n, kind)


# ------------------------------------------------------------------------------ out-of-place form

@pytest.mark.parametrize("algo", ALGOS)
@pytest.mark.parametrize("extra", [0, la.LA_SCHED_STAGED, la.LA_SCHED_INNER_RING, la.LA_SCHED_P2P_GATHER])
def test_out_of_place_send_untouched_receive_complete(oracle, algo, extra):
    for (topo, n), kind in itertools.product([((2, 2, 2), 100003), ((1, 1, 1), 1000), ((3, 1, 2), 7), ((2, 3, 1), 40961)],
                                             ("i32wrap", "f32order", "bf16")):
        N, G, Q = topo
        P = N * G * Q
        x = make(P, n, kind, seed=n)
        sched = la.la_schedule_build(la.la_topology_create(N, G, Q), algo, n, NAME[x.dtype], la.LA_SCHED_OUT_OF_PLACE | extra)
        send = [to_dev(x[r]) for r in range(P)]
        recv = [torch.full_like(send[r], 7) for r in range(P)]
        print("oop case", algo, extra, topo, n, kind, flush=True)
        la.la_allreduce_emulated_out_of_place(sched, [t.data_ptr() for t in send], [t.data_ptr() for t in recv], n,
                                              NAME[x.dtype], la.LA_SUM, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        ref = oracle.allreduce(oracle_name(algo, extra), N, G, Q, x)
        assert np.array_equal(bits(np.stack([to_host(t) for t in recv])), bits(ref)), (algo, extra, topo, n, kind)
        assert np.array_equal(bits(np.stack([to_host(t) for t in send])), bits(x))


# ------------------------------------------------------------------------------ shared-buffer model

@pytest.mark.parametrize("algo", ["lane", "lane_multiproc"])
@pytest.mark.parametrize("extra", [0, la.LA_SCHED_STAGED, la.LA_SCHED_SHARED_BUFFERS])
def test_fused_gather_small_topologies(oracle, algo, extra):
    cases = [((2, 2, 2), 100003), ((3, 2, 1), 40961), ((1, 3, 2), 7), ((2, 1, 3), 12289), ((1, 1, 1), 100),
             ((2, 3, 2), 5), ((4, 2, 2), 262147), ((1, 4, 2), 300007)]
    for (topo, n), kind in itertools.product(cases, ("i32wrap", "f32order", "bf16")):
        N, G, Q = topo
        B = N * G if extra & la.LA_SCHED_SHARED_BUFFERS else N * G * Q
        x = make(B, n, kind, seed=n)
        print("fused case", algo, extra, topo, n, kind, flush=True)
        got = gpu_allreduce(topo, algo, x, la.LA_SCHED_FUSED_GATHER | extra)
        if extra & la.LA_SCHED_SHARED_BUFFERS:
            ref = oracle.allreduce("lane_multiproc", N, G, 1 if algo == "lane" else Q, x, shared=True)
        else:
            ref = oracle.allreduce(algo, N, G, Q, x)
        assert np.array_equal(bits(got), bits(ref)), (algo, extra, topo, n, kind)


@pytest.mark.parametrize("algo", ["lane", "lane_multiproc"])
@pytest.mark.parametrize("extra", [0, la.LA_SCHED_SHARED_BUFFERS])
def test_single_launch_small_topologies(oracle, algo, extra):
    cases = [((2, 2, 2), 100003), ((3, 2, 1), 40961), ((1, 3, 2), 7), ((2, 1, 3), 12289), ((1, 1, 1), 100),
             ((2, 3, 2), 5), ((4, 2, 2), 262147), ((1, 4, 2), 300007), ((3, 1, 1), 70001)]
    for (topo, n), kind in itertools.product(cases, ("i32wrap", "f32order", "bf16")):
        N, G, Q = topo
        B = N * G if extra & la.LA_SCHED_SHARED_BUFFERS else N * G * Q
        x = make(B, n, kind, seed=n)
        print("one-launch case", algo, extra, topo, n, kind, flush=True)
        got = gpu_allreduce(topo, algo, x, la.LA_SCHED_SINGLE_LAUNCH | extra)
        if extra & la.LA_SCHED_SHARED_BUFFERS:
            ref = oracle.allreduce("lane_multiproc", N, G, 1 if algo == "lane" else Q, x, shared=True)
        else:
            ref = oracle.allreduce(algo, N, G, Q, x)
        assert np.array_equal(bits(got), bits(ref)), (algo, extra, topo, n, kind)


def test_single_launch_every_launch_shape_and_misaligned_views(oracle):
    """forced tile shapes, and rank buffers that start at odd element offsets (head / tail peel and
    the element-wise path when the operands disagree modulo 16 bytes)"""
    topo, n = (2, 2, 2), 50021
    P = 8
    x = make(P, n, "bf16", seed=11)
    ref = oracle.allreduce("lane_multiproc", *topo, x)
    t = la.la_topology_create(*topo)
    sched = la.la_schedule_build(t, "lane_multiproc", n, "bfloat16", la.LA_SCHED_SINGLE_LAUNCH)
    try:
        for unroll, block in ((1, 256), (2, 256), (4, 256), (1, 1024), (2, 1024), (4, 1024), (8, 1024)):
            la.la_tuning_set("unroll", unroll)
            la.la_tuning_set("block", block)
            got = gpu_allreduce(topo, "lane_multiproc", x, la.LA_SCHED_SINGLE_LAUNCH)
            assert np.array_equal(bits(got), bits(ref)), (unroll, block)
    finally:
        la.la_tuning_set("unroll", 0)
        la.la_tuning_set("block", 0)
    for offsets in ([3] * P, [1, 2, 3, 4, 5, 6, 7, 9]):
        slabs = [torch.zeros(n + 16, dtype=torch.bfloat16, device="cuda") for _ in range(P)]
        views = [slabs[r][offsets[r]: offsets[r] + n] for r in range(P)]
        for r in range(P):
            views[r].copy_(to_dev(x[r]))
        la.allreduce_tensors(sched, views)
        torch.cuda.synchronize()
        got = np.stack([to_host(v) for v in views])
        assert np.array_equal(bits(got), bits(ref)), offsets


RS, AG = la.LA_SCHED_ONLY_REDUCE_SCATTER, la.LA_SCHED_ONLY_ALLGATHER


def half_rounds(algo, flags, N, G, Q):
    """oracle rounds that make up the reduce-scatter half of a schedule"""
    P = N * G * Q
    if algo == "ring":
        return P - 1
    if algo == "rabenseifner":
        return P.bit_length() - 1
    return N if flags & la.LA_SCHED_INNER_RING else 2


def owned_mask(sched, B, n):
    mask = np.zeros((B, n), dtype=bool)
    for b in range(B):
        for off, ln in sched.owned_ranges(b):
            mask[b, off:off + ln] = True
    return mask


@pytest.mark.parametrize("algo,flags", [(a, f) for a in ALGOS for f in (0, la.LA_SCHED_STAGED, la.LA_SCHED_INNER_RING, la.LA_SCHED_P2P_GATHER)]
                         + [("rabenseifner", 0)])
def test_stand_alone_reduce_scatter_and_allgather(oracle, algo, flags):
    """First half: the state equals the oracle stopped after its reduce-scatter rounds, and the
    owned ranges already hold the all-reduce.  Second half, started from buffers that hold
    nothing but the owned ranges (the rest is NaN / a marker), yields the oracle's all-reduce."""
    cases = [((2, 2, 2), 100003), ((4, 2, 1), 40961), ((1, 4, 2), 7), ((4, 2, 2), 262147), ((1, 1, 1), 33)]
    if algo != "rabenseifner":
        cases += [((3, 2, 1), 12289), ((2, 3, 2), 5)]
    for (topo, n), kind in itertools.product(cases, ("i32wrap", "f32order", "bf16")):
        P = topo[0] * topo[1] * topo[2]
        x = make(P, n, kind, seed=n)
        print("case", algo, flags, topo, n, kind, flush=True)
        name = oracle_name(algo, flags)
        ref_full = oracle.allreduce(name, *topo, x)
        ref_half = oracle.allreduce(name, *topo, x, max_rounds=half_rounds(algo, flags, *topo))
        mid = gpu_allreduce(topo, algo, x, flags | RS)
        assert np.array_equal(bits(mid), bits(ref_half)), (algo, flags, topo, n, kind)
        t = la.la_topology_create(*topo)
        mask = owned_mask(la.la_schedule_build(t, algo, n, NAME[x.dtype], flags | AG), P, n)
        assert np.array_equal(mask.sum(axis=0), np.ones(n, dtype=np.int64))
        assert np.array_equal(bits(mid[mask]), bits(ref_full[mask]))
        marker = {np.dtype(np.int32): np.int32(-559038737), np.dtype(np.float32): np.float32(np.nan),
                  np.dtype(np.uint16): np.uint16(0x7fc1)}[x.dtype]
        start = np.where(mask, ref_full, marker).astype(x.dtype)
        out = gpu_allreduce(topo, algo, start, flags | AG)
        assert np.array_equal(bits(out), bits(ref_full)), (algo, flags, topo, n, kind)


@pytest.mark.parametrize("algo", ALGOS)
def test_stand_alone_halves_out_of_place(oracle, algo):
    for topo, n in [((2, 2, 2), 100003), ((3, 2, 1), 4099), ((1, 1, 1), 33)]:
        P = topo[0] * topo[1] * topo[2]
        x = make(P, n, "f32order", seed=n)
        ref = oracle.allreduce(algo, *topo, x)
        t = la.la_topology_create(*topo)
        outs = []
        for half, src in ((RS, x), (AG, None)):
            sched = la.la_schedule_build(t, algo, n, "float32", half | la.LA_SCHED_OUT_OF_PLACE)
            mask = owned_mask(sched, P, n)
            if src is None:
                src = np.where(mask, ref, np.float32(np.nan)).astype(np.float32)
            send = [to_dev(src[r]) for r in range(P)]
            recv = [torch.full((n,), -7.0, dtype=torch.float32, device="cuda") for _ in range(P)]
            la.la_allreduce_emulated_out_of_place(sched, [b.data_ptr() for b in send], [b.data_ptr() for b in recv], n,
                                                  "float32", la.LA_SUM, torch.cuda.current_stream().cuda_stream)
            torch.cuda.synchronize()
            got = np.stack([to_host(b) for b in recv])
            assert np.array_equal(bits(np.stack([to_host(b) for b in send])), bits(src))
            outs.append((got, mask))
        (mid, mask), (full, _) = outs
        assert np.array_equal(bits(mid[mask]), bits(ref[mask])), (algo, topo, n)
        assert np.array_equal(bits(full), bits(ref)), (algo, topo, n)


def test_stand_alone_halves_config2_full_size(oracle):
    """16 ranks x 16 Mi fp32: sampled columns of each half against the oracle run on those columns."""
    topo, n = (4, 4, 1), 1 << 24
    P = 16
    x = synth.make_inputs(P, n, "uniform_pm1", seed=synth.BASE_SEED + 2)
    t = la.la_topology_create(*topo)
    rs = la.la_schedule_build(t, "lane", n, "float32", RS)
    ag = la.la_schedule_build(t, "lane", n, "float32", AG)
    bufs = [to_dev(x[r]) for r in range(P)]
    la.allreduce_tensors(rs, bufs)
    torch.cuda.synchronize()
    mid = np.stack([to_host(b) for b in bufs])
    exact = oracle.definition_sum(x)
    mask = owned_mask(rs, P, n)
    assert np.array_equal(mask.sum(axis=0), np.ones(n, dtype=np.int64))
    owned_vals = mid[mask.argmax(axis=0), np.arange(n)]
    mag = np.abs(x.astype(np.float64)).sum(axis=0)
    assert np.all(np.abs(owned_vals.astype(np.float64) - exact) <= TOL_F32 * mag)
    ref = oracle.allreduce("lane", *topo, x)
    assert np.array_equal(bits(owned_vals), bits(ref[0]))
    la.allreduce_tensors(ag, bufs)
    torch.cuda.synchronize()
    out = np.stack([to_host(b) for b in bufs])
    assert np.array_equal(bits(out), bits(ref))


SHARED = la.LA_SCHED_SHARED_BUFFERS


@pytest.mark.parametrize("algo", ["ring", "lane_multiproc", "lane"])
@pytest.mark.parametrize("extra", [0, la.LA_SCHED_P2P_GATHER, la.LA_SCHED_STAGED])
def test_shared_buffers_small_topologies(oracle, algo, extra):
    for (topo, n), kind in itertools.product([((2, 2, 2), 100003), ((3, 2, 4), 40961), ((1, 3, 2), 7), ((2, 1, 3), 12289),
                                              ((2, 4, 3), 262147)], ("i32wrap", "f32order", "bf16")):
        N, G, Q = topo
        B = N * G
        x = make(B, n, kind, seed=n)
        print("shared case", algo, extra, topo, n, kind, flush=True)
        t = la.la_topology_create(N, G, Q)
        sched = la.la_schedule_build(t, algo, n, NAME[x.dtype], SHARED | extra)
        assert sched.num_buffers == B
        bufs = [to_dev(x[b]) for b in range(B)]
        la.allreduce_tensors(sched, bufs)
        torch.cuda.synchronize()
        got = np.stack([to_host(b) for b in bufs])
        if algo == "lane":
            ref = oracle.allreduce("lane_multiproc", N, G, 1, x, shared=True)
        else:
            ref = oracle.allreduce(algo, N, G, Q, x, shared=True)
        assert np.array_equal(bits(got), bits(ref)), (algo, extra, topo, n, kind)


@pytest.mark.parametrize("algo,extra", [("ring", 0), ("lane_multiproc", 0), ("lane_multiproc", la.LA_SCHED_STAGED)])
def test_shared_buffers_full_size_16_gpus_4_procs_64Mi_fp32(oracle, algo, extra):
    # the paper's regime: a large fp32 buffer per GPU, several processes per GPU each on a slice
    N, G, Q, n = 4, 4, 4, 1 << 26
    B = N * G
    x = synth.make_inputs(B, n, "normal", workers=16)
    sched = la.la_schedule_build(la.la_topology_create(N, G, Q), algo, n, "float32", SHARED | extra)
    bufs = [to_dev(x[b]) for b in range(B)]
    la.allreduce_tensors(sched, bufs)
    torch.cuda.synchronize()
    got0 = to_host(bufs[0])
    for b in range(1, B):
        assert torch.equal(bufs[b].view(torch.int32), bufs[0].view(torch.int32)), b
    del bufs
    torch.cuda.empty_cache()
    oracle.set_threads(min(16, oracle.max_threads()))
    ref = oracle.allreduce(algo, N, G, Q, x, in_place=True, shared=True)
    assert np.array_equal(bits(got0), bits(ref[0]))


# ------------------------------------------------------------------------------ la_reduce_segments

@pytest.mark.parametrize("algo,extra", [("lane_multiproc", 0), ("lane_multiproc", la.LA_SCHED_FUSED_GATHER), ("ring", 0)])
def test_paper_size_8_nodes_4_gpus_16_procs_128Mi_fp32(oracle, algo, extra):
    """The size the paper's Delta runs are quoted on (Results: 2^27 floats per GPU, 8 nodes of 4
    GPUs, up to 16 processes per GPU), shared-buffer model: 32 buffers of 512 MiB resident."""
    N, G, Q, n = 8, 4, 16, 1 << 27
    B = N * G
    print("generating", B, "x", n, flush=True)
    x = synth.make_inputs(B, n, "uniform_pm1", workers=16)
    sched = la.la_schedule_build(la.la_topology_create(N, G, Q), algo, n, "float32", SHARED | extra)
    bufs = [to_dev(x[b]) for b in range(B)]
    print("running", algo, extra, flush=True)
    la.allreduce_tensors(sched, bufs)
    torch.cuda.synchronize()
    got0 = to_host(bufs[0])
    for b in range(1, B):
        assert torch.equal(bufs[b].view(torch.int32), bufs[0].view(torch.int32)), b
    del bufs
    torch.cuda.empty_cache()
    idx = np.unique(np.concatenate([np.arange(0, 4096), np.arange(n - 4096, n), np.random.default_rng(2).integers(0, n, 100000)]))
    check_tolerance(oracle, np.ascontiguousarray(x[:, idx]), got0[idx])
    print("oracle", flush=True)
    oracle.set_threads(min(16, oracle.max_threads()))
    ref = oracle.allreduce(algo, N, G, Q, x, in_place=True, shared=True)
    assert np.array_equal(bits(got0), bits(ref[0]))


def test_largest_paper_topology_128_buffers_of_1_GiB(oracle):
    """32 nodes x 4 GPUs (the largest node count of the Results section) at 2^28 elements per GPU
    buffer, 16 processes per GPU: 128 GiB resident in one GPU's HBM.  Too large for the schedule
    oracle on the host, so: int32 data generated on the device from per-buffer seeds, every buffer
    must end bit-equal to buffer 0, and 200,000 sampled columns (plus the ends and the middle of
    the buffer) must equal the definition, the wrapping sum, computed by the oracle from the inputs
    of those columns; then fp32 data against the schedule oracle on the sampled columns."""
    N, G, Q, n = 32, 4, 16, 1 << 28
    B = N * G
    torch.cuda.empty_cache()
    free, _ = torch.cuda.mem_get_info()
    if free < (B * n * 4) * 1.05:
        pytest.skip("needs 135 GiB of free device memory")
    idx = np.unique(np.concatenate([np.arange(0, 2048), np.arange(n - 2048, n), np.arange(n // 2 - 1024, n // 2 + 1024),
                                    np.random.default_rng(3).integers(0, n, 200000)]))
    didx = torch.from_numpy(idx).cuda()

    def inputs():
        out = []
        for b in range(B):
            g = torch.Generator(device="cuda")
            g.manual_seed(synth.BASE_SEED + b)
            out.append(torch.randint(-(1 << 31), (1 << 31) - 1, (n,), dtype=torch.int32, device="cuda", generator=g))
        return out

    want = None
    for algo, flags in (("lane_multiproc", SHARED), ("lane_multiproc", SHARED | la.LA_SCHED_FUSED_GATHER), ("ring", SHARED)):
        work = inputs()
        cols = np.stack([t[didx].cpu().numpy() for t in work])
        if want is None:
            want = oracle.definition_sum(cols)
        else:
            assert np.array_equal(oracle.definition_sum(cols), want)   # the same inputs again
        sched = la.la_schedule_build(la.la_topology_create(N, G, Q), algo, n, "int32", flags)
        print("running", algo, flags, flush=True)
        la.allreduce_tensors(sched, work)
        torch.cuda.synchronize()
        for b in range(1, B):
            assert torch.equal(work[b], work[0]), (algo, flags, b)
        got = work[0][didx].cpu().numpy()
        assert np.array_equal(got, want), (algo, flags)
        del work, sched
        torch.cuda.empty_cache()

    # fp32, bit for bit: in Algorithm 2 the order in which an element is summed (the GPUs of a node
    # in ascending order, then the nodes in ascending order) does not depend on where the element
    # lies in the buffer, so the schedule oracle run on the sampled columns alone gives the bits
    # every sampled element must have.
    def finputs():
        out = []
        for b in range(B):
            g = torch.Generator(device="cuda")
            g.manual_seed(synth.BASE_SEED + 1000 + b)
            out.append(torch.rand(n, dtype=torch.float32, device="cuda", generator=g).mul_(2.0).sub_(1.0))
        return out

    for flags in (SHARED, SHARED | la.LA_SCHED_SINGLE_LAUNCH):
        work = finputs()
        cols = np.stack([t[didx].cpu().numpy() for t in work])
        ref = oracle.allreduce("lane_multiproc", N, G, Q, cols, shared=True)
        sched = la.la_schedule_build(la.la_topology_create(N, G, Q), "lane_multiproc", n, "float32", flags)
        print("running fp32", flags, flush=True)
        la.allreduce_tensors(sched, work)
        torch.cuda.synchronize()
        for b in range(1, B):
            assert torch.equal(work[b].view(torch.int32), work[0].view(torch.int32)), (flags, b)
        got = work[0][didx].cpu().numpy()
        assert np.array_equal(bits(got), bits(ref[0])), flags
        del work, sched
        torch.cuda.empty_cache()


@pytest.mark.parametrize("kind", ["i32wrap", "f32order", "bf16"])
def test_reduce_segments_matches_oracle(oracle, kind):
    n = 200000
    for k, seg_len, offs in ((1, 4096, [0, 8192, 100000]), (2, 5000, [3, 7001, 150001]), (3, 1, [5, 9, 11]),
                             (5, 33333, [1, 40000, 80001, 160000]), (8, 12345, [77]), (9, 7, [0, 7, 14, 21, 199993]),
                             (0, 100, [0, 500]), (4, 0, [0, 1]), (16, 2049, [1000, 5000, 9000])):
        x = make(k + 1, n, kind, seed=k)
        dst = to_dev(x[0])
        srcs = [to_dev(x[t + 1]) for t in range(k)]
        print("reduce_segments", kind, k, seg_len, offs, flush=True)
        la.la_reduce_segments(dst.data_ptr(), [s.data_ptr() for s in srcs], offs, seg_len, NAME[x.dtype],
                              la.LA_SUM, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        ref = oracle.reduce_segments(x[0], [x[t + 1] for t in range(k)], offs, seg_len)
        assert np.array_equal(bits(to_host(dst)), bits(ref)), (k, seg_len)


def test_reduce_segments_many_segments_and_misaligned_sources(oracle):
    n, seg_len = 1 << 20, 1000
    offs = [i * 1024 + (i % 5) for i in range(1000)]
    x = make(4, n + 8, "f32order", seed=4)
    dst = to_dev(x[0])
    srcs_full = [to_dev(x[t]) for t in (1, 2, 3)]
    srcs = [srcs_full[0][1:], srcs_full[1][2:], srcs_full[2][0:]]  # different 16-byte phases
    la.la_reduce_segments(dst.data_ptr(), [s.data_ptr() for s in srcs], offs, seg_len, "float32")
    torch.cuda.synchronize()
    ref = oracle.reduce_segments(x[0], [x[1][1:], x[2][2:], x[3]], offs, seg_len)
    assert np.array_equal(bits(to_host(dst)), bits(ref))


@pytest.mark.parametrize("flags", [0, la.LA_SCHED_FUSED_GATHER, la.LA_SCHED_SINGLE_LAUNCH, la.LA_SCHED_P2P_GATHER])
def test_merged_and_unmerged_launch_segments_give_the_same_bits(oracle, flags):
    """Table-adjacent segments that continue each other are launched as one (the pieces of a part in
    the inter-node step, everything in the one-launch form); with the knob off every table segment
    is launched by itself.  Both must equal the oracle bit for bit, on lengths that leave ragged
    pieces and on views at an odd offset."""
    topo = (3, 2, 2)
    for kind, n, shift in (("f32order", 100003, 0), ("bf16", 77777, 3), ("i32wrap", 4099, 1), ("f32order", 1 << 18, 0)):
        x = make(12, n, kind, seed=9)
        ref = oracle.allreduce("lane_multiproc", *topo, x)
        for merge in (1, 0):
            try:
                la.la_tuning_set("merge", merge)
                t = la.la_topology_create(*topo)
                sched = la.la_schedule_build(t, "lane_multiproc", n, NAME[x.dtype], flags)
                full = [to_dev(np.concatenate([x[r][:shift], x[r], x[r][:8]])) for r in range(12)]
                views = [f[shift: shift + n] for f in full]
                print("merge", merge, kind, n, shift, flags, flush=True)
                la.la_allreduce_emulated(sched, [v.data_ptr() for v in views], n, NAME[x.dtype], la.LA_SUM,
                                         torch.cuda.current_stream().cuda_stream)
                torch.cuda.synchronize()
                got = np.stack([to_host(v) for v in views])
            finally:
                la.la_tuning_set("merge", 1)
            assert np.array_equal(bits(got), bits(ref)), (kind, n, shift, flags, merge)


# ------------------------------------------------------------------------------ one launch for all steps

class fused_launch:
    """with fused_launch(mode): ... sets the "fuse" knob (1: every run of two or more steps with at most two
    sources and destinations per segment goes out as one launch; -1: the automatic choice; 0: none);
    .count = fused launches made inside"""

    def __init__(self, mode=1):
        self.mode = mode

    def __enter__(self):
        la.la_tuning_set("fuse", self.mode)
        self.start = la.la_tuning_get("fused_launches")
        return self

    def __exit__(self, *exc):
        self.count = la.la_tuning_get("fused_launches") - self.start
        la.la_tuning_set("fuse", -1)
        return False


@pytest.mark.parametrize("algo,flags", [("ring", 0), ("lane", 0), ("lane_multiproc", 0), ("lane", la.LA_SCHED_INNER_RING),
                                        ("lane_multiproc", la.LA_SCHED_INNER_RING), ("lane_multiproc", la.LA_SCHED_P2P_GATHER),
                                        ("lane_multiproc", la.LA_SCHED_FUSED_GATHER), ("rabenseifner", 0),
                                        ("recursive_doubling", 0)])
def test_fused_launch_small_topologies_ragged_sizes_all_dtypes(oracle, algo, flags):
    """The whole schedule in one launch, every chain start to end by one wave: bit-equal to the
    oracle (and so to the step-by-step launches) on lengths with ragged chains, heads and tails."""
    topos = [(2, 2, 2), (4, 2, 1), (1, 4, 2)] if algo in ("rabenseifner", "recursive_doubling") else \
            [(2, 2, 2), (3, 2, 1), (1, 3, 2), (2, 1, 3), (5, 1, 1), (4, 2, 2)]
    for topo in topos:
        P = topo[0] * topo[1] * topo[2]
        for n, kind in ((1, "i32wrap"), (7, "f32order"), (1000, "bf16"), (4097, "f32order"), (65536, "i32wrap"),
                        (100003, "bf16"), (262144 + 5, "f32order")):
            x = make(P, n, kind, seed=n)
            ref = oracle.allreduce(oracle_name(algo, flags), *topo, x)
            print("fused", algo, flags, topo, n, kind, flush=True)
            with fused_launch() as f:
                got = gpu_allreduce(topo, algo, x, flags)
            runs = la.la_schedule_fusion_runs(la.la_schedule_build(la.la_topology_create(*topo), algo, n, NAME[x.dtype], flags))
            assert f.count == runs, (algo, topo, n, f.count, runs)
            assert np.array_equal(bits(got), bits(ref)), (algo, flags, topo, n, kind)


@pytest.mark.parametrize("op", ["sum", "prod", "max", "min"])
def test_fused_launch_operations_and_wide_types(oracle, op):
    topo, n = (3, 2, 2), 30011
    for kind in ("i32wrap", "f32order", "bf16", "f16", "f64"):
        x = wide_inputs(12, n, kind, 3) if kind in ("f16", "f64") else make(12, n, kind, seed=5)
        for algo, flags in (("ring", 0), ("lane_multiproc", la.LA_SCHED_INNER_RING)):
            ref = oracle.allreduce(oracle_name(algo, flags), *topo, x, op=op)
            print("fused", op, kind, algo, flush=True)
            with fused_launch() as f:
                got = gpu_allreduce(topo, algo, x, flags, op=op)
            assert f.count == 1
            assert np.array_equal(bits(got), bits(ref)), (op, kind, algo)


def test_fused_launch_views_at_odd_offsets_and_fallback(oracle):
    """Views that share an odd element offset have heads and tails in every chain; views whose offsets
    differ modulo 16 bytes cannot run fused and must fall back to the step-by-step launches."""
    topo, n = (2, 2, 2), 50001
    for kind in ("f32order", "bf16", "i32wrap"):
        x = make(8, n, kind, seed=11)
        ref = oracle.allreduce("ring", *topo, x)
        for shifts, fused in (([3] * 8, 1), ([1] * 8, 1), ([0, 1, 2, 3, 4, 5, 6, 7], 0)):
            full = [to_dev(np.concatenate([x[r][:shifts[r]], x[r], x[r][:8]])) for r in range(8)]
            views = [full[r][shifts[r]: shifts[r] + n] for r in range(8)]
            sched = la.la_schedule_build(la.la_topology_create(*topo), "ring", n, NAME[x.dtype])
            print("fused views", kind, shifts, flush=True)
            with fused_launch() as f:
                la.la_allreduce_emulated(sched, [v.data_ptr() for v in views], n, NAME[x.dtype], la.LA_SUM,
                                         torch.cuda.current_stream().cuda_stream)
                torch.cuda.synchronize()
            assert f.count == fused, (kind, shifts, f.count)
            got = np.stack([to_host(v) for v in views])
            assert np.array_equal(bits(got), bits(ref)), (kind, shifts)
            # the elements around the views are untouched
            for r in range(8):
                h = to_host(full[r])
                assert np.array_equal(h[:shifts[r]], x[r][:shifts[r]]) and np.array_equal(h[shifts[r] + n:], x[r][:8])


def test_fused_launch_out_of_place_shared_buffers_and_repeats(oracle):
    topo, n = (2, 2, 2), 70001
    x = make(8, n, "f32order", seed=2)
    ref = oracle.allreduce("ring", *topo, x)
    sched = la.la_schedule_build(la.la_topology_create(*topo), "ring", n, "float32", la.LA_SCHED_OUT_OF_PLACE)
    send = [to_dev(x[r]) for r in range(8)]
    recv = [torch.full((n,), float("nan"), dtype=torch.float32, device="cuda") for _ in range(8)]
    with fused_launch() as f:
        for _ in range(3):  # the second and third call reuse the binding's fused tables
            la.la_allreduce_emulated_out_of_place(sched, [t.data_ptr() for t in send], [t.data_ptr() for t in recv], n,
                                                  "float32", la.LA_SUM, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
    assert f.count == 3
    assert np.array_equal(bits(np.stack([to_host(t) for t in recv])), bits(ref))
    assert np.array_equal(np.stack([to_host(t) for t in send]), x)
    # shared buffers, standard approach: Q rings in one launch per iteration; fused: one launch in all
    xs = make(4, n, "bf16", seed=4)
    refs = oracle.allreduce("ring", *topo, xs, shared=True)
    sh = la.la_schedule_build(la.la_topology_create(*topo), "ring", n, "bfloat16", la.LA_SCHED_SHARED_BUFFERS)
    bufs = [to_dev(xs[b]) for b in range(4)]
    with fused_launch() as f:
        la.allreduce_tensors(sh, bufs)
        torch.cuda.synchronize()
    assert f.count == 1
    assert np.array_equal(bits(np.stack([to_host(b) for b in bufs])), bits(refs))
    # a staged ring: the pack and reduce steps work through the staging area and keep their launches,
    # the gather loop (rank buffer to rank buffer) is one fused launch
    st = la.la_schedule_build(la.la_topology_create(*topo), "ring", n, "float32", la.LA_SCHED_STAGED)
    bufs = [to_dev(x[r]) for r in range(8)]
    with fused_launch() as f:
        la.allreduce_tensors(st, bufs)
        torch.cuda.synchronize()
    assert f.count == 1
    assert np.array_equal(bits(np.stack([to_host(b) for b in bufs])), bits(ref))
    # with the knob off nothing is fused, and the result is the same
    bufs = [to_dev(x[r]) for r in range(8)]
    plain = la.la_schedule_build(la.la_topology_create(*topo), "ring", n, "float32")
    with fused_launch(0) as f:
        la.allreduce_tensors(plain, bufs)
        torch.cuda.synchronize()
    assert f.count == 0
    assert np.array_equal(bits(np.stack([to_host(b) for b in bufs])), bits(ref))
    # the automatic choice fuses the ring (14 steps, one operation per step and chain) ...
    bufs = [to_dev(x[r]) for r in range(8)]
    with fused_launch(-1) as f:
        la.allreduce_tensors(plain, bufs)
        torch.cuda.synchronize()
    assert f.count == 1
    assert np.array_equal(bits(np.stack([to_host(b) for b in bufs])), bits(ref))
    # ... with and without taking the incoming chunk from registers
    try:
        la.la_tuning_set("forward", 0)
        bufs = [to_dev(x[r]) for r in range(8)]
        with fused_launch(-1) as f:
            la.allreduce_tensors(plain, bufs)
            torch.cuda.synchronize()
        assert f.count == 1
        assert np.array_equal(bits(np.stack([to_host(b) for b in bufs])), bits(ref))
    finally:
        la.la_tuning_set("forward", 1)
    # ... but not recursive doubling (4 steps, 8 operations per step on its one chain)
    rd = la.la_schedule_build(la.la_topology_create(*topo), "recursive_doubling", n, "float32")
    bufs = [to_dev(x[r]) for r in range(8)]
    with fused_launch(-1) as f:
        la.allreduce_tensors(rd, bufs)
        torch.cuda.synchronize()
    assert f.count == 0
    assert np.array_equal(bits(np.stack([to_host(b) for b in bufs])), bits(oracle.allreduce("recursive_doubling", *topo, x)))


@pytest.mark.parametrize("algo,flags", [("ring", 0), ("lane_multiproc", 0), ("lane", la.LA_SCHED_INNER_RING), ("rabenseifner", 0)])
def test_fused_launch_of_the_stand_alone_halves(oracle, algo, flags):
    """Reduce-scatter half then all-gather half, each as one fused launch: together the all-reduce.
    (The all-gather half of a lane schedule broadcasts original inputs: one source, many destinations.)"""
    topo, n = ((2, 2, 2) if algo == "rabenseifner" else (3, 2, 2)), 40003
    P = topo[0] * topo[1] * topo[2]
    for kind in ("f32order", "bf16"):
        x = make(P, n, kind, seed=6)
        ref = oracle.allreduce(oracle_name(algo, flags), *topo, x)
        t = la.la_topology_create(*topo)
        rs = la.la_schedule_build(t, algo, n, NAME[x.dtype], flags | la.LA_SCHED_ONLY_REDUCE_SCATTER)
        ag = la.la_schedule_build(t, algo, n, NAME[x.dtype], flags | la.LA_SCHED_ONLY_ALLGATHER)
        bufs = [to_dev(x[r]) for r in range(P)]
        print("fused halves", algo, flags, kind, rs.num_steps, ag.num_steps, flush=True)
        with fused_launch() as f:
            la.allreduce_tensors(rs, bufs)
            la.allreduce_tensors(ag, bufs)
            torch.cuda.synchronize()
        assert f.count == la.la_schedule_fusion_runs(rs) + la.la_schedule_fusion_runs(ag)
        assert np.array_equal(bits(np.stack([to_host(b) for b in bufs])), bits(ref)), (algo, flags, kind)


@pytest.mark.parametrize("algo,flags,topo,n", [("ring", 0, (32, 4, 8), 1 << 20),
                                               ("lane_multiproc", la.LA_SCHED_INNER_RING, (32, 4, 8), 1 << 20),
                                               ("ring", 0, (4, 4, 1), 1 << 24),
                                               ("lane_multiproc", la.LA_SCHED_INNER_RING, (8, 4, 4), 1 << 22)])
def test_fused_launch_full_size(oracle, algo, flags, topo, n):
    """Algorithm 1 over 1024 ranks (2046 steps), the ring as inter-node stage of configs 5 and 3, and the
    ring of config 2, each as ONE launch, against the oracle at full size."""
    P = topo[0] * topo[1] * topo[2]
    x = synth.make_inputs(P, n, "uniform_pm1")
    bufs = [to_dev(x[r]) for r in range(P)]
    sched = la.la_schedule_build(la.la_topology_create(*topo), algo, n, "float32", flags)
    print("fused full size", algo, flags, topo, n, "steps", sched.num_steps, flush=True)
    with fused_launch() as f:
        la.allreduce_tensors(sched, bufs)
        torch.cuda.synchronize()
    assert f.count == 1
    got0 = to_host(bufs[0])
    for r in range(1, P):  # all ranks identical, compared on the device
        assert torch.equal(bufs[r], bufs[0]), r
    del bufs
    torch.cuda.empty_cache()
    ref = oracle.allreduce(oracle_name(algo, flags), *topo, x, in_place=True)
    assert np.array_equal(bits(got0), bits(ref[0]))


# ------------------------------------------------------------------------------ random combinations

def test_random_flag_combinations_on_the_gpu(oracle):
    """Seeded sweep: algorithm x flag subset x topology x length x type; whatever the library
    accepts must equal the oracle bit for bit, in place or out of place."""
    rng = np.random.default_rng(813397)
    pool = [la.LA_SCHED_P2P_GATHER, la.LA_SCHED_STAGED, la.LA_SCHED_INNER_RING, la.LA_SCHED_SHARED_BUFFERS,
            la.LA_SCHED_OUT_OF_PLACE, la.LA_SCHED_FUSED_GATHER, la.LA_SCHED_SINGLE_LAUNCH]
    algos = ["ring", "lane", "lane_multiproc", "recursive_doubling", "rabenseifner"]
    ran = 0
    for case in range(900):
        algo = algos[rng.integers(len(algos))]
        flags = 0
        for b in pool:
            if rng.random() < 0.3:
                flags |= b
        N, G, Q = (int(v) for v in rng.integers(1, 4, size=3))
        if algo in ("recursive_doubling", "rabenseifner"):
            N, G, Q = (int(v) for v in 2 ** rng.integers(0, 3, size=3))
        n = int(rng.choice([1, 7, 255, 4099, 40961, 150001]))
        kind = ("f32order", "bf16", "i32wrap")[case % 3]
        topo = la.la_topology_create(N, G, Q)
        try:
            sched = la.la_schedule_build(topo, algo, n, NAME[make(1, 1, kind).dtype], flags)
        except la.LaError as err:
            assert err.status in (la.LA_ERR_INVALID_ARG, la.LA_ERR_UNSUPPORTED)
            continue
        B = sched.num_buffers
        x = make(B, n, kind, seed=case)
        print("random case", case, algo, flags, (N, G, Q), n, kind, flush=True)
        if flags & la.LA_SCHED_SHARED_BUFFERS:
            name, Qo = ("lane_multiproc", 1) if algo == "lane" else (algo, Q)
            ref = oracle.allreduce(name, N, G, Qo, x, shared=True)
        else:
            ref = oracle.allreduce(oracle_name(algo, flags) if algo.startswith("lane") else algo, N, G, Q, x)
        if flags & la.LA_SCHED_OUT_OF_PLACE:
            send = [to_dev(x[r]) for r in range(B)]
            recv = [torch.full_like(send[r], 3) for r in range(B)]
            la.la_allreduce_emulated_out_of_place(sched, [t.data_ptr() for t in send], [t.data_ptr() for t in recv], n,
                                                  NAME[x.dtype], la.LA_SUM, torch.cuda.current_stream().cuda_stream)
            torch.cuda.synchronize()
            assert np.array_equal(bits(np.stack([to_host(t) for t in send])), bits(x))
            got = np.stack([to_host(t) for t in recv])
        else:
            bufs = [to_dev(x[r]) for r in range(B)]
            la.allreduce_tensors(sched, bufs)
            torch.cuda.synchronize()
            got = np.stack([to_host(t) for t in bufs])
        assert np.array_equal(bits(got), bits(ref)), (case, algo, flags, (N, G, Q), n, kind)
        ran += 1
    assert ran >= 350, ran


def test_random_knobs_views_operations_and_types_on_the_gpu(oracle):
    """Seeded sweep over what the sweep above holds fixed: all five element types, all four
    operations, buffers that are views at element offsets inside larger allocations (one common
    offset: vector path with heads and tails; independent offsets: no common 16-byte phase), and
    the launch knobs (runs fused or not, forwarding, merging, forced tile shapes and cache
    policies, graph replay).  Bit-equal to the oracle (NaN payloads aside), send buffers and the
    guard elements around every view untouched."""
    rng = np.random.default_rng(2508)
    pool = [la.LA_SCHED_P2P_GATHER, la.LA_SCHED_STAGED, la.LA_SCHED_INNER_RING, la.LA_SCHED_SHARED_BUFFERS,
            la.LA_SCHED_OUT_OF_PLACE, la.LA_SCHED_FUSED_GATHER, la.LA_SCHED_SINGLE_LAUNCH]
    algos = ["ring", "lane", "lane_multiproc", "recursive_doubling", "rabenseifner"]
    defaults = dict(fuse=-1, forward=1, merge=1, unroll=0, block=0, cache_policy=-1, graph=-1)
    GUARD = 77

    def draw(B, n, kind, op):
        if kind == "i32":
            x = rng.integers(-(1 << 31), 1 << 31, size=(B, n), dtype=np.int64).astype(np.int32)
            if op == "prod":
                x[:, ::2] = rng.integers(-5, 6, size=x[:, ::2].shape)
            return x
        if kind == "f32":
            return (rng.standard_normal((B, n)) * np.exp2(rng.integers(-30, 30, size=(B, n)))).astype(np.float32)
        if kind == "bf16":
            return oracle.bf16_round((rng.standard_normal((B, n)) * np.exp2(rng.integers(-8, 8, size=(B, n)))).astype(np.float32))
        if kind == "f16":
            return (rng.standard_normal((B, n)) * np.exp2(rng.integers(-16, 4, size=(B, n)))).astype(np.float16)
        return rng.standard_normal((B, n)) * np.exp2(rng.integers(-40, 40, size=(B, n)))

    def view(row, off):
        n = row.shape[0]
        whole = np.full(n + off + 40, GUARD, dtype=row.dtype)
        whole[off: off + n] = row
        t = to_dev(whole)
        return t, t[off: off + n]

    ran = 0
    for case in range(700):
        algo = algos[rng.integers(len(algos))]
        flags = 0
        for b in pool:
            if rng.random() < 0.25:
                flags |= b
        N, G, Q = (int(v) for v in rng.integers(1, 5, size=3))
        if algo in ("recursive_doubling", "rabenseifner"):
            N, G, Q = (int(v) for v in 2 ** rng.integers(0, 3, size=3))
        n = int(rng.choice([1, 3, 17, 255, 1000, 4099, 40961, 150001]))
        kind = ("i32", "f32", "bf16", "f16", "f64")[int(rng.integers(5))]
        op = ("sum", "sum", "prod", "max", "min")[int(rng.integers(5))]
        knobs = dict(fuse=int(rng.choice([-1, -1, 0, 1])), forward=int(rng.choice([1, 1, 0])), merge=int(rng.choice([1, 1, 0])),
                     unroll=int(rng.choice([0, 0, 1, 2, 4, 8])), block=int(rng.choice([0, 0, 256, 1024])),
                     cache_policy=int(rng.choice([-1, -1, 0, 3, 6, 7])), graph=int(rng.choice([-1, -1, 0, 1])))
        mode = int(rng.integers(4))
        name = NAME[draw(1, 1, kind, op).dtype]
        try:
            sched = la.la_schedule_build(la.la_topology_create(N, G, Q), algo, n, name, flags)
        except la.LaError as err:
            assert err.status in (la.LA_ERR_INVALID_ARG, la.LA_ERR_UNSUPPORTED)
            continue
        B = sched.num_buffers
        x = draw(B, n, kind, op)
        offs = [0] * B if mode < 2 else ([int(rng.integers(0, 33))] * B if mode == 2 else [int(v) for v in rng.integers(0, 9, size=B)])
        print("knob case", case, algo, flags, (N, G, Q), n, kind, op, knobs, offs[:4], flush=True)
        if flags & la.LA_SCHED_SHARED_BUFFERS:
            oname, Qo = ("lane_multiproc", 1) if algo == "lane" else (algo, Q)
            ref = oracle.allreduce(oname, N, G, Qo, x, shared=True, op=op)
        else:
            ref = oracle.allreduce(oracle_name(algo, flags) if algo.startswith("lane") else algo, N, G, Q, x, op=op)
        stream = torch.cuda.current_stream().cuda_stream
        try:
            for key, v in knobs.items():
                la.la_tuning_set(key, v)
            out = [view(x[r], offs[r]) for r in range(B)]
            if flags & la.LA_SCHED_OUT_OF_PLACE:
                send = out
                out = [view(np.full_like(x[r], 3), offs[r]) for r in range(B)]
                la.la_allreduce_emulated_out_of_place(sched, [v.data_ptr() for _, v in send], [v.data_ptr() for _, v in out],
                                                      n, name, la.OPS[op], stream)
                torch.cuda.synchronize()
                assert all(np.array_equal(bits(to_host(send[r][1])), bits(x[r])) for r in range(B)), "send buffers changed"
            else:
                la.la_allreduce_emulated(sched, [v.data_ptr() for _, v in out], n, name, la.OPS[op], stream)
                torch.cuda.synchronize()
        finally:
            for key, v in defaults.items():
                la.la_tuning_set(key, v)
        got = np.stack([to_host(v) for _, v in out])
        for r in range(B):
            w = to_host(out[r][0])
            assert np.all(w[: offs[r]] == GUARD) and np.all(w[offs[r] + n:] == GUARD), ("guard elements written", case, r)
        u = {2: np.uint16, 4: np.uint32, 8: np.uint64}[x.dtype.itemsize]
        if x.dtype == np.uint16:
            nan_ref, nan_got = ((ref & 0x7f80) == 0x7f80) & ((ref & 0x7f) != 0), ((got & 0x7f80) == 0x7f80) & ((got & 0x7f) != 0)
        elif x.dtype != np.int32:
            nan_ref, nan_got = np.isnan(ref), np.isnan(got)
        else:
            nan_ref = nan_got = np.zeros(ref.shape, bool)
        assert np.array_equal(nan_got, nan_ref), (case, "NaN pattern")
        assert np.array_equal(got.view(u)[~nan_ref], ref.view(u)[~nan_ref]), (case, algo, flags, (N, G, Q), n, kind, op, knobs)
        ran += 1
    assert ran >= 250, ran


# ------------------------------------------------------------------------------ full-size configs

def full_size_case(oracle, topo, algo, n, dist, flags=la.LA_SCHED_DEFAULT, tol=True):
    N, G, Q = topo
    P = N * G * Q
    x = synth.make_inputs(P, n, dist, workers=16)
    t = la.la_topology_create(N, G, Q)
    sched = la.la_schedule_build(t, algo, n, NAME[x.dtype], flags)
    bufs = [to_dev(x[r]) for r in range(P)]
    la.allreduce_tensors(sched, bufs)
    torch.cuda.synchronize()
    got0 = to_host(bufs[0])
    for r in range(1, P):  # every rank ends with the same bits
        assert torch.equal(bufs[r].view(torch.int16 if x.dtype == np.uint16 else torch.int32),
                           bufs[0].view(torch.int16 if x.dtype == np.uint16 else torch.int32)), r
    del bufs
    torch.cuda.empty_cache()
    if tol:
        # sampled columns against the definition
        idx = np.unique(np.concatenate([np.arange(0, 4096), np.arange(n - 4096, n),
                                        np.random.default_rng(1).integers(0, n, 200000)]))
        check_tolerance(oracle, np.ascontiguousarray(x[:, idx]), got0[idx])
    oracle.set_threads(min(16, oracle.max_threads()))
    ref = oracle.allreduce(oracle_name(algo, flags), N, G, Q, x, in_place=True)
    assert np.array_equal(bits(got0), bits(ref[0]))
    assert np.array_equal(bits(ref[P - 1]), bits(ref[0]))


@pytest.mark.parametrize("algo,topo", [("lane", (2, 1, 1)), ("ring", (1, 2, 1)), ("lane_multiproc", (1, 1, 2))])
def test_buffers_beyond_4_GiB_use_64_bit_offsets(oracle, algo, topo):
    """More than 2^32 bytes per rank buffer: segment offsets, tile offsets and lengths must not
    pass through 32 bits anywhere (int32 data, wrapping sums: bit-exact against the oracle)."""
    n = (1 << 30) + 12345
    x = np.empty((2, n), dtype=np.int32)
    base = np.arange(n, dtype=np.uint32)
    np.multiply(base, np.uint32(2654435761), out=x[0].view(np.uint32))
    np.multiply(base, np.uint32(40503), out=x[1].view(np.uint32))
    x[1] += 7
    del base
    sched = la.la_schedule_build(la.la_topology_create(*topo), algo, n, "int32")
    bufs = [to_dev(x[r]) for r in range(2)]
    la.allreduce_tensors(sched, bufs)
    torch.cuda.synchronize()
    assert torch.equal(bufs[0], bufs[1])
    got0 = to_host(bufs[0])
    del bufs
    torch.cuda.empty_cache()
    want = (x[0].view(np.uint32) + x[1].view(np.uint32)).view(np.int32)   # two operands: the definition itself
    assert np.array_equal(got0, want)
    ref = oracle.allreduce(algo, *topo, x, in_place=True)
    assert np.array_equal(got0, ref[0]) and np.array_equal(ref[1], ref[0])


def test_config2_lane_16_ranks_16Mi_fp32(oracle):
    full_size_case(oracle, (4, 4, 1), "lane", 1 << 24, "normal")


def test_config2_ring_16_ranks_16Mi_fp32(oracle):
    full_size_case(oracle, (4, 4, 1), "ring", 1 << 24, "normal")


def test_config3_lane_multiproc_128_ranks_4Mi_fp32(oracle):
    full_size_case(oracle, (8, 4, 4), "lane_multiproc", 1 << 22, "uniform_pm1")


def test_config4_gradient_bucket_bf16_128Mi(oracle):
    full_size_case(oracle, (2, 4, 2), "lane_multiproc", 1 << 27, "normal_bf16")


def test_config4_lane_leader_owned_bf16_128Mi(oracle):
    full_size_case(oracle, (2, 4, 2), "lane", 1 << 27, "normal_bf16")


def test_config5_scale_out_1024_ranks_1Mi_fp32(oracle):
    topo = (32, 4, 8)
    sched = la.la_schedule_build(la.la_topology_create(*topo), "lane_multiproc", 1 << 20, "float32")
    shape = [(s["stage_name"], s["num_segments"], s["fan_in"], s["fan_out"]) for s in sched.steps()]
    assert shape == [("S1", 1024, 32, 1), ("S2", 1024, 32, 32), ("S3", 1024, 1, 31)]
    full_size_case(oracle, topo, "lane_multiproc", 1 << 20, "uniform_pm1")


def test_config3_inner_ring(oracle):
    full_size_case(oracle, (8, 4, 4), "lane_multiproc", 1 << 22, "uniform_pm1", flags=la.LA_SCHED_INNER_RING)


def test_config5_scale_out_inner_ring(oracle):
    full_size_case(oracle, (32, 4, 8), "lane_multiproc", 1 << 20, "uniform_pm1", flags=la.LA_SCHED_INNER_RING)


def test_config2_fused_gather(oracle):
    full_size_case(oracle, (4, 4, 1), "lane", 1 << 24, "normal", flags=la.LA_SCHED_FUSED_GATHER)


def test_config4_fused_gather(oracle):
    full_size_case(oracle, (2, 4, 2), "lane_multiproc", 1 << 27, "normal_bf16", flags=la.LA_SCHED_FUSED_GATHER)


def test_config5_fused_gather_fan_out_1024(oracle):
    full_size_case(oracle, (32, 4, 8), "lane_multiproc", 1 << 20, "uniform_pm1", flags=la.LA_SCHED_FUSED_GATHER, tol=False)


def test_config2_single_launch(oracle):
    full_size_case(oracle, (4, 4, 1), "lane", 1 << 24, "normal", flags=la.LA_SCHED_SINGLE_LAUNCH)


def test_config4_single_launch_bf16_two_roundings(oracle):
    full_size_case(oracle, (2, 4, 2), "lane_multiproc", 1 << 27, "normal_bf16", flags=la.LA_SCHED_SINGLE_LAUNCH)


def test_config3_single_launch(oracle):
    full_size_case(oracle, (8, 4, 4), "lane_multiproc", 1 << 22, "uniform_pm1", flags=la.LA_SCHED_SINGLE_LAUNCH)


def test_config5_single_launch_fan_in_and_out_1024(oracle):
    full_size_case(oracle, (32, 4, 8), "lane_multiproc", 1 << 20, "uniform_pm1", flags=la.LA_SCHED_SINGLE_LAUNCH, tol=False)


def test_config5_scale_out_point_to_point_gather(oracle):
    full_size_case(oracle, (32, 4, 8), "lane_multiproc", 1 << 20, "uniform_pm1", flags=la.LA_SCHED_P2P_GATHER, tol=False)
