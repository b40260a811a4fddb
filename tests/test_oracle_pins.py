"""Pins for the CPU oracle: every function of oracle/la_oracle.c is checked against something
other than itself -- the definition computed with Python integers / math.fsum, IEEE closed
forms, library routines (numpy.array_split, torch's bf16 conversion), the index walk that
Algorithm 1 prescribes, the stage boundaries of Algorithm 2, hand-worked order-sensitive
cases (tests/golden/), and brute force over tiny topologies."""
import itertools
import math
import os

import numpy as np
import pytest

from paper_2508_13397_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
ALGOS = ("ring", "lane", "lane_multiproc", "lane_ring", "lane_multiproc_ring")
TOL = {np.dtype(np.float32): 1e-5, np.dtype(np.uint16): 8e-3}


def exact_int_sum(x):
    """column sums with Python integers, wrapped to int32"""
    out = []
    for i in range(x.shape[1]):
        s = sum(int(v) for v in x[:, i])
        s &= 0xFFFFFFFF
        out.append(s - (1 << 32) if s >= (1 << 31) else s)
    return np.array(out, dtype=np.int32)


def bf16_bits_to_f64(h):
    return (h.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


# --------------------------------------------------------------------------- split

def test_part_is_numpy_array_split(oracle):
    for length in range(0, 45):
        for m in range(1, 10):
            ref = np.array_split(np.arange(length), m)
            pos = 0
            for i in range(m):
                off, cnt = oracle.part(length, m, i)
                assert cnt == len(ref[i]) and off == pos
                pos += cnt
            assert pos == length


# --------------------------------------------------------------------------- bf16

def test_bf16_round_matches_torch_on_random_bit_patterns(oracle):
    import torch

    rng = np.random.default_rng(7)
    bits = rng.integers(0, 1 << 32, size=400000, dtype=np.uint64).astype(np.uint32)
    # make sure exact ties, near-ties, denormals, infinities and the largest finite are present
    special = np.array([0x3F808000, 0x3F818000, 0x3F808001, 0x3F807FFF, 0x7F7FFFFF, 0xFF7FFFFF,
                        0x7F800000, 0xFF800000, 0x00000001, 0x00008000, 0x00018000, 0x80008000,
                        0x007FFFFF, 0x00000000, 0x80000000, 0x7F7F8000, 0x7F7F7FFF], dtype=np.uint32)
    ties = (rng.integers(0, 1 << 16, size=5000, dtype=np.uint64).astype(np.uint32) << 16) | 0x8000
    bits = np.concatenate([bits, special, ties])
    x = bits.view(np.float32)
    got = oracle.bf16_round(x)
    ref = torch.from_numpy(x.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    nan = np.isnan(x)
    assert np.array_equal(got[~nan], ref[~nan])
    # NaN in, NaN out (payload free)
    back = (got[nan].astype(np.uint32) << 16).view(np.float32)
    assert np.all(np.isnan(back))


def test_bf16_round_closed_forms(oracle):
    # bf16 keeps 8 significant bits: ulp(1) = 2^-7, so 1 + 2^-8 is an exact tie
    cases = {
        1.0: 0x3F80,
        1.0 + 2.0 ** -8: 0x3F80,                 # tie, 0x3F80 is even
        1.0 + 2.0 ** -7 + 2.0 ** -8: 0x3F82,     # tie, 0x3F81 is odd -> up
        1.0 + 2.0 ** -8 + 2.0 ** -20: 0x3F81,    # just above half
        1.0 + 2.0 ** -8 - 2.0 ** -20: 0x3F80,    # just below half
        -2.5: 0xC020,
        float(np.finfo(np.float32).max): 0x7F80,  # rounds up to +inf
        0.0: 0x0000,
    }
    x = np.array(list(cases.keys()), dtype=np.float32)
    assert [int(v) for v in oracle.bf16_round(x)] == list(cases.values())


def test_bf16_widen_all_patterns(oracle):
    import torch

    h = np.arange(1 << 16, dtype=np.uint16)
    got = oracle.bf16_widen(h).view(np.uint32)
    ref = torch.from_numpy(h.view(np.int16).copy()).view(torch.bfloat16).to(torch.float32).numpy().view(np.uint32)
    nan = np.isnan(ref.view(np.float32))
    assert np.array_equal(got[~nan], ref[~nan])
    assert np.array_equal(got, h.astype(np.uint32) << 16)


def test_f16_round_matches_numpy(oracle):
    rng = np.random.default_rng(9)
    bits = rng.integers(0, 1 << 32, size=600000, dtype=np.uint64).astype(np.uint32)
    # dense coverage of the binary16 range: normals, subnormals (below 2^-14), ties, overflow
    mags = np.exp2(rng.uniform(-27, 17, size=400000)).astype(np.float32) * rng.choice([-1.0, 1.0], size=400000).astype(np.float32)
    ties = (np.arange(0, 1 << 16, dtype=np.uint32).view(np.uint32))
    halves = ties.astype(np.uint16).view(np.float16).astype(np.float32)
    halves = halves[np.isfinite(halves)]
    with np.errstate(over="ignore"):
        mid = (halves + np.nextafter(halves.astype(np.float16), np.float16(np.inf)).astype(np.float32)) / np.float32(2)  # exact midpoints
    special = np.array([65504.0, 65519.99, 65520.0, 65536.0, 1e9, 2.0 ** -24, 2.0 ** -25, 2.0 ** -25 * 1.0000001, 2.0 ** -26,
                        2.0 ** -14, 2.0 ** -14 * (1 - 2.0 ** -12), 0.0, -0.0, np.inf, -np.inf], dtype=np.float32)
    x = np.concatenate([bits.view(np.float32), mags, mid[np.isfinite(mid)], special])
    got = oracle.f16_round(x)
    with np.errstate(over="ignore"):
        ref = x.astype(np.float16).view(np.uint16)
    nan = np.isnan(x)
    assert np.array_equal(got[~nan], ref[~nan])
    assert np.all(np.isnan(got[nan].view(np.float16)))


def test_f16_widen_all_patterns(oracle):
    h = np.arange(1 << 16, dtype=np.uint16)
    got = oracle.f16_widen(h)
    ref = h.view(np.float16).astype(np.float32)
    ok = ~np.isnan(ref)
    assert np.array_equal(got.view(np.uint32)[ok], ref.view(np.uint32)[ok])
    assert np.all(np.isnan(got[~ok]))


# --------------------------------------------------------------------------- the definition

def test_definition_int32_vs_python_integers_with_wrap(oracle):
    rng = np.random.default_rng(3)
    x = rng.integers(-(1 << 31), 1 << 31, size=(7, 50), dtype=np.int64).astype(np.int32)
    assert np.array_equal(oracle.definition_sum(x), exact_int_sum(x))
    y = np.full((3, 4), 2147483647, dtype=np.int32)  # 3 * INT_MAX wraps to INT_MAX - 2
    assert np.array_equal(oracle.definition_sum(y), np.full(4, 2147483645, dtype=np.int32))


def test_definition_float_vs_fsum(oracle):
    x = synth.make_inputs(12, 64, "normal")
    got = oracle.definition_sum(x)
    ref = np.array([math.fsum(float(v) for v in x[:, i]) for i in range(x.shape[1])])
    assert np.allclose(got, ref, rtol=0, atol=1e-13 * np.abs(x).sum(axis=0).max())
    h = synth.make_inputs(12, 64, "normal_bf16")
    got = oracle.definition_sum(h)
    w = bf16_bits_to_f64(h)
    ref = np.array([math.fsum(w[:, i]) for i in range(w.shape[1])])
    assert np.allclose(got, ref, rtol=0, atol=1e-13)


def py_int_reduce(x, op):
    out = []
    for i in range(x.shape[1]):
        col = [int(v) for v in x[:, i]]
        if op == "sum":
            s = sum(col)
        elif op == "prod":
            s = 1
            for v in col:
                s *= v
        else:
            s = max(col) if op == "max" else min(col)
        s &= 0xFFFFFFFF
        out.append(s - (1 << 32) if s >= (1 << 31) else s)
    return np.array(out, dtype=np.int32)


def test_definition_of_operations_vs_python(oracle):
    rng = np.random.default_rng(21)
    x = rng.integers(-(1 << 31), 1 << 31, size=(6, 40), dtype=np.int64).astype(np.int32)
    x[:, :10] = rng.integers(-9, 10, size=(6, 10))
    for op in ("sum", "prod", "max", "min"):
        assert np.array_equal(oracle.definition_reduce(x, op), py_int_reduce(x, op)), op
    f = synth.make_inputs(7, 33, "normal")
    assert np.allclose(oracle.definition_reduce(f, "prod"), [math.prod(float(v) for v in f[:, i]) for i in range(33)], rtol=1e-14)
    assert np.array_equal(oracle.definition_reduce(f, "max"), f.astype(np.float64).max(axis=0))
    assert np.array_equal(oracle.definition_reduce(f, "min"), f.astype(np.float64).min(axis=0))
    d = np.random.default_rng(2).standard_normal((5, 20))
    assert np.allclose(oracle.definition_reduce(d, "sum"), [math.fsum(d[:, i]) for i in range(20)], rtol=0, atol=1e-15 * 5)
    h = np.random.default_rng(3).standard_normal((5, 20)).astype(np.float16)
    assert np.allclose(oracle.definition_reduce(h, "sum"), [math.fsum(float(v) for v in h[:, i]) for i in range(20)], rtol=0, atol=1e-14)


def test_operations_closed_forms(oracle):
    nan, pz, nz = np.float32(np.nan), np.float32(0.0), np.float32(-0.0)
    # columns: (+0,-0), (-0,+0), (nan,1), (1,nan), (nan,nan), (2,3), (-inf, 5)
    a = np.array([pz, nz, nan, 1.0, nan, 2.0, -np.inf], dtype=np.float32)
    b = np.array([nz, pz, 1.0, nan, nan, 3.0, 5.0], dtype=np.float32)
    x = np.stack([a, b])
    for algo in ("ring", "lane"):
        mx = oracle.allreduce(algo, 2, 1, 1, x, op="max")[0]
        mn = oracle.allreduce(algo, 2, 1, 1, x, op="min")[0]
        assert [int(v) for v in mx[:2].view(np.uint32)] == [0x00000000, 0x00000000]      # +0 is the larger zero
        assert [int(v) for v in mn[:2].view(np.uint32)] == [0x80000000, 0x80000000]      # -0 the smaller
        assert mx[2] == 1.0 and mx[3] == 1.0 and mn[2] == 1.0 and mn[3] == 1.0          # a NaN loses against a number
        assert np.isnan(mx[4]) and np.isnan(mn[4])
        assert (mx[5], mn[5], mx[6], mn[6]) == (3.0, 2.0, 5.0, -np.inf)
    i = np.array([[-5, 7, -2147483648, 65536], [3, -7, 2147483647, 65536]], dtype=np.int32)
    assert list(oracle.allreduce("lane", 1, 2, 1, i, op="max")[0]) == [3, 7, 2147483647, 65536]
    assert list(oracle.allreduce("lane", 1, 2, 1, i, op="min")[0]) == [-5, -7, -2147483648, 65536]
    assert list(oracle.allreduce("lane", 1, 2, 1, i, op="prod")[0]) == [-15, -49, -2147483648, 0]  # 2^32 wraps to 0


def test_f16_rounds_once_per_reduce_step(oracle):
    # binary16 has 11 significant bits: ulp(1) = 2^-10, so 1 + 2^-11 is an exact tie
    vals3 = np.array([1.0, 2.0 ** -11, 2.0 ** -11], dtype=np.float16)
    x3 = np.repeat(vals3[:, None], 3, axis=1)
    one = oracle.allreduce("lane", 1, 3, 1, x3)          # one 3-way step: fp32 sum 1 + 2^-10, exact
    assert np.all(one.view(np.uint16) == 0x3C01)
    ring = oracle.allreduce("ring", 3, 1, 1, x3)          # rounds after every hop
    # chunk 0: rnd(rnd(1 + 2^-11) + 2^-11) = 1; chunk 1: rnd(rnd(2^-11 + 2^-11) + 1) = 1 + 2^-10; chunk 2: like chunk 0
    assert [int(v) for v in ring[0].view(np.uint16)] == [0x3C00, 0x3C01, 0x3C00]


@pytest.mark.parametrize("algo", ["ring", "lane_multiproc"])
def test_schedules_with_operations_and_wide_types(oracle, algo):
    rng = np.random.default_rng(33)
    for (N, G, Q) in [(2, 2, 2), (3, 1, 2), (1, 3, 1), (2, 3, 1)]:
        P = N * G * Q
        for n in (1, 7, 24, 40):
            xi = rng.integers(-(1 << 31), 1 << 31, size=(P, n), dtype=np.int64).astype(np.int32)
            xi[:, : n // 2] = rng.integers(-6, 7, size=(P, n // 2))
            for op in ("prod", "max", "min"):
                out = oracle.allreduce(algo, N, G, Q, xi, op=op)
                assert np.array_equal(out, np.broadcast_to(py_int_reduce(xi, op), out.shape)), (algo, op, N, G, Q, n)
            f = synth.make_inputs(P, n, "uniform_pm1", seed=n) + np.float32(1.5)   # in [0.5, 2.5): products stay in range
            for op in ("max", "min"):
                out = oracle.allreduce(algo, N, G, Q, f, op=op)
                assert np.array_equal(out[P - 1].astype(np.float64), oracle.definition_reduce(f, op))
            pr = oracle.allreduce(algo, N, G, Q, f, op="prod")[0].astype(np.float64)
            assert np.allclose(pr, oracle.definition_reduce(f, "prod"), rtol=1e-5, atol=0)
            d = rng.standard_normal((P, n))
            got = oracle.allreduce(algo, N, G, Q, d)
            exact = np.array([math.fsum(d[:, i]) for i in range(n)])
            assert np.all(np.abs(got[0] - exact) <= 1e-14 * np.abs(d).sum(axis=0))
            h = rng.standard_normal((P, n)).astype(np.float16)
            goth = oracle.allreduce(algo, N, G, Q, h)
            assert all(np.array_equal(goth[0].view(np.uint16), goth[r].view(np.uint16)) for r in range(P))
            if algo != "ring":  # two roundings of 2^-11 each
                hx = h.astype(np.float64)
                exact = np.array([math.fsum(hx[:, i]) for i in range(n)])
                assert np.all(np.abs(goth[0].astype(np.float64) - exact) <= 2e-3 * np.abs(hx).sum(axis=0))


# --------------------------------------------------------------------------- brute force

TOPOS = list(itertools.product((1, 2, 3), repeat=3))


@pytest.mark.parametrize("algo", ALGOS)
def test_bruteforce_int32_every_small_topology(oracle, algo):
    rng = np.random.default_rng(11)
    for (N, G, Q) in TOPOS:
        P = N * G * Q
        for n in list(range(1, 41)):
            x = rng.integers(-1000, 1001, size=(P, n), dtype=np.int32)
            if n % 7 == 0:  # exercise the wrap as well
                x = rng.integers(-(1 << 31), 1 << 31, size=(P, n), dtype=np.int64).astype(np.int32)
            out = oracle.allreduce(algo, N, G, Q, x)
            ref = exact_int_sum(x) if n <= 8 else x.astype(np.int64).sum(axis=0).astype(np.uint64).astype(np.uint32).view(np.int32)
            assert np.array_equal(out, np.broadcast_to(ref, out.shape)), (algo, N, G, Q, n)


@pytest.mark.parametrize("algo", ALGOS)
@pytest.mark.parametrize("dist", ["uniform_pm1", "normal_bf16"])
def test_bruteforce_floats_within_bound_and_all_ranks_identical(oracle, algo, dist):
    for (N, G, Q) in TOPOS:
        P = N * G * Q
        for n in (1, 2, 3, 5, 8, 13, 27, 40):
            x = synth.make_inputs(P, n, dist, seed=synth.BASE_SEED + 1000 * n)
            out = oracle.allreduce(algo, N, G, Q, x)
            assert all(np.array_equal(out[0], out[r]) for r in range(P)), (algo, N, G, Q, n)
            if x.dtype == np.uint16:
                xs, got = bf16_bits_to_f64(x), bf16_bits_to_f64(out[0])
                if "ring" in algo:
                    continue  # a ring rounds once per hop: only the bitwise parity is gated there
            else:
                xs, got = x.astype(np.float64), out[0].astype(np.float64)
            exact = np.array([math.fsum(xs[:, i]) for i in range(n)])
            bound = TOL[x.dtype] * np.abs(xs).sum(axis=0)
            assert np.all(np.abs(got - exact) <= bound), (algo, N, G, Q, n)


# --------------------------------------------------------------------------- special cases

@pytest.mark.parametrize("algo", ALGOS)
@pytest.mark.parametrize("topo", [(2, 1, 1), (1, 2, 1), (1, 1, 2)])
def test_two_ranks_is_one_ieee_add(oracle, algo, topo):
    x = synth.make_inputs(2, 257, "normal")
    out = oracle.allreduce(algo, *topo, x)
    ref = x[0] + x[1]  # numpy float32 add
    assert np.array_equal(out[0].view(np.uint32), ref.view(np.uint32))
    assert np.array_equal(out[1].view(np.uint32), ref.view(np.uint32))


@pytest.mark.parametrize("algo", ALGOS)
def test_single_rank_is_identity(oracle, algo):
    x = synth.make_inputs(1, 33, "normal")
    assert np.array_equal(oracle.allreduce(algo, 1, 1, 1, x), x)


def test_lane_equals_lane_multiproc_when_one_process_per_gpu(oracle):
    x = synth.order_sensitive_f32(12, 50)
    a, ta = oracle.allreduce("lane", 3, 4, 1, x, want_trace=True)
    b, tb = oracle.allreduce("lane_multiproc", 3, 4, 1, x, want_trace=True)
    assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    assert np.array_equal(ta, tb)


def test_single_node_has_no_inter_node_messages(oracle):
    x = synth.make_inputs(6, 31, "int_pm1000")
    out, tr = oracle.allreduce("lane_multiproc", 1, 3, 2, x, want_trace=True)
    assert np.array_equal(out[0], exact_int_sum(x))
    assert not np.any((tr["phase"] == oracle.PH_LANE_S2A) | (tr["phase"] == oracle.PH_LANE_S2B))


def test_one_gpu_one_proc_is_pure_inter_node(oracle):
    x = synth.make_inputs(5, 23, "int_pm1000")
    out, tr = oracle.allreduce("lane", 5, 1, 1, x, want_trace=True)
    assert np.array_equal(out[3], exact_int_sum(x))
    assert not np.any((tr["phase"] == oracle.PH_LANE_S1) | (tr["phase"] == oracle.PH_LANE_S3))


# --------------------------------------------------------------------------- summation order

def f32_sum_in_order(x, order):
    """left-to-right float32 sum of column vectors x[order[0]], x[order[1]], ... (numpy adds)"""
    acc = x[order[0]].copy()
    for r in order[1:]:
        acc = acc + x[r]
    return acc


def test_ring_order_is_chunk_owner_first_then_successors(oracle):
    # Algorithm 1: chunk c starts at rank c (sp = r) and walks to r+1, r+2, ...; each receiver adds
    # the incoming partial sum to its own copy.
    P, per = 5, 6
    x = synth.order_sensitive_f32(P, P * per)
    out = oracle.allreduce("ring", 5, 1, 1, x)
    for c in range(P):
        sl = slice(c * per, (c + 1) * per)
        ref = f32_sum_in_order(x[:, sl], [(c + t) % P for t in range(P)])
        assert np.array_equal(out[2, sl].view(np.uint32), ref.view(np.uint32))
    # the data does tell orders apart: the reverse walk gives other bits somewhere
    rev = np.concatenate([f32_sum_in_order(x[:, c * per:(c + 1) * per], [(c - t) % P for t in range(P)])
                          for c in range(P)])
    assert not np.array_equal(rev.view(np.uint32), out[0].view(np.uint32))


def test_lane_order_is_node_sums_then_across_nodes(oracle):
    N, G, Q = 3, 2, 2
    R, P = G * Q, N * G * Q
    n = R * N * 4  # every part and piece has 4 elements
    x = synth.order_sensitive_f32(P, n)
    out = oracle.allreduce("lane_multiproc", N, G, Q, x)
    node_sums = [f32_sum_in_order(x, [v * R + l for l in range(R)]) for v in range(N)]
    ref = node_sums[0]
    for v in range(1, N):
        ref = ref + node_sums[v]
    assert np.array_equal(out[7].view(np.uint32), ref.view(np.uint32))
    flat = f32_sum_in_order(x, list(range(P)))
    assert not np.array_equal(flat.view(np.uint32), ref.view(np.uint32))


def load_golden(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                rows.append([float(t) for t in line.split()])
    return rows


def test_golden_ring_three_ranks_cancellation(oracle):
    rows = load_golden("ring_p3_cancellation.txt")
    x = np.array(rows[:3], dtype=np.float32)
    expect = np.array(rows[3], dtype=np.float32)
    out = oracle.allreduce("ring", 3, 1, 1, x)
    for r in range(3):
        assert np.array_equal(out[r], expect)


def test_golden_lane_two_by_two_cancellation(oracle):
    rows = load_golden("lane_2x2_cancellation.txt")
    x = np.array(rows[:4], dtype=np.float32)
    expect = np.array(rows[4], dtype=np.float32)
    for algo in ("lane", "lane_multiproc"):
        out = oracle.allreduce(algo, 2, 2, 1, x)
        for r in range(4):
            assert np.array_equal(out[r], expect)


def test_bf16_rounds_once_per_reduce_step(oracle):
    # lane, 2 nodes x 2 GPUs: S1 adds two operands in fp32 and rounds, S2a adds two of those and
    # rounds: for one element in lane 0, piece 0:  rnd(rnd(a+b) + rnd(c+d))
    vals = np.array([1.0, 2.0 ** -8, 1.0, 3 * 2.0 ** -8], dtype=np.float32)  # exact in bf16
    x = np.repeat(synth.to_bf16_bits(vals)[:, None], 4, axis=1)
    out = oracle.allreduce("lane", 2, 2, 1, x)
    # node 0: 1 + 2^-8 -> tie -> 1.0 ; node 1: 1 + 3*2^-8 = 1 + 2^-7 + 2^-8 -> tie -> 1 + 2^-6
    # across nodes: 2 + 2^-6 is exact in bf16 (ulp(2) = 2^-6): 0x4001
    assert np.all(out == 0x4001)
    # a single fp32 accumulation rounded once would give 2 + 2^-6 as well only by luck; check a
    # case where it differs: k-way S1 with 3 operands rounds once, not twice
    vals3 = np.array([1.0, 2.0 ** -8, 2.0 ** -8], dtype=np.float32)
    x3 = np.repeat(synth.to_bf16_bits(vals3)[:, None], 3, axis=1)
    out3 = oracle.allreduce("lane", 1, 3, 1, x3)
    # fp32: 1 + 2^-8 + 2^-8 = 1 + 2^-7 exactly -> 0x3F81; pairwise rounding would give 1.0
    assert np.all(out3 == 0x3F81)
    ring3 = oracle.allreduce("ring", 3, 1, 1, x3)
    # ring rounds after every step. chunk 0: rnd(rnd(1 + 2^-8) + 2^-8) = 1.0;
    # chunk 1: rnd(rnd(2^-8 + 2^-8) + 1) = rnd(2^-7 + 1) = 0x3F81; chunk 2: rnd(rnd(2^-8+1) + 2^-8) = 1.0
    assert list(ring3[0]) == [0x3F80, 0x3F81, 0x3F80]


# --------------------------------------------------------------------------- Algorithm 1 walk

def test_ring_message_pattern(oracle):
    N, G, Q = 2, 4, 1
    P, n = 8, 64
    x = synth.make_inputs(P, n, "int_pm1000")
    out, tr = oracle.allreduce("ring", N, G, Q, x, want_trace=True)
    assert len(tr) == 2 * (P - 1) * P
    for r in range(P):
        mine = tr[tr["src"] == r]
        assert len(mine) == 2 * (P - 1)                    # 2(p-1) messages per process
        assert np.all(mine["dst"] == (r + 1) % P)          # only to the next process in the ring
        assert np.all(mine["cnt"] == n // P)               # a 1/P fraction each
    rs0 = tr[(tr["phase"] == oracle.PH_RING_RS) & (tr["step"] == 0)]
    assert np.array_equal(rs0["off"], rs0["src"].astype(np.uint64) * (n // P))          # sp = r
    ag0 = tr[(tr["phase"] == oracle.PH_RING_AG) & (tr["step"] == P - 1)]
    assert np.array_equal(ag0["off"], ((ag0["src"] + 1) % P).astype(np.uint64) * (n // P))  # sp = r+1
    # sp decreases by one chunk per step
    r3 = tr[(tr["src"] == 3) & (tr["phase"] == oracle.PH_RING_RS)]
    assert [int(o) // (n // P) for o in r3["off"]] == [(3 - i) % P for i in range(P - 1)]
    # four processes per node: two of them talk only inside the node, two have an off-node partner
    for node in range(N):
        off_node = set()
        for m in tr:
            if m["src"] // 4 != m["dst"] // 4:
                for r in (int(m["src"]), int(m["dst"])):
                    if r // 4 == node:
                        off_node.add(r)
        assert len(off_node) == 2


def test_ring_after_first_loop_rank_owns_next_chunk(oracle):
    P, n = 6, 30
    x = synth.make_inputs(P, n, "int_pm1000")
    mid = oracle.allreduce("ring", 3, 2, 1, x, max_rounds=P - 1)
    total = exact_int_sum(x)
    per = n // P
    for r in range(P):
        c = (r + 1) % P
        assert np.array_equal(mid[r, c * per:(c + 1) * per], total[c * per:(c + 1) * per])
        # the chunk it started sending is still untouched
        assert np.array_equal(mid[r, r * per:(r + 1) * per], x[r, r * per:(r + 1) * per])


# --------------------------------------------------------------------------- Algorithm 2 stages

@pytest.mark.parametrize("algo", ["lane", "lane_multiproc"])
def test_lane_stage_boundaries(oracle, algo):
    N, G, Q = 2, 2, 3
    R, P = G * Q, N * G * Q
    J = R if algo == "lane_multiproc" else G
    n = J * N * 5
    c, piece = n // J, n // J // N
    x = synth.make_inputs(P, n, "int_pm1000")
    total = exact_int_sum(x)
    owner_local = (lambda j: j) if algo == "lane_multiproc" else (lambda j: j * Q)

    s1 = oracle.allreduce(algo, N, G, Q, x, max_rounds=1)
    s2a = oracle.allreduce(algo, N, G, Q, x, max_rounds=2)
    s2b = oracle.allreduce(algo, N, G, Q, x, max_rounds=3)
    s3 = oracle.allreduce(algo, N, G, Q, x, max_rounds=4)
    full = oracle.allreduce(algo, N, G, Q, x)
    assert np.array_equal(s3, full)
    for node in range(N):
        node_sum = x[node * R:(node + 1) * R].astype(np.int64).sum(axis=0).astype(np.int32)
        for l in range(R):
            r = node * R + l
            for j in range(J):
                sl = slice(j * c, (j + 1) * c)
                if owner_local(j) == l:
                    # stage 1 leaves the node's partial sum at offset j * c of the owner
                    assert np.array_equal(s1[r, sl], node_sum[sl])
                    # stage 2a: only the owner's own piece (index = node) is complete
                    mine = slice(j * c + node * piece, j * c + (node + 1) * piece)
                    assert np.array_equal(s2a[r, mine], total[mine])
                    other = slice(j * c + (1 - node) * piece, j * c + (2 - node) * piece)
                    assert np.array_equal(s2a[r, other], node_sum[other])
                    assert np.array_equal(s2b[r, sl], total[sl])
                else:
                    for st in (s1, s2a, s2b):
                        assert np.array_equal(st[r, sl], x[r, sl])
    assert np.array_equal(full, np.broadcast_to(total, full.shape))


def test_lane_message_shapes(oracle):
    N, G, Q = 4, 2, 2
    R, P = G * Q, N * G * Q
    n = R * N * 3
    x = synth.make_inputs(P, n, "int_pm1000")
    _, tr = oracle.allreduce("lane_multiproc", N, G, Q, x, want_trace=True)
    node = lambda r: r // R
    for ph, same_node, cnt in ((oracle.PH_LANE_S1, True, n // R), (oracle.PH_LANE_S2A, False, n // R // N),
                               (oracle.PH_LANE_S2B, False, n // R // N), (oracle.PH_LANE_S3, True, n // R)):
        t = tr[tr["phase"] == ph]
        assert len(t) > 0 and np.all(t["cnt"] == cnt)
        assert np.all((node(t["src"]) == node(t["dst"])) == same_node)
    # inter-node partners are the corresponding processes of the other nodes (same local index),
    # and a process only ever moves inter-node data inside its own sub-chunk
    t = tr[(tr["phase"] == oracle.PH_LANE_S2A) | (tr["phase"] == oracle.PH_LANE_S2B)]
    assert np.all(t["src"] % R == t["dst"] % R)
    j = (t["src"] % R).astype(np.uint64)
    assert np.all((t["off"] >= j * (n // R)) & (t["off"] + t["cnt"] <= (j + 1) * (n // R)))
    # the inter-node message is the buffer divided by (processes per node * nodes)
    assert n // R // N == n // (G * Q) // N
    # without the per-process split the leader's inter-node message is Q times larger
    _, tl = oracle.allreduce("lane", N, G, Q, x, want_trace=True)
    t2 = tl[tl["phase"] == oracle.PH_LANE_S2A]
    assert np.all(t2["cnt"] == n // G // N) and np.all(t2["src"] % Q == 0)


# --------------------------------------------------------------------------- ring inside the lane stage

def test_lane_ring_is_the_flat_ring_when_every_node_has_one_rank(oracle):
    x = synth.order_sensitive_f32(5, 37)
    a, ta = oracle.allreduce("ring", 5, 1, 1, x, want_trace=True)
    for algo in ("lane_ring", "lane_multiproc_ring"):
        b, tb = oracle.allreduce(algo, 5, 1, 1, x, want_trace=True)
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
        for key in ("src", "dst", "off", "cnt"):
            assert np.array_equal(ta[key], tb[key])


def test_lane_ring_order_node_sums_walk_the_ring(oracle):
    N, G, Q = 4, 2, 1
    R, P = G * Q, N * G * Q
    per = 3
    n = G * N * per  # every piece has `per` elements
    x = synth.order_sensitive_f32(P, n)
    out = oracle.allreduce("lane_ring", N, G, Q, x)
    node_sums = [f32_sum_in_order(x, [v * R + l for l in range(R)]) for v in range(N)]
    for j in range(G):
        for c in range(N):  # piece c of part j starts at member c and walks to c+1, c+2, ...
            sl = slice(j * N * per + c * per, j * N * per + (c + 1) * per)
            ref = node_sums[c][sl]
            for t in range(1, N):
                ref = ref + node_sums[(c + t) % N][sl]
            assert np.array_equal(out[5, sl].view(np.uint32), ref.view(np.uint32)), (j, c)
    direct = oracle.allreduce("lane", N, G, Q, x)
    assert not np.array_equal(direct.view(np.uint32), out.view(np.uint32))  # the data tells them apart


def test_lane_ring_messages_and_boundaries(oracle):
    N, G, Q = 3, 2, 2
    R, P = G * Q, N * G * Q
    n = R * N * 4
    c, piece = n // R, n // R // N
    x = synth.make_inputs(P, n, "int_pm1000")
    total = exact_int_sum(x)
    out, tr = oracle.allreduce("lane_multiproc_ring", N, G, Q, x, want_trace=True)
    assert np.array_equal(out, np.broadcast_to(total, out.shape))
    for ph in (oracle.PH_LANE_S2_RING_RS, oracle.PH_LANE_S2_RING_AG):
        t = tr[tr["phase"] == ph]
        assert len(t) == (N - 1) * P and np.all(t["cnt"] == piece)
        assert np.all(t["src"] % R == t["dst"] % R)                    # same local index
        assert np.all(t["dst"] // R == (t["src"] // R + 1) % N)        # only to the next node
        for r in range(P):
            assert np.sum(t["src"] == r) == N - 1
    assert not np.any((tr["phase"] == oracle.PH_LANE_S2A) | (tr["phase"] == oracle.PH_LANE_S2B))
    # rounds: S1, N-1 reduce rounds, N-1 gather rounds, S3
    mid = oracle.allreduce("lane_multiproc_ring", N, G, Q, x, max_rounds=1 + (N - 1))
    for v in range(N):
        for l in range(R):
            r = v * R + l
            own_piece = (v + 1) % N  # after the reduce loop member v holds the finished piece v+1
            sl = slice(l * c + own_piece * piece, l * c + (own_piece + 1) * piece)
            assert np.array_equal(mid[r, sl], total[sl])
    before_s3 = oracle.allreduce("lane_multiproc_ring", N, G, Q, x, max_rounds=1 + 2 * (N - 1))
    for v in range(N):
        for l in range(R):
            r = v * R + l
            assert np.array_equal(before_s3[r, l * c:(l + 1) * c], total[l * c:(l + 1) * c])
            other = (l + 1) % R
            assert np.array_equal(before_s3[r, other * c:(other + 1) * c], x[r, other * c:(other + 1) * c])


# --------------------------------------------------------------------------- Background section algorithms

POW2_TOPOS = [(1, 1, 1), (2, 1, 1), (1, 2, 2), (2, 2, 1), (2, 2, 2), (4, 2, 2), (1, 4, 4)]


@pytest.mark.parametrize("algo", ["recursive_doubling", "rabenseifner"])
def test_small_message_algorithms_bruteforce(oracle, algo):
    rng = np.random.default_rng(5)
    for (N, G, Q) in POW2_TOPOS:
        P = N * G * Q
        for n in list(range(1, 20)) + [33, 40, 64]:
            x = rng.integers(-(1 << 31), 1 << 31, size=(P, n), dtype=np.int64).astype(np.int32)
            out = oracle.allreduce(algo, N, G, Q, x)
            assert np.array_equal(out, np.broadcast_to(exact_int_sum(x), out.shape)), (algo, N, G, Q, n)
            f = synth.make_inputs(P, n, "uniform_pm1", seed=n)
            got = oracle.allreduce(algo, N, G, Q, f)
            assert all(np.array_equal(got[0], got[r]) for r in range(P))
            exact = np.array([math.fsum(f[:, i].astype(np.float64)) for i in range(n)])
            assert np.all(np.abs(got[0] - exact) <= 1e-5 * np.abs(f).sum(axis=0))
    with pytest.raises(RuntimeError):
        oracle.allreduce(algo, 3, 1, 1, np.zeros((3, 4), dtype=np.int32))   # not a power of two


def test_recursive_doubling_messages_and_order(oracle):
    P, n = 8, 24
    x = synth.order_sensitive_f32(P, n)
    out, tr = oracle.allreduce("recursive_doubling", 2, 2, 2, x, want_trace=True)
    assert len(tr) == P * 3                                      # log2(p) messages per rank ...
    assert np.all(tr["cnt"] == n) and np.all(tr["off"] == 0)     # ... each carrying the whole buffer
    for s in range(3):
        t = tr[tr["step"] == s]
        assert np.array_equal(t["dst"], t["src"] ^ (1 << s))
    # the sum is a balanced tree over neighbours at distance 1, 2, 4
    v = [x[r] for r in range(P)]
    for s in range(3):
        v = [v[r] + v[r ^ (1 << s)] for r in range(P)]
    assert np.array_equal(out[0].view(np.uint32), v[0].view(np.uint32))
    assert np.array_equal(out[5].view(np.uint32), v[0].view(np.uint32))
    flat = f32_sum_in_order(x, list(range(P)))
    assert not np.array_equal(flat.view(np.uint32), v[0].view(np.uint32))


def test_rabenseifner_messages_halve_and_order(oracle):
    P, n = 8, 64
    x = synth.order_sensitive_f32(P, n)
    out, tr = oracle.allreduce("rabenseifner", 1, 4, 2, x, want_trace=True)
    assert len(tr) == P * 6                                      # 2 log2(p) messages per rank
    rs, ag = tr[tr["phase"] == oracle.PH_RABENSEIFNER_RS], tr[tr["phase"] == oracle.PH_RABENSEIFNER_AG]
    for s, (d, size) in enumerate(((4, 32), (2, 16), (1, 8))):   # data cut in half at each step
        t = rs[rs["step"] == s]
        assert np.all(t["cnt"] == size) and np.array_equal(t["dst"], t["src"] ^ d)
    for s, (d, size) in enumerate(((1, 8), (2, 16), (4, 32))):
        t = ag[ag["step"] == 3 + s]
        assert np.all(t["cnt"] == size) and np.array_equal(t["dst"], t["src"] ^ d)
    # after the reduce-scatter rank r owns block number bit-composed from its rank: lower ranks keep first halves
    xi = synth.make_inputs(P, n, "int_pm1000")
    mid = oracle.allreduce("rabenseifner", 1, 4, 2, xi, max_rounds=3)
    total = exact_int_sum(xi)
    for r in range(P):
        assert np.array_equal(mid[r, r * 8:(r + 1) * 8], total[r * 8:(r + 1) * 8])
    # order: partners at distance 4 first, then 2, then 1
    v = [x[r] for r in range(P)]
    for d in (4, 2, 1):
        v = [v[r] + v[r ^ d] for r in range(P)]
    assert np.array_equal(out[3].view(np.uint32), v[0].view(np.uint32))
    rd = oracle.allreduce("recursive_doubling", 1, 4, 2, x)
    assert not np.array_equal(rd.view(np.uint32), out.view(np.uint32))


# --------------------------------------------------------------------------- shared-buffer model

SHARED_ALGOS = ("ring", "lane_multiproc")


@pytest.mark.parametrize("algo", SHARED_ALGOS)
def test_shared_bruteforce_every_small_topology(oracle, algo):
    rng = np.random.default_rng(17)
    for (N, G, Q) in TOPOS:
        B = N * G
        for n in (1, 2, 3, 5, 8, 12, 13, 27, 36, 40):
            x = rng.integers(-(1 << 31), 1 << 31, size=(B, n), dtype=np.int64).astype(np.int32)
            out = oracle.allreduce(algo, N, G, Q, x, shared=True)
            assert np.array_equal(out, np.broadcast_to(exact_int_sum(x), out.shape)), (algo, N, G, Q, n)
            f = synth.make_inputs(B, n, "uniform_pm1", seed=n)
            got = oracle.allreduce(algo, N, G, Q, f, shared=True)
            assert all(np.array_equal(got[0], got[b]) for b in range(B))
            exact = np.array([math.fsum(f[:, i].astype(np.float64)) for i in range(n)])
            assert np.all(np.abs(got[0] - exact) <= 1e-5 * np.abs(f).sum(axis=0))


def test_shared_model_with_one_process_per_gpu_is_the_private_model(oracle):
    x = synth.order_sensitive_f32(6, 41)
    for shared_algo, private_algo in (("ring", "ring"), ("lane_multiproc", "lane")):
        a, ta = oracle.allreduce(shared_algo, 3, 2, 1, x, shared=True, want_trace=True)
        b, tb = oracle.allreduce(private_algo, 3, 2, 1, x, want_trace=True)
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
        for key in ("src", "dst", "off", "cnt"):
            assert np.array_equal(ta[key], tb[key])


def test_shared_standard_messages_scale_with_processes_per_gpu(oracle):
    N, G, n = 2, 3, 6 * 4 * 5  # divisible by N*G*Q for Q = 1, 2, 4
    M = N * G
    x = synth.make_inputs(M, n, "int_pm1000")
    counts = {}
    for Q in (1, 2, 4):
        out, tr = oracle.allreduce("ring", N, G, Q, x, shared=True, want_trace=True)
        assert np.array_equal(out[0], exact_int_sum(x))
        counts[Q] = len(tr)
        assert np.all(tr["cnt"] == n // Q // M)                  # each message 1/PPG of the size
        q = tr["src"] % Q
        assert np.all(tr["dst"] % Q == q)                         # only inside new_comm (equal local rank)
        assert np.all(tr["dst"] // Q == (tr["src"] // Q + 1) % M)  # to the next GPU's process
        lo = q.astype(np.uint64) * (n // Q)
        assert np.all((tr["off"] >= lo) & (tr["off"] + tr["cnt"] <= lo + n // Q))  # own slice only
        for r in range(M * Q):
            assert np.sum(tr["src"] == r) == 2 * (M - 1)
    assert counts[2] == 2 * counts[1] and counts[4] == 4 * counts[1]  # message count grows by PPG


def test_shared_lane_stages_and_order(oracle):
    N, G, Q = 3, 3, 2
    M = N * G
    per = 2
    n = Q * G * N * per
    slice_len, c = n // Q, n // Q // G
    x = synth.order_sensitive_f32(M, n)
    out, tr = oracle.allreduce("lane_multiproc", N, G, Q, x, shared=True, want_trace=True)
    # order: GPUs of a node in ascending order, then nodes in ascending order
    node = [f32_sum_in_order(x, [v * G + g for g in range(G)]) for v in range(N)]
    ref = node[0]
    for v in range(1, N):
        ref = ref + node[v]
    assert np.array_equal(out[4].view(np.uint32), ref.view(np.uint32))
    # message shapes: on-node stages move n/(Q*G), inter-node stages n/(Q*G*N)
    gpu_of = lambda r: r // Q
    for ph, cnt, same_node in ((oracle.PH_LANE_S1, c, True), (oracle.PH_LANE_S2A, c // N, False),
                               (oracle.PH_LANE_S2B, c // N, False), (oracle.PH_LANE_S3, c, True)):
        t = tr[tr["phase"] == ph]
        assert len(t) and np.all(t["cnt"] == cnt)
        assert np.all((gpu_of(t["src"]) // G == gpu_of(t["dst"]) // G) == same_node)
        assert np.all(t["src"] % Q == t["dst"] % Q)
        if not same_node:
            assert np.all(gpu_of(t["src"]) % G == gpu_of(t["dst"]) % G)   # corresponding GPU on the other node
    # after stage 1 the process (node, g, q) holds the node sum of chunk g of slice q, at q*(n/Q) + g*c
    xi = synth.make_inputs(M, n, "int_pm1000")
    s1 = oracle.allreduce("lane_multiproc", N, G, Q, xi, shared=True, max_rounds=1)
    for v in range(N):
        nsum = xi[v * G:(v + 1) * G].astype(np.int64).sum(axis=0).astype(np.int32)
        for g in range(G):
            for q in range(Q):
                sl = slice(q * slice_len + g * c, q * slice_len + (g + 1) * c)
                assert np.array_equal(s1[v * G + g, sl], nsum[sl])
                o = (g + 1) % G
                other = slice(q * slice_len + o * c, q * slice_len + (o + 1) * c)
                assert np.array_equal(s1[v * G + g, other], xi[v * G + g, other])


# --------------------------------------------------------------------------- reduce_segments

def test_reduce_segments_vs_numpy(oracle):
    n, k, seg_len = 200, 3, 17
    offs = [5, 40, 100, 183]
    x = synth.order_sensitive_f32(k + 1, n)
    got = oracle.reduce_segments(x[0], [x[1], x[2], x[3]], offs, seg_len)
    ref = x[0].copy()
    for o in offs:
        acc = x[0][o:o + seg_len].copy()
        for t in range(1, k + 1):
            acc = acc + x[t][o:o + seg_len]
        ref[o:o + seg_len] = acc
    assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))
    xi = np.random.default_rng(5).integers(-(1 << 31), 1 << 31, size=(4, n), dtype=np.int64).astype(np.int32)
    goti = oracle.reduce_segments(xi[0], [xi[1], xi[2], xi[3]], offs, seg_len)
    refi = xi[0].copy()
    for o in offs:
        sl = slice(o, o + seg_len)
        refi[sl] = (xi[:, sl].astype(np.int64).sum(axis=0) & 0xFFFFFFFF).astype(np.uint32).view(np.int32)
    assert np.array_equal(goti, refi)
    assert np.array_equal(oracle.reduce_segments(xi[0], [], offs, seg_len), xi[0])
