"""Host logic of the library, on the CPU: the C ABI loads and exports what the header declares,
argument errors are reported, and the generated step tables -- executed here by a small numpy
interpreter that knows nothing but "sum the sources in order, store to the destinations" --
reproduce the oracle bit for bit.  No GPU call is made."""
import itertools
import os
import re

import numpy as np
import pytest

import paper_2508_13397_amd as la
from paper_2508_13397_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ALGOS = ("ring", "lane", "lane_multiproc")
FLAG_SETS = (la.LA_SCHED_DEFAULT, la.LA_SCHED_P2P_GATHER, la.LA_SCHED_STAGED,
             la.LA_SCHED_P2P_GATHER | la.LA_SCHED_STAGED, la.LA_SCHED_INNER_RING,
             la.LA_SCHED_INNER_RING | la.LA_SCHED_STAGED | la.LA_SCHED_P2P_GATHER)


def oracle_name(algo, flags):
    """the oracle's name of what a schedule built with these flags computes"""
    return algo + "_ring" if (flags & la.LA_SCHED_INNER_RING) and algo != "ring" else algo


# ----------------------------------------------------------------------------- ABI surface

def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "lane_allreduce.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(la_[a-z_0-9]+)\s*\(", header))
    assert declared == set(la.EXPORTS)
    L = la.lib()
    for name in declared:
        assert getattr(L, name) is not None


def test_binding_fails_loudly_when_the_library_is_not_built():
    """No fallback: with the shared library absent every entry point of the binding raises."""
    import subprocess
    import sys

    code = (
        "import sys; sys.path.insert(0, %r)\n"
        "import paper_2508_13397_amd.binding as b\n"
        "b.LIB_PATH = b.LIB_PATH + '.absent'\n"
        "import paper_2508_13397_amd as la\n"
        "for call in (lambda: la.lib(), lambda: la.la_topology_create(2, 2, 1), lambda: la.la_status_string(0)):\n"
        "    try:\n"
        "        call()\n"
        "    except ImportError as e:\n"
        "        assert 'no CPU fallback' in str(e)\n"
        "    else:\n"
        "        sys.exit(5)\n"
        "assert 'oracle' not in sys.modules\n"
        "sys.exit(0)\n"
    ) % ROOT
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stderr[-1500:]


def test_product_package_does_not_import_the_oracle():
    """the oracle is test infrastructure: nothing under the package, nor the library's sources,
    names it"""
    pkg = os.path.join(ROOT, "paper_2508_13397_amd")
    for base, _, files in os.walk(pkg):
        if "_build" in base or "__pycache__" in base:
            continue
        for f in files:
            if f.endswith((".py", ".cpp", ".hpp", ".hip", ".h")):
                text = open(os.path.join(base, f)).read()
                assert "import oracle" not in text and "from oracle" not in text and "la_oracle" not in text, f


def test_header_is_plain_c_and_a_c_program_links_against_the_library(tmp_path):
    """The boundary is a C ABI: the header compiles as strict C99 (and as C++), and a C program
    that uses only host-side calls links against the shared library and runs without a GPU."""
    import subprocess

    inc = os.path.join(ROOT, "include")
    src = tmp_path / "consumer.c"
    src.write_text(
        '#include <stdio.h>\n#include "lane_allreduce.h"\n'
        "int main(void) {\n"
        "    la_topology_t* t = 0; la_schedule_t* s = 0; size_t rd = 0, wr = 0; int k = 0, m = 0;\n"
        "    if (la_topology_create(4, 4, 1, &t) != LA_OK || la_topology_num_ranks(t) != 16) return 1;\n"
        "    if (la_schedule_build(t, LA_ALGO_LANE, 1u << 20, LA_F32, &s) != LA_OK) return 2;\n"
        "    if (la_schedule_num_steps(s) != 3) return 3;\n"
        "    if (la_schedule_step_info(s, 0, 0, 0, 0, 0, &k, &m, &rd, &wr) != LA_OK || k != 4 || m != 1) return 4;\n"
        "    if (rd != (size_t)16 << 22 || wr != (size_t)4 << 22) return 5;\n"
        '    if (la_schedule_build(t, LA_ALGO_LANE, 0, LA_F32, &s) != LA_ERR_INVALID_ARG || !la_last_error()[0]) return 6;\n'
        '    printf("%s\\n", la_status_string(LA_OK));\n'
        "    return la_schedule_destroy(s) == LA_OK && la_topology_destroy(t) == LA_OK ? 0 : 7;\n"
        "}\n")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-I", inc, str(src)], check=True)
    subprocess.run(["g++", "-std=c++11", "-fsyntax-only", "-x", "c++", "-I", inc, str(src)], check=True)
    exe = str(tmp_path / "consumer")
    libdir = os.path.join(ROOT, "paper_2508_13397_amd")
    subprocess.run(["gcc", "-std=c99", "-I", inc, str(src), "-o", exe, "-L", libdir, "-llaneallreduce",
                    "-Wl,-rpath," + libdir], check=True)
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and r.stdout.strip() == "LA_OK", (r.returncode, r.stdout, r.stderr[-500:])


def test_status_strings():
    assert la.la_status_string(la.LA_OK) == "LA_OK"
    assert la.la_status_string(la.LA_ERR_INVALID_ARG) == "LA_ERR_INVALID_ARG"
    assert la.la_status_string(la.LA_ERR_UNSUPPORTED) == "LA_ERR_UNSUPPORTED"
    assert la.la_status_string(la.LA_ERR_OUT_OF_MEMORY) == "LA_ERR_OUT_OF_MEMORY"
    assert la.la_status_string(la.LA_ERR_DEVICE) == "LA_ERR_DEVICE"


@pytest.mark.parametrize("dims", [(0, 1, 1), (1, 0, 1), (1, 1, 0), (-2, 4, 1), (1 << 10, 1 << 10, 2)])
def test_topology_rejects_bad_dimensions(dims):
    with pytest.raises(la.LaError) as e:
        la.la_topology_create(*dims)
    assert e.value.status == la.LA_ERR_INVALID_ARG


def test_topology_rank_count_and_null_handling():
    t = la.la_topology_create(32, 4, 8)
    assert t.num_ranks == 1024
    L = la.lib()
    assert L.la_topology_num_ranks(None) == -1
    assert L.la_schedule_num_steps(None) == -1
    assert L.la_topology_destroy(None) == la.LA_OK and L.la_schedule_destroy(None) == la.LA_OK
    assert L.la_topology_create(1, 1, 1, None) == la.LA_ERR_INVALID_ARG


def test_schedule_build_errors():
    t = la.la_topology_create(2, 2, 1)
    for kwargs, status in (
        (dict(algo="lane", n=0, dtype="float32"), la.LA_ERR_INVALID_ARG),
        (dict(algo=9, n=16, dtype="float32"), la.LA_ERR_UNSUPPORTED),
        (dict(algo="lane", n=16, dtype=9), la.LA_ERR_UNSUPPORTED),
        (dict(algo="lane", n=16, dtype="float32", flags=512), la.LA_ERR_UNSUPPORTED),
        (dict(algo="ring", n=16, dtype="float32", flags=256), la.LA_ERR_UNSUPPORTED),
        (dict(algo="lane", n=16, dtype="float32", flags=256 | 128), la.LA_ERR_INVALID_ARG),
        (dict(algo="lane", n=16, dtype="float32", flags=256 | 2), la.LA_ERR_INVALID_ARG),
        (dict(algo="lane", n=16, dtype="float32", flags=256 | 64), la.LA_ERR_INVALID_ARG),
        (dict(algo="ring", n=16, dtype="float32", flags=128), la.LA_ERR_UNSUPPORTED),
        (dict(algo="rabenseifner", n=16, dtype="float32", flags=128), la.LA_ERR_UNSUPPORTED),
        (dict(algo="lane", n=16, dtype="float32", flags=128 | 1), la.LA_ERR_INVALID_ARG),
        (dict(algo="lane", n=16, dtype="float32", flags=128 | 4), la.LA_ERR_INVALID_ARG),
        (dict(algo="lane", n=16, dtype="float32", flags=128 | 32), la.LA_ERR_INVALID_ARG),
        (dict(algo="lane", n=16, dtype="float32", flags=1 << 20), la.LA_ERR_UNSUPPORTED),
        (dict(algo="lane", n=16, dtype="float32", flags=32 | 64), la.LA_ERR_INVALID_ARG),
        (dict(algo="recursive_doubling", n=16, dtype="float32", flags=32), la.LA_ERR_UNSUPPORTED),
        (dict(algo="ring", n=16, dtype="float32", flags=64 | 8 | 2), la.LA_ERR_UNSUPPORTED),
    ):
        with pytest.raises(la.LaError) as e:
            la.la_schedule_build(t, **kwargs)
        assert e.value.status == status
        assert la.la_last_error() != ""
    import ctypes

    out = ctypes.c_void_p()
    assert la.lib().la_schedule_build(None, 1, 16, 1, ctypes.byref(out)) == la.LA_ERR_INVALID_ARG
    s = la.la_schedule_build(t, "lane", 16, "float32")
    with pytest.raises(la.LaError):
        s.step_info(99)


def test_tuning_knobs():
    assert (la.la_tuning_get("unroll"), la.la_tuning_get("cache_policy"), la.la_tuning_get("block")) == (0, -1, 0)
    assert (la.la_tuning_get("merge"), la.la_tuning_get("forward"), la.la_tuning_get("fuse"), la.la_tuning_get("graph")) == (1, 1, -1, -1)
    assert la.la_tuning_get("fused_launches") >= 0  # a counter, read-only
    with pytest.raises(la.LaError):
        la.la_tuning_set("fused_launches", 0)
    try:
        for key, good, bad in (("unroll", (1, 2, 4, 8, 0), (3, -1, 16)), ("cache_policy", (0, 1, 2, 3, 4, 5, 6, 7, -1), (8, -2)),
                               ("block", (256, 1024, 0), (128, 512, 2048)), ("graph", (0, 1, -1), (2, -2)),
                               ("merge", (0, 1), (2, -1)), ("forward", (0, 1), (2, -1)), ("fuse", (0, 1, -1), (2, -2))):
            for v in good:
                la.la_tuning_set(key, v)
                assert la.la_tuning_get(key) == v
            for v in bad:
                with pytest.raises(la.LaError):
                    la.la_tuning_set(key, v)
    finally:
        la.la_tuning_set("unroll", 0)
        la.la_tuning_set("cache_policy", -1)
        la.la_tuning_set("block", 0)
    with pytest.raises(la.LaError):
        la.la_tuning_set("no_such_knob", 1)
    assert la.la_tuning_get("no_such_knob") == -2


def test_run_calls_reject_bad_arguments_before_touching_a_device():
    import ctypes

    t = la.la_topology_create(2, 1, 1)
    s = la.la_schedule_build(t, "lane", 64, "float32")
    L = la.lib()
    bufs = (ctypes.c_void_p * 2)(0x1000, 0x2000)
    assert L.la_allreduce_emulated(None, bufs, 64, la.LA_F32, la.LA_SUM, None) == la.LA_ERR_INVALID_ARG
    assert L.la_allreduce_emulated(s.handle, None, 64, la.LA_F32, la.LA_SUM, None) == la.LA_ERR_INVALID_ARG
    assert L.la_allreduce_emulated(s.handle, bufs, 32, la.LA_F32, la.LA_SUM, None) == la.LA_ERR_INVALID_ARG
    assert L.la_allreduce_emulated(s.handle, bufs, 64, la.LA_I32, la.LA_SUM, None) == la.LA_ERR_INVALID_ARG
    assert L.la_allreduce_emulated(s.handle, bufs, 64, la.LA_F32, 4, None) == la.LA_ERR_UNSUPPORTED
    null_buf = (ctypes.c_void_p * 2)(0x1000, 0)
    assert L.la_allreduce_emulated(s.handle, null_buf, 64, la.LA_F32, la.LA_SUM, None) == la.LA_ERR_INVALID_ARG
    odd = (ctypes.c_void_p * 2)(0x1001, 0x2000)
    assert L.la_allreduce_emulated(s.handle, odd, 64, la.LA_F32, la.LA_SUM, None) == la.LA_ERR_INVALID_ARG
    same = (ctypes.c_void_p * 2)(0x1000, 0x1000)
    assert L.la_allreduce_emulated(s.handle, same, 64, la.LA_F32, la.LA_SUM, None) == la.LA_ERR_INVALID_ARG
    overlap = (ctypes.c_void_p * 2)(0x1000, 0x1080)
    assert L.la_allreduce_emulated(s.handle, overlap, 64, la.LA_F32, la.LA_SUM, None) == la.LA_ERR_INVALID_ARG
    assert L.la_schedule_run_step(s.handle, 5, bufs, None) == la.LA_ERR_INVALID_ARG
    oop = la.la_schedule_build(t, "lane", 64, "float32", la.LA_SCHED_OUT_OF_PLACE)
    other = (ctypes.c_void_p * 2)(0x5000, 0x6000)
    f = L.la_allreduce_emulated_out_of_place
    assert L.la_allreduce_emulated(oop.handle, bufs, 64, la.LA_F32, la.LA_SUM, None) == la.LA_ERR_INVALID_ARG
    assert f(s.handle, other, bufs, 64, la.LA_F32, la.LA_SUM, None) == la.LA_ERR_INVALID_ARG   # in-place schedule
    assert f(oop.handle, None, bufs, 64, la.LA_F32, la.LA_SUM, None) == la.LA_ERR_INVALID_ARG
    assert f(oop.handle, bufs, bufs, 64, la.LA_F32, la.LA_SUM, None) == la.LA_ERR_INVALID_ARG   # send aliases receive
    assert f(oop.handle, other, bufs, 64, la.LA_F32, 9, None) == la.LA_ERR_UNSUPPORTED
    assert f(oop.handle, other, bufs, 32, la.LA_F32, la.LA_SUM, None) == la.LA_ERR_INVALID_ARG
    offs = (ctypes.c_size_t * 2)(0, 8)
    srcs = (ctypes.c_void_p * 1)(0x3000)
    rs = L.la_reduce_segments
    assert rs(None, srcs, 1, offs, 2, 8, la.LA_F32, la.LA_SUM, None) == la.LA_ERR_INVALID_ARG
    assert rs(0x1000, None, 1, offs, 2, 8, la.LA_F32, la.LA_SUM, None) == la.LA_ERR_INVALID_ARG
    assert rs(0x1000, srcs, -1, offs, 2, 8, la.LA_F32, la.LA_SUM, None) == la.LA_ERR_INVALID_ARG
    assert rs(0x1000, srcs, 1, None, 2, 8, la.LA_F32, la.LA_SUM, None) == la.LA_ERR_INVALID_ARG
    assert rs(0x1002, srcs, 1, offs, 2, 8, la.LA_F32, la.LA_SUM, None) == la.LA_ERR_INVALID_ARG
    assert rs(0x1000, srcs, 1, offs, 2, 9, la.LA_F32, la.LA_SUM, None) == la.LA_ERR_INVALID_ARG  # overlap
    assert rs(0x1000, srcs, 1, offs, 2, 8, 5, la.LA_SUM, None) == la.LA_ERR_UNSUPPORTED
    assert rs(0x1000, srcs, 1, offs, 2, 8, la.LA_F32, 7, None) == la.LA_ERR_UNSUPPORTED
    alias = (ctypes.c_void_p * 1)(0x1000)
    assert rs(0x1000, alias, 1, offs, 2, 8, la.LA_F32, la.LA_SUM, None) == la.LA_ERR_INVALID_ARG
    # nothing to do: accepted without any device work
    assert rs(0x1000, srcs, 0, offs, 2, 8, la.LA_F32, la.LA_SUM, None) == la.LA_OK
    assert rs(0x1000, srcs, 1, offs, 0, 8, la.LA_F32, la.LA_SUM, None) == la.LA_OK
    assert rs(0x1000, srcs, 1, offs, 2, 0, la.LA_F32, la.LA_SUM, None) == la.LA_OK


# ----------------------------------------------------------------------------- table interpreter

def bf16_narrow(x32):
    import torch

    return torch.from_numpy(x32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def sum_in_order(ops, group=None):
    """one segment: the operands added in table order (uint16 = bf16 bits: fp32 accumulation, one
    rounding at the end; int32 wraps).  With group < len(ops): runs of `group` operands are summed
    (and rounded) first, then the run results in order."""
    if group and group < len(ops):
        return sum_in_order([sum_in_order(ops[i:i + group]) for i in range(0, len(ops), group)])
    if ops[0].dtype == np.uint16:
        if len(ops) == 1:
            return ops[0].copy()
        acc = (ops[0].astype(np.uint32) << 16).view(np.float32)
        for x in ops[1:]:
            acc = acc + (x.astype(np.uint32) << 16).view(np.float32)
        return bf16_narrow(np.ascontiguousarray(acc))
    if ops[0].dtype == np.int32:
        acc = ops[0].view(np.uint32).copy()
        for x in ops[1:]:
            acc = acc + x.view(np.uint32)
        return acc.view(np.int32)
    acc = ops[0].copy()
    for x in ops[1:]:
        acc = acc + x
    return acc


def run_tables(sched, inputs, snapshot=True, upto=None):
    """Execute the step tables on host arrays.  With snapshot=True every step reads the state
    from before the step (what concurrent workgroups see if the step is hazard-free)."""
    P, n = inputs.shape
    state = [inputs[r].copy() for r in range(P)] + [np.zeros(max(sched.staging_elems, 1), dtype=inputs.dtype)]
    steps = range(sched.num_steps if upto is None else upto)
    for i in steps:
        t = sched.step_table(i)
        old = [b.copy() for b in state] if snapshot else state
        for g in range(t["num_segments"]):
            ln = int(t["seg_len"][g])
            ops = [old[int(b)][int(o):int(o) + ln] for b, o in zip(t["src_buf"][g], t["src_off"][g])]
            res = sum_in_order(ops, t["group"])
            for b, o in zip(t["dst_buf"][g], t["dst_off"][g]):
                state[int(b)][int(o):int(o) + ln] = res
    return np.stack(state[:P])


TOPOS = [t for t in itertools.product((1, 2, 3), repeat=3)]


@pytest.mark.parametrize("algo", ALGOS)
@pytest.mark.parametrize("flags", FLAG_SETS)
def test_tables_reproduce_oracle_bitwise_small_topologies(oracle, algo, flags):
    for (N, G, Q) in TOPOS:
        P = N * G * Q
        topo = la.la_topology_create(N, G, Q)
        for n in (1, 2, 5, 17, 36, 40):
            for kind in ("i32", "f32", "bf16"):
                if kind == "i32":
                    x = np.random.default_rng(n).integers(-(1 << 31), 1 << 31, size=(P, n), dtype=np.int64).astype(np.int32)
                elif kind == "f32":
                    x = synth.order_sensitive_f32(P, n)
                else:
                    x = synth.to_bf16_bits(synth.order_sensitive_f32(P, n) * np.float32(2.0 ** -20))
                dt = {"i32": "int32", "f32": "float32", "bf16": "bfloat16"}[kind]
                sched = la.la_schedule_build(topo, algo, n, dt, flags)
                got = run_tables(sched, x)
                ref = oracle.allreduce(oracle_name(algo, flags), N, G, Q, x)
                assert np.array_equal(got.view(np.uint8), ref.view(np.uint8)), (algo, flags, N, G, Q, n, kind)
                if n == 17:
                    seq = run_tables(sched, x, snapshot=False)
                    assert np.array_equal(seq.view(np.uint8), got.view(np.uint8))


SHARED = la.LA_SCHED_SHARED_BUFFERS


@pytest.mark.parametrize("algo", ["ring", "lane_multiproc", "lane"])
@pytest.mark.parametrize("extra", [0, la.LA_SCHED_P2P_GATHER, la.LA_SCHED_STAGED, la.LA_SCHED_P2P_GATHER | la.LA_SCHED_STAGED])
def test_shared_buffer_tables_reproduce_oracle_bitwise(oracle, algo, extra):
    for (N, G, Q) in TOPOS:
        B = N * G
        topo = la.la_topology_create(N, G, Q)
        for n in (1, 3, 10, 17, 36, 40):
            for kind in ("i32", "f32", "bf16"):
                if kind == "i32":
                    x = np.random.default_rng(n).integers(-(1 << 31), 1 << 31, size=(B, n), dtype=np.int64).astype(np.int32)
                elif kind == "f32":
                    x = synth.order_sensitive_f32(B, n)
                else:
                    x = synth.to_bf16_bits(synth.order_sensitive_f32(B, n) * np.float32(2.0 ** -20))
                dt = {"i32": "int32", "f32": "float32", "bf16": "bfloat16"}[kind]
                sched = la.la_schedule_build(topo, algo, n, dt, SHARED | extra)
                assert sched.num_buffers == B
                got = run_tables(sched, x)
                if algo == "lane":  # one process per GPU does the whole buffer
                    ref = oracle.allreduce("lane_multiproc", N, G, 1, x, shared=True)
                else:
                    ref = oracle.allreduce(algo, N, G, Q, x, shared=True)
                assert np.array_equal(got.view(np.uint8), ref.view(np.uint8)), (algo, extra, N, G, Q, n, kind)
                if n == 17:
                    seq = run_tables(sched, x, snapshot=False)
                    assert np.array_equal(seq.view(np.uint8), got.view(np.uint8))


def test_shared_buffer_shapes_and_bytes():
    N, G, Q, n, e = 4, 4, 4, 1 << 22, 4
    M = N * G
    t = la.la_topology_create(N, G, Q)
    std = la.la_schedule_build(t, "ring", n, "float32", SHARED)
    one = la.la_schedule_build(la.la_topology_create(N, G, 1), "ring", n, "float32", SHARED)
    assert std.num_buffers == M and std.num_steps == one.num_steps == 2 * (M - 1)
    for a, b in zip(std.steps(), one.steps()):
        # Q times the messages, each 1/Q of the size, same bytes
        assert a["num_segments"] == Q * b["num_segments"] and a["seg_len_max"] * Q == b["seg_len_max"]
        assert (a["bytes_read"], a["bytes_written"]) == (b["bytes_read"], b["bytes_written"])
    assert sum(totals(std)) == 5 * (M - 1) * n * e
    lane = la.la_schedule_build(t, "lane_multiproc", n, "float32", SHARED)
    st = {x["stage"]: x for x in lane.steps()}
    assert (st[la.LA_STAGE_S1]["fan_in"], st[la.LA_STAGE_S1]["num_segments"], st[la.LA_STAGE_S1]["seg_len_max"]) == (G, M * Q, n // (Q * G))
    assert (st[la.LA_STAGE_S1]["bytes_read"], st[la.LA_STAGE_S1]["bytes_written"]) == (M * n * e, N * n * e)
    assert (st[la.LA_STAGE_S2]["fan_in"], st[la.LA_STAGE_S2]["seg_len_max"]) == (N, n // (Q * G * N))   # inter-node piece / procs per node
    assert (st[la.LA_STAGE_S3]["bytes_read"], st[la.LA_STAGE_S3]["bytes_written"]) == (N * n * e, (M - N) * n * e)
    # copy-in / copy-out: one private slot per process, the all-reduce touches staging only
    staged = la.la_schedule_build(t, "lane_multiproc", n, "float32", SHARED | la.LA_SCHED_STAGED)
    assert staged.staging_elems >= M * n
    steps = staged.steps()
    assert steps[0]["stage"] == steps[-1]["stage"] == la.LA_STAGE_PACK
    assert steps[0]["num_segments"] == steps[-1]["num_segments"] == M * Q
    for i in range(1, staged.num_steps - 1):
        tb = staged.step_table(i)
        assert np.all(tb["src_buf"] == M) and np.all(tb["dst_buf"] == M)
    assert np.all(staged.step_table(0)["dst_buf"] == M) and np.all(staged.step_table(0)["src_buf"] < M)
    with pytest.raises(la.LaError) as err:
        la.la_schedule_build(t, "lane_multiproc", n, "float32", SHARED | la.LA_SCHED_INNER_RING)
    assert err.value.status == la.LA_ERR_UNSUPPORTED


def run_tables_out_of_place(sched, inputs):
    """Interpreter for LA_SCHED_OUT_OF_PLACE tables: buffers [0,B) receive (pre-filled with junk),
    B staging, B+1+b send buffer b.  Returns (receive buffers, send buffers) after the run."""
    B, n = inputs.shape
    junk = np.full(n, 0x5A5A5A5A5A5A5A5A, dtype=np.uint64).view(np.uint8)[: n * inputs.dtype.itemsize].view(inputs.dtype)
    state = [junk.copy() for _ in range(B)] + [np.zeros(max(sched.staging_elems, 1), dtype=inputs.dtype)] + \
            [inputs[b].copy() for b in range(B)]
    for i in range(sched.num_steps):
        t = sched.step_table(i)
        old = [b.copy() for b in state]
        assert np.all(t["dst_buf"] <= B)  # send buffers are never written
        for g in range(t["num_segments"]):
            ln = int(t["seg_len"][g])
            ops = [old[int(b)][int(o):int(o) + ln] for b, o in zip(t["src_buf"][g], t["src_off"][g])]
            res = sum_in_order(ops, t["group"])
            for b, o in zip(t["dst_buf"][g], t["dst_off"][g]):
                state[int(b)][int(o):int(o) + ln] = res
    return np.stack(state[:B]), np.stack(state[B + 1:])


@pytest.mark.parametrize("algo", ALGOS)
@pytest.mark.parametrize("extra", [0, la.LA_SCHED_P2P_GATHER, la.LA_SCHED_STAGED, la.LA_SCHED_INNER_RING,
                                   la.LA_SCHED_SHARED_BUFFERS, la.LA_SCHED_SHARED_BUFFERS | la.LA_SCHED_STAGED])
def test_out_of_place_tables(oracle, algo, extra):
    OOP = la.LA_SCHED_OUT_OF_PLACE
    shared = bool(extra & la.LA_SCHED_SHARED_BUFFERS)
    for (N, G, Q) in TOPOS:
        B = N * G if shared else N * G * Q
        topo = la.la_topology_create(N, G, Q)
        for n in (1, 4, 17, 36):
            for x in (np.random.default_rng(n).integers(-(1 << 31), 1 << 31, size=(B, n), dtype=np.int64).astype(np.int32),
                      synth.order_sensitive_f32(B, n)):
                sched = la.la_schedule_build(topo, algo, n, "int32" if x.dtype == np.int32 else "float32", OOP | extra)
                recv, send = run_tables_out_of_place(sched, x)
                if shared:
                    ref = oracle.allreduce("lane_multiproc" if algo == "lane" else algo, N, G, 1 if algo == "lane" else Q, x, shared=True)
                else:
                    ref = oracle.allreduce(oracle_name(algo, extra), N, G, Q, x)
                assert np.array_equal(recv.view(np.uint8), ref.view(np.uint8)), (algo, extra, N, G, Q, n)
                assert np.array_equal(send.view(np.uint8), x.view(np.uint8))


def test_out_of_place_ring_reads_send_buffers_like_algorithm_1():
    P, n = 4, 64
    s = la.la_schedule_build(la.la_topology_create(2, 2, 1), "ring", n, "float32", la.LA_SCHED_OUT_OF_PLACE)
    first = s.step_table(0)
    assert np.all(first["src_buf"] > P)                      # first iteration: both operands from buf_send
    for i in range(1, P - 1):
        t = s.step_table(i)
        assert np.all(t["src_buf"][:, 0] > P)                # own copy: still the original input
        assert np.all(t["src_buf"][:, 1] < P)                # incoming partial sum: from the previous rank's buf_recv
    for i in range(P - 1, 2 * (P - 1)):
        assert np.all(s.step_table(i)["src_buf"] < P)        # gather loop: buf_recv only
    single = la.la_schedule_build(la.la_topology_create(1, 1, 1), "lane", n, "float32", la.LA_SCHED_OUT_OF_PLACE)
    assert [x["stage"] for x in single.steps()] == [la.LA_STAGE_COPY_INPUT]


@pytest.mark.parametrize("algo", ["recursive_doubling", "rabenseifner"])
@pytest.mark.parametrize("extra", [0, la.LA_SCHED_STAGED, la.LA_SCHED_OUT_OF_PLACE])
def test_small_message_algorithm_tables(oracle, algo, extra):
    for (N, G, Q) in [(1, 1, 1), (2, 1, 1), (1, 2, 2), (2, 2, 2), (4, 2, 2)]:
        P = N * G * Q
        topo = la.la_topology_create(N, G, Q)
        for n in (1, 3, 8, 17, 40, 64):
            for x in (np.random.default_rng(n).integers(-(1 << 31), 1 << 31, size=(P, n), dtype=np.int64).astype(np.int32),
                      synth.order_sensitive_f32(P, n)):
                sched = la.la_schedule_build(topo, algo, n, "int32" if x.dtype == np.int32 else "float32", extra)
                ref = oracle.allreduce(algo, N, G, Q, x)
                if extra & la.LA_SCHED_OUT_OF_PLACE:
                    got, send = run_tables_out_of_place(sched, x)
                    assert np.array_equal(send.view(np.uint8), x.view(np.uint8))
                else:
                    got = run_tables(sched, x)
                    assert np.array_equal(run_tables(sched, x, snapshot=False).view(np.uint8), got.view(np.uint8))
                assert np.array_equal(got.view(np.uint8), ref.view(np.uint8)), (algo, extra, N, G, Q, n)


def test_small_message_algorithm_shapes():
    P, n, e = 16, 1 << 20, 4
    t = la.la_topology_create(4, 4, 1)
    rd = la.la_schedule_build(t, "recursive_doubling", n, "float32")
    assert rd.num_steps == 4                                                  # log2 p exchanges ...
    assert all((x["num_segments"], x["seg_len_max"], x["fan_in"], x["fan_out"]) == (P // 2, n, 2, 2) for x in rd.steps())  # ... of the whole buffer
    rab = la.la_schedule_build(t, "rabenseifner", n, "float32")
    assert rab.num_steps == 8                                                 # 2 log2 p
    assert [x["seg_len_max"] for x in rab.steps()] == [n >> 1, n >> 2, n >> 3, n >> 4, n >> 4, n >> 3, n >> 2, n >> 1]
    assert sum(totals(rab)) == (3 * (P - 1) * n // P * P + 2 * (P - 1) * n // P * P) * e // 1  # 5 (p-1)/p n per rank, p ranks
    for algo in ("recursive_doubling", "rabenseifner"):
        with pytest.raises(la.LaError) as err:
            la.la_schedule_build(la.la_topology_create(3, 2, 1), algo, n, "float32")
        assert err.value.status == la.LA_ERR_UNSUPPORTED
        with pytest.raises(la.LaError):
            la.la_schedule_build(t, algo, n, "float32", la.LA_SCHED_SHARED_BUFFERS)


# ----------------------------------------------------------------------------- fused all-gathers

FUSED = la.LA_SCHED_FUSED_GATHER


@pytest.mark.parametrize("algo", ["lane", "lane_multiproc"])
@pytest.mark.parametrize("extra", [0, la.LA_SCHED_STAGED, la.LA_SCHED_OUT_OF_PLACE, SHARED, SHARED | la.LA_SCHED_STAGED])
def test_fused_gather_tables_reproduce_oracle_bitwise(oracle, algo, extra):
    """With the all-gathers folded into the last reduce's store the result is still the oracle's,
    bit for bit, and the schedule has no copy launch left (staging and input copies aside)."""
    for (N, G, Q) in TOPOS:
        topo = la.la_topology_create(N, G, Q)
        B = N * G if extra & SHARED else N * G * Q
        for n in (1, 5, 17, 40):
            for x in (np.random.default_rng(n).integers(-(1 << 31), 1 << 31, size=(B, n), dtype=np.int64).astype(np.int32),
                      synth.order_sensitive_f32(B, n), synth.to_bf16_bits(synth.order_sensitive_f32(B, n) * np.float32(2.0 ** -20))):
                dt = {np.dtype(np.int32): "int32", np.dtype(np.float32): "float32", np.dtype(np.uint16): "bfloat16"}[x.dtype]
                sched = la.la_schedule_build(topo, algo, n, dt, FUSED | extra)
                if extra & SHARED:
                    ref = oracle.allreduce("lane_multiproc", N, G, 1 if algo == "lane" else Q, x, shared=True)
                else:
                    ref = oracle.allreduce(algo, N, G, Q, x)
                if extra & la.LA_SCHED_OUT_OF_PLACE:
                    got, send = run_tables_out_of_place(sched, x)
                    assert np.array_equal(send.view(np.uint8), x.view(np.uint8))
                else:
                    got = run_tables(sched, x)
                    assert np.array_equal(run_tables(sched, x, snapshot=False).view(np.uint8), got.view(np.uint8))
                assert np.array_equal(got.view(np.uint8), ref.view(np.uint8)), (algo, extra, N, G, Q, n, dt)
                stages = [st["stage_name"] for st in sched.steps()]
                assert not {"S2b", "S3", "S2"} & set(stages)
                if not extra:
                    R = G * Q
                    assert stages == ([] if R == 1 and N == 1 else ["S1+S3"] if N == 1 else (["S1"] if R > 1 else []) + ["S2+S3"])


def test_fused_gather_shapes_and_bytes():
    """C2 shape: S1 (4 -> 1) and one launch with k = N sources and m = N * R destinations; the
    bytes are those of the unfused schedule minus S3's read of every owner's part."""
    n, e = 1 << 20, 4
    N, G, Q = 4, 4, 1
    P, R = N * G * Q, G * Q
    t = la.la_topology_create(N, G, Q)
    fused = la.la_schedule_build(t, "lane", n, "float32", FUSED)
    plain = la.la_schedule_build(t, "lane", n, "float32")
    assert [(x["stage_name"], x["fan_in"], x["fan_out"], x["num_segments"]) for x in fused.steps()] == \
        [("S1", R, 1, N * G), ("S2+S3", N, N * R, G * N)]
    rf, wf = totals(fused)
    rp, wp = totals(plain)
    assert (rf, wf) == ((P + N) * n * e, (N + P) * n * e)
    assert rp - rf == N * n * e          # S3 no longer re-reads the owners' parts
    assert wp == wf                      # every buffer is still written once per all-gathered element
    one = la.la_schedule_build(la.la_topology_create(1, 4, 2), "lane_multiproc", n, "float32", FUSED)
    assert [(x["stage_name"], x["fan_in"], x["fan_out"]) for x in one.steps()] == [("S1+S3", 8, 8)]


# ----------------------------------------------------------------------------- one launch

ONE = la.LA_SCHED_SINGLE_LAUNCH


@pytest.mark.parametrize("algo", ["lane", "lane_multiproc"])
@pytest.mark.parametrize("extra", [0, la.LA_SCHED_OUT_OF_PLACE, SHARED, SHARED | la.LA_SCHED_OUT_OF_PLACE])
def test_single_launch_tables_reproduce_oracle_bitwise(oracle, algo, extra):
    """Algorithm 2 as one two-level reduce: node sums first (rounded as stored), then across the
    nodes.  Order-sensitive fp32 and bf16 inputs tell it apart from a flat sum and from a sum that
    skips the intermediate rounding."""
    for (N, G, Q) in TOPOS:
        topo = la.la_topology_create(N, G, Q)
        B = N * G if extra & SHARED else N * G * Q
        for n in (1, 5, 17, 40):
            for x in (np.random.default_rng(n).integers(-(1 << 31), 1 << 31, size=(B, n), dtype=np.int64).astype(np.int32),
                      synth.order_sensitive_f32(B, n), synth.to_bf16_bits(synth.order_sensitive_f32(B, n) * np.float32(2.0 ** -20))):
                dt = {np.dtype(np.int32): "int32", np.dtype(np.float32): "float32", np.dtype(np.uint16): "bfloat16"}[x.dtype]
                sched = la.la_schedule_build(topo, algo, n, dt, ONE | extra)
                if extra & SHARED:
                    ref = oracle.allreduce("lane_multiproc", N, G, 1 if algo == "lane" else Q, x, shared=True)
                else:
                    ref = oracle.allreduce(algo, N, G, Q, x)
                if extra & la.LA_SCHED_OUT_OF_PLACE:
                    got, send = run_tables_out_of_place(sched, x)
                    assert np.array_equal(send.view(np.uint8), x.view(np.uint8))
                else:
                    got = run_tables(sched, x)
                assert np.array_equal(got.view(np.uint8), ref.view(np.uint8)), (algo, extra, N, G, Q, n, dt)
                steps = sched.steps()
                reduces = [st for st in steps if st["stage_name"] != "copy-input"]
                assert len(reduces) == (0 if B == 1 else 1)
                if reduces:
                    R = G if extra & SHARED else G * Q
                    st = reduces[0]
                    assert (st["fan_in"], st["fan_out"]) == (N * R, N * R)
                    assert st["group"] == (R if N > 1 and R > 1 else N * R)


def test_single_launch_differs_from_flat_and_unrounded_sums():
    """The two-level order is not decoration: on order-sensitive inputs a flat sum over all ranks,
    and for bf16 a two-level sum without the intermediate rounding, give other bits."""
    N, G, Q, n = 3, 2, 2, 64
    P = N * G * Q
    topo = la.la_topology_create(N, G, Q)
    x = synth.order_sensitive_f32(P, n)
    sched = la.la_schedule_build(topo, "lane_multiproc", n, "float32", ONE)
    got = run_tables(sched, x)
    flat = x[0].copy()
    for r in range(1, P):
        flat = flat + x[r]
    assert not np.array_equal(got[0].view(np.uint32), flat.view(np.uint32))
    xb = synth.to_bf16_bits(synth.make_inputs(P, n, "normal", seed=5))
    sb = la.la_schedule_build(topo, "lane_multiproc", n, "bfloat16", ONE)
    gotb = run_tables(sb, xb)
    wide = (xb.astype(np.uint32) << 16).view(np.float32)
    node = [sum_f32(wide[w * G * Q:(w + 1) * G * Q]) for w in range(N)]
    unrounded = bf16_narrow(np.ascontiguousarray(sum_f32(np.stack(node))))
    assert not np.array_equal(gotb[0], unrounded)


def sum_f32(rows):
    acc = rows[0].copy()
    for r in rows[1:]:
        acc = acc + r
    return acc


def test_single_launch_bytes_are_the_lower_bound():
    n, e = 1 << 20, 4
    t = la.la_topology_create(4, 4, 1)
    one = la.la_schedule_build(t, "lane", n, "float32", ONE)
    assert one.num_steps == 1
    assert totals(one) == (16 * n * e, 16 * n * e)      # every input read once, every output written once


# ----------------------------------------------------------------------------- random flag combinations

def test_random_flag_combinations_either_refused_or_equal_to_the_oracle(oracle):
    """Seeded sweep over algorithms x flag subsets x topologies x lengths: a combination is either
    refused with an argument error, or its tables reproduce the oracle bit for bit (fp32 and bf16
    order-sensitive inputs, wrapping int32).  Guards the passes that are layered on one another (staging,
    out-of-place, shared buffers, the fused forms) against combinations no other test names."""
    rng = np.random.default_rng(20250813)
    bits_pool = [la.LA_SCHED_P2P_GATHER, la.LA_SCHED_STAGED, la.LA_SCHED_INNER_RING, SHARED, la.LA_SCHED_OUT_OF_PLACE,
                 la.LA_SCHED_FUSED_GATHER, la.LA_SCHED_SINGLE_LAUNCH]
    algos = ["ring", "lane", "lane_multiproc", "recursive_doubling", "rabenseifner"]
    ran = refused = 0
    seen = set()
    for case in range(1200):
        algo = algos[rng.integers(len(algos))]
        flags = 0
        for b in bits_pool:
            if rng.random() < 0.3:
                flags |= b
        N, G, Q = (int(v) for v in rng.integers(1, 5, size=3))
        if algo in ("recursive_doubling", "rabenseifner"):
            N, G, Q = (int(v) for v in 2 ** rng.integers(0, 3, size=3))
        n = int(rng.integers(1, 70))
        topo = la.la_topology_create(N, G, Q)
        dt = ("float32", "bfloat16", "int32")[case % 3]
        try:
            sched = la.la_schedule_build(topo, algo, n, dt, flags)
        except la.LaError as err:
            assert err.status in (la.LA_ERR_INVALID_ARG, la.LA_ERR_UNSUPPORTED), (algo, flags)
            refused += 1
            continue
        B = sched.num_buffers
        assert B == (N * G if flags & SHARED else N * G * Q)
        x = synth.order_sensitive_f32(B, n)
        if dt == "bfloat16":
            x = synth.to_bf16_bits(x * np.float32(2.0 ** -20))
        elif dt == "int32":
            x = rng.integers(-(1 << 31), 1 << 31, size=(B, n), dtype=np.int64).astype(np.int32)
        if flags & SHARED:
            name, Qo = ("lane_multiproc", 1) if algo == "lane" else (algo, Q)
            ref = oracle.allreduce(name, N, G, Qo, x, shared=True)
        else:
            # the point-to-point gather and the inner ring are ignored where there is no inter-node stage
            lane = algo in ("lane", "lane_multiproc")
            ref = oracle.allreduce(oracle_name(algo, flags) if lane else algo, N, G, Q, x)
        if flags & la.LA_SCHED_OUT_OF_PLACE:
            got, send = run_tables_out_of_place(sched, x)
            assert np.array_equal(send.view(np.uint8), x.view(np.uint8))
        else:
            got = run_tables(sched, x)
        assert np.array_equal(got.view(np.uint8), ref.view(np.uint8)), (algo, flags, N, G, Q, n)
        ran += 1
        seen.add((algo, flags))
    assert ran >= 450 and refused >= 90 and len(seen) >= 100, (ran, refused, len(seen))


# ----------------------------------------------------------------------------- stand-alone halves

RS, AG = la.LA_SCHED_ONLY_REDUCE_SCATTER, la.LA_SCHED_ONLY_ALLGATHER


def reduce_scatter_rounds(algo, flags, N, G, Q):
    """communication rounds of the oracle that make up the first half: the first loop of
    Algorithm 1; MPI_Reduce_scatter on the node group plus the reduce-scatter inside the lane
    all-reduce of Algorithm 2; the halving phase of Rabenseifner's algorithm"""
    if flags & SHARED:
        return N * G - 1 if algo == "ring" else 2
    P = N * G * Q
    if algo == "ring":
        return P - 1
    if algo == "rabenseifner":
        return P.bit_length() - 1
    return 1 + (N - 1) if flags & la.LA_SCHED_INNER_RING else 2


def owned_mask(sched, nbuf, n):
    mask = np.zeros((nbuf, n), dtype=bool)
    for b in range(nbuf):
        for off, ln in sched.owned_ranges(b):
            assert ln > 0 and off + ln <= n
            assert not mask[b, off:off + ln].any()
            mask[b, off:off + ln] = True
    return mask


HALF_CASES = [(a, f) for a in ALGOS for f in FLAG_SETS] + [("rabenseifner", 0), ("rabenseifner", la.LA_SCHED_STAGED)] + \
             [(a, SHARED | f) for a in ALGOS for f in (0, la.LA_SCHED_P2P_GATHER)]


@pytest.mark.parametrize("algo,flags", HALF_CASES)
def test_reduce_scatter_half_then_allgather_half(oracle, algo, flags):
    """The first half leaves the complete reduction on the owned ranges (which tile the vector
    once per node group / ring), bit-equal to the oracle stopped after its reduce-scatter
    rounds; the second half, run on a state that holds ONLY those ranges, gives the oracle's
    all-reduce; and the two halves in a row are the fused schedule."""
    topos = [(1, 1, 1), (2, 1, 1), (1, 2, 2), (2, 2, 2), (4, 2, 2)] if algo == "rabenseifner" else TOPOS
    for (N, G, Q) in topos:
        P = N * G * Q
        topo = la.la_topology_create(N, G, Q)
        for n in (1, 5, 17, 40):
            for x in (np.random.default_rng(n).integers(-(1 << 31), 1 << 31, size=(P, n), dtype=np.int64).astype(np.int32),
                      synth.order_sensitive_f32(P, n)):
                dt = "int32" if x.dtype == np.int32 else "float32"
                rs = la.la_schedule_build(topo, algo, n, dt, flags | RS)
                ag = la.la_schedule_build(topo, algo, n, dt, flags | AG)
                full = la.la_schedule_build(topo, algo, n, dt, flags)
                B = full.num_buffers
                assert rs.num_buffers == ag.num_buffers == B
                assert rs.num_steps + ag.num_steps >= full.num_steps   # the fused S2 launch splits in two
                xb = x[:B].copy()               # one buffer per GPU (shared) or per rank
                name, Qo, kw = oracle_name(algo, flags), Q, {}
                if flags & SHARED:   # "lane" with shared buffers: one process per GPU does the whole buffer
                    name, Qo, kw = ("lane_multiproc", 1, dict(shared=True)) if algo == "lane" else (algo, Q, dict(shared=True))
                ref_full = oracle.allreduce(name, N, G, Qo, xb, **kw)
                ref_half = oracle.allreduce(name, N, G, Qo, xb, max_rounds=reduce_scatter_rounds(algo, flags, N, G, Q), **kw)
                mask = owned_mask(rs, B, n)
                assert [ag.owned_ranges(b) for b in range(B)] == [rs.owned_ranges(b) for b in range(B)]
                # every element of the vector is owned exactly once per ring / per node-spanning group
                assert np.array_equal(mask.sum(axis=0), np.full(n, 1))
                mid = run_tables(rs, xb)
                assert np.array_equal(mid.view(np.uint8), ref_half.view(np.uint8)), (algo, flags, N, G, Q, n)
                assert np.array_equal(mid[mask].view(np.uint8), ref_full[mask].view(np.uint8))
                # all-gather from a state that holds nothing but the owned ranges
                poisoned = np.where(mask, mid, np.array(0x7fc0dead, dtype=np.uint32).view(x.dtype) if x.dtype == np.float32 else np.int32(-559038737))
                out = run_tables(ag, poisoned.astype(x.dtype))
                assert np.array_equal(out.view(np.uint8), ref_full.view(np.uint8)), (algo, flags, N, G, Q, n)
                assert np.array_equal(run_tables(ag, mid).view(np.uint8), run_tables(full, xb).view(np.uint8))


@pytest.mark.parametrize("algo", ALGOS + ("rabenseifner",))
def test_halves_out_of_place(oracle, algo):
    """Out of place the first half writes only what a rank owns (plus partial sums on the way);
    the second takes the owned ranges from the send buffers and fills every receive buffer."""
    for (N, G, Q) in [(1, 1, 1), (2, 2, 2), (4, 2, 1), (1, 4, 2)] + ([] if algo == "rabenseifner" else [(3, 2, 1), (2, 3, 2)]):
        P = N * G * Q
        topo = la.la_topology_create(N, G, Q)
        for n in (3, 17, 64):
            x = synth.order_sensitive_f32(P, n)
            ref = oracle.allreduce(algo, N, G, Q, x)
            rs = la.la_schedule_build(topo, algo, n, "float32", RS | la.LA_SCHED_OUT_OF_PLACE)
            ag = la.la_schedule_build(topo, algo, n, "float32", AG | la.LA_SCHED_OUT_OF_PLACE)
            mask = owned_mask(rs, P, n)
            mid, send = run_tables_out_of_place(rs, x)
            assert np.array_equal(send.view(np.uint8), x.view(np.uint8))
            assert np.array_equal(mid[mask].view(np.uint8), ref[mask].view(np.uint8)), (algo, N, G, Q, n)
            only_owned = np.where(mask, mid, np.float32(np.nan))
            out, send2 = run_tables_out_of_place(ag, only_owned)
            assert np.array_equal(send2.view(np.uint8), only_owned.view(np.uint8))
            assert np.array_equal(out.view(np.uint8), ref.view(np.uint8)), (algo, N, G, Q, n)


def test_halves_shapes_and_bytes():
    """Lane halves at the scale-up shape: S1 + S2a, then S2b as one broadcast launch + S3; the
    byte totals of the two halves add up to the point-to-point form's minus nothing."""
    n, e = 1 << 20, 4
    t = la.la_topology_create(4, 4, 2)
    rs = la.la_schedule_build(t, "lane_multiproc", n, "float32", RS)
    ag = la.la_schedule_build(t, "lane_multiproc", n, "float32", AG)
    assert [(x["stage_name"], x["fan_in"], x["fan_out"]) for x in rs.steps()] == [("S1", 8, 1), ("S2a", 4, 1)]
    assert [(x["stage_name"], x["fan_in"], x["fan_out"]) for x in ag.steps()] == [("S2b", 1, 3), ("S3", 1, 7)]
    P = 32
    r_rs, w_rs = totals(rs)
    r_ag, w_ag = totals(ag)
    assert (r_rs, w_rs) == (4 * (8 * n + 4 * n // 4 * 1) * e // 1 - 0, 4 * (n + n // 4) * e)
    assert (r_ag, w_ag) == (4 * (n // 4 + n) * e, 4 * (3 * n // 4 + 7 * n) * e)
    ring_rs = la.la_schedule_build(t, "ring", n, "float32", RS)
    ring_ag = la.la_schedule_build(t, "ring", n, "float32", AG)
    assert ring_rs.num_steps == ring_ag.num_steps == P - 1
    assert {x["stage_name"] for x in ring_rs.steps()} == {"ring-RS"} and {x["stage_name"] for x in ring_ag.steps()} == {"ring-AG"}
    lane = la.la_schedule_build(t, "lane", n, "float32", RS)
    # the C call reports the count whatever the capacity and writes at most `capacity` pairs
    import ctypes
    sh = la.la_schedule_build(t, "lane_multiproc", n, "float32", RS | SHARED)     # 2 processes: 2 ranges per buffer
    offs, lens = (ctypes.c_uint64 * 4)(9, 9, 9, 9), (ctypes.c_uint64 * 4)(9, 9, 9, 9)
    L = la.lib()
    assert L.la_schedule_owned_ranges(sh.handle, 0, 0, None, None) == 2
    assert L.la_schedule_owned_ranges(sh.handle, 0, 1, offs, lens) == 2 and (offs[1], lens[1]) == (9, 9) and lens[0] == n // 32
    assert L.la_schedule_owned_ranges(sh.handle, 0, 4, offs, lens) == 2 and offs[1] == n // 2 and offs[2] == 9
    assert L.la_schedule_owned_ranges(sh.handle, 99, 4, offs, lens) == -1 and L.la_schedule_owned_ranges(None, 0, 0, None, None) == -1
    assert L.la_schedule_step_group(sh.handle, 0) == 4 and L.la_schedule_step_group(sh.handle, 9) == -1
    assert [lane.owned_ranges(r) for r in (1, 3, 5)] == [[], [], []]           # only the leader of a GPU owns data
    assert lane.owned_ranges(2) == [(n // 4, n // 16)]


def test_hazard_freedom_every_step_reads_no_range_another_segment_writes():
    for algo, flags, (N, G, Q), n in itertools.product(ALGOS, FLAG_SETS, [(2, 2, 2), (3, 1, 2), (2, 3, 1)], (7, 48)):
        sched = la.la_schedule_build(la.la_topology_create(N, G, Q), algo, n, "float32", flags)
        for i in range(sched.num_steps):
            t = sched.step_table(i)
            writes, reads = {}, []
            for g in range(t["num_segments"]):
                ln = int(t["seg_len"][g])
                for b, o in zip(t["dst_buf"][g], t["dst_off"][g]):
                    for e in range(int(o), int(o) + ln):
                        assert (int(b), e) not in writes, "two writers"
                        writes[(int(b), e)] = g
                for b, o in zip(t["src_buf"][g], t["src_off"][g]):
                    reads.append((int(b), int(o), ln, g, [int(v) for v in t["src_off"][g]]))
            for b, o, ln, g, _ in reads:
                for e in range(o, o + ln):
                    w = writes.get((b, e))
                    assert w is None or w == g, "a segment reads what another one writes"


# ----------------------------------------------------------------------------- shapes and bytes

def totals(sched):
    rd = sum(s["bytes_read"] for s in sched.steps())
    wr = sum(s["bytes_written"] for s in sched.steps())
    return rd, wr


@pytest.mark.parametrize("topo,algo,n,e,dtype", [
    ((2, 4, 1), "lane", 65536, 4, "float32"),
    ((4, 4, 1), "lane", 1 << 24, 4, "float32"),
    ((8, 4, 4), "lane_multiproc", 1 << 22, 4, "float32"),
    ((2, 4, 2), "lane_multiproc", 1 << 27, 2, "bfloat16"),
    ((32, 4, 8), "lane_multiproc", 1 << 20, 4, "float32"),
])
def test_lane_bytes_match_closed_forms(topo, algo, n, e, dtype):
    N, G, Q = topo
    P = N * G * Q
    t = la.la_topology_create(*topo)
    unit = n * e
    # one copy per (source, destination): S1, S2a, S2b, S3
    s = la.la_schedule_build(t, algo, n, dtype, la.LA_SCHED_P2P_GATHER)
    st = {x["stage"]: x for x in s.steps()}
    assert [x["stage"] for x in s.steps()] == [la.LA_STAGE_S1, la.LA_STAGE_S2A, la.LA_STAGE_S2B, la.LA_STAGE_S3]
    assert (st[la.LA_STAGE_S1]["bytes_read"], st[la.LA_STAGE_S1]["bytes_written"]) == (P * unit, N * unit)
    assert (st[la.LA_STAGE_S2A]["bytes_read"], st[la.LA_STAGE_S2A]["bytes_written"]) == (N * unit, unit)
    assert (st[la.LA_STAGE_S2B]["bytes_read"], st[la.LA_STAGE_S2B]["bytes_written"]) == ((N - 1) * unit, (N - 1) * unit)
    assert (st[la.LA_STAGE_S3]["bytes_read"], st[la.LA_STAGE_S3]["bytes_written"]) == ((P - N) * unit, (P - N) * unit)
    assert sum(totals(s)) == (3 * P + 2 * N - 1) * unit
    # multi-destination stores: every reduced range is read once
    d = la.la_schedule_build(t, algo, n, dtype)
    assert [x["stage"] for x in d.steps()] == [la.LA_STAGE_S1, la.LA_STAGE_S2, la.LA_STAGE_S3]
    assert totals(d) == ((P + 2 * N) * unit, (P + N) * unit)


def test_ring_bytes_match_closed_form():
    P, n, e = 16, 1 << 24, 4
    s = la.la_schedule_build(la.la_topology_create(4, 4, 1), "ring", n, "float32")
    assert s.num_steps == 2 * (P - 1)
    kinds = [x["stage"] for x in s.steps()]
    assert kinds == [la.LA_STAGE_RING_RS] * (P - 1) + [la.LA_STAGE_RING_AG] * (P - 1)
    assert all(x["num_segments"] == P and x["seg_len_max"] == n // P for x in s.steps())
    assert all(x["fan_in"] == 2 for x in s.steps()[: P - 1]) and all(x["fan_in"] == 1 for x in s.steps()[P - 1:])
    assert sum(totals(s)) == 5 * (P - 1) * n * e


def test_scale_out_shape_segment_counts_and_fan_in():
    t = la.la_topology_create(32, 4, 8)
    s = la.la_schedule_build(t, "lane_multiproc", 1 << 20, "float32", la.LA_SCHED_P2P_GATHER)
    by = {x["stage"]: x for x in s.steps()}
    assert (by[la.LA_STAGE_S1]["num_segments"], by[la.LA_STAGE_S1]["fan_in"], by[la.LA_STAGE_S1]["seg_len_max"]) == (1024, 32, 32768)
    assert (by[la.LA_STAGE_S2A]["num_segments"], by[la.LA_STAGE_S2A]["fan_in"], by[la.LA_STAGE_S2A]["seg_len_max"]) == (1024, 32, 1024)
    assert (by[la.LA_STAGE_S2B]["num_segments"], by[la.LA_STAGE_S2B]["seg_len_max"]) == (31744, 1024)
    assert (by[la.LA_STAGE_S3]["num_segments"], by[la.LA_STAGE_S3]["seg_len_max"]) == (31744, 32768)
    d = la.la_schedule_build(t, "lane_multiproc", 1 << 20, "float32")
    by = {x["stage"]: x for x in d.steps()}
    assert (by[la.LA_STAGE_S2]["num_segments"], by[la.LA_STAGE_S2]["fan_in"], by[la.LA_STAGE_S2]["fan_out"]) == (1024, 32, 32)
    assert (by[la.LA_STAGE_S3]["num_segments"], by[la.LA_STAGE_S3]["fan_in"], by[la.LA_STAGE_S3]["fan_out"]) == (1024, 1, 31)


def test_inner_ring_shape_and_bytes():
    N, G, Q, n, e = 8, 4, 4, 1 << 22, 4
    P = N * G * Q
    s = la.la_schedule_build(la.la_topology_create(N, G, Q), "lane_multiproc", n, "float32", la.LA_SCHED_INNER_RING)
    stages = [x["stage"] for x in s.steps()]
    assert stages == [la.LA_STAGE_S1] + [la.LA_STAGE_S2_RING_RS] * (N - 1) + [la.LA_STAGE_S2_RING_AG] * (N - 1) + [la.LA_STAGE_S3]
    piece = n // (G * Q) // N
    for x in s.steps()[1:-1]:
        assert (x["num_segments"], x["seg_len_max"]) == (P, piece)   # every rank moves one piece per iteration
    # inter-node stage: 2 reads + 1 write per reduce iteration, 1 + 1 per gather iteration, of N*n/N each
    inner = sum(x["bytes_read"] + x["bytes_written"] for x in s.steps()[1:-1])
    assert inner == 5 * (N - 1) * n * e
    # the flat ring ignores the flag
    a = la.la_schedule_build(la.la_topology_create(2, 2, 1), "ring", 64, "float32", la.LA_SCHED_INNER_RING)
    b = la.la_schedule_build(la.la_topology_create(2, 2, 1), "ring", 64, "float32")
    assert a.num_steps == b.num_steps
    for i in range(a.num_steps):
        ta, tb = a.step_table(i), b.step_table(i)
        assert all(np.array_equal(ta[key], tb[key]) for key in ta)


def test_lane_tables_equal_lane_multiproc_tables_with_one_process_per_gpu():
    t = la.la_topology_create(3, 4, 1)
    for flags in FLAG_SETS:
        a = la.la_schedule_build(t, "lane", 1000, "float32", flags)
        b = la.la_schedule_build(t, "lane_multiproc", 1000, "float32", flags)
        assert a.num_steps == b.num_steps
        for i in range(a.num_steps):
            ta, tb = a.step_table(i), b.step_table(i)
            for key in ta:
                assert np.array_equal(ta[key], tb[key]), key


def test_degenerate_topologies():
    one = la.la_schedule_build(la.la_topology_create(1, 1, 1), "lane", 100, "float32")
    assert one.num_steps == 0  # a single rank: nothing to do
    assert la.la_schedule_build(la.la_topology_create(1, 1, 1), "ring", 100, "float32").num_steps == 0
    single_node = la.la_schedule_build(la.la_topology_create(1, 4, 2), "lane_multiproc", 100, "float32")
    assert [x["stage"] for x in single_node.steps()] == [la.LA_STAGE_S1, la.LA_STAGE_S3]
    only_nodes = la.la_schedule_build(la.la_topology_create(5, 1, 1), "lane", 100, "float32")
    assert [x["stage"] for x in only_nodes.steps()] == [la.LA_STAGE_S2]
    # fewer elements than parts: empty parts vanish from the tables
    tiny = la.la_schedule_build(la.la_topology_create(2, 3, 2), "lane_multiproc", 3, "int32")
    assert all(x["num_segments"] <= 6 for x in tiny.steps())


def test_staged_schedule_reads_remote_operands_only_from_staging():
    N, G, Q, n = 2, 2, 2, 64
    P = N * G * Q
    s = la.la_schedule_build(la.la_topology_create(N, G, Q), "lane_multiproc", n, "float32", la.LA_SCHED_STAGED)
    assert s.staging_elems > 0
    stages = [x["stage"] for x in s.steps()]
    assert stages == [la.LA_STAGE_PACK, la.LA_STAGE_S1, la.LA_STAGE_PACK, la.LA_STAGE_S2, la.LA_STAGE_S3]
    for i, x in enumerate(s.steps()):
        t = s.step_table(i)
        if x["stage"] in (la.LA_STAGE_S1, la.LA_STAGE_S2):
            for g in range(t["num_segments"]):
                home = int(t["dst_buf"][g][0])
                assert all(int(b) in (home, P) for b in t["src_buf"][g])
                assert sum(int(b) == home for b in t["src_buf"][g]) == 1
        if x["stage"] == la.LA_STAGE_PACK:
            assert np.all(t["dst_buf"] == P) and np.all(t["src_buf"] < P)
