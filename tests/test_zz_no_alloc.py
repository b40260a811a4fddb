"""la_reduce_segments_static (the entry point that allocates nothing: its tables live in a static
device array) against la_reduce_segments, through the C ABI, bit for bit, and against the CPU
oracle; two calls in a row, the second with a smaller input, so that what the first call left in
the shared array must not show."""
import numpy as np
import pytest

import paper_2508_13397_amd as la
from paper_2508_13397_amd import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

NAME = {np.dtype(np.int32): "int32", np.dtype(np.float32): "float32", np.dtype(np.uint16): "bfloat16"}


def to_dev(row):
    if row.dtype == np.uint16:
        return torch.from_numpy(row.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(row).cuda()


def to_host(t):
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def inputs(kind, P, n, seed):
    if kind == "i32":
        return np.random.default_rng(seed).integers(-(1 << 31), 1 << 31, size=(P, n), dtype=np.int64).astype(np.int32)
    if kind == "f32":
        return synth.order_sensitive_f32(P, n)
    return synth.make_inputs(P, n, "normal_bf16", seed=synth.BASE_SEED + seed)


def run_both(oracle, kind, k, n, offs, seg_len, shifts=None, op="sum"):
    """the same call through both entry points on separate copies of dst; returns nothing, asserts"""
    if not torch.cuda.is_available():
        pytest.fail("this test needs a GPU")
    x = inputs(kind, k + 1, n + 8, seed=k)
    shifts = shifts or [0] * (k + 1)
    rows = [x[t][shifts[t]: shifts[t] + n] for t in range(k + 1)]
    full = [to_dev(x[t]) for t in range(k + 1)]
    views = [full[t][shifts[t]: shifts[t] + n] for t in range(k + 1)]
    dst_a = views[0].clone() if shifts[0] == 0 else None
    if dst_a is None:  # keep the destination's own misalignment in the copy as well
        base = full[0].clone()
        dst_a = base[shifts[0]: shifts[0] + n]
    dst_b = views[0]
    stream = torch.cuda.current_stream().cuda_stream
    srcs = [v.data_ptr() for v in views[1:]]
    print("reduce_segments_static", kind, "k", k, "n", n, "segments", len(offs), "len", seg_len, "shifts", shifts, flush=True)
    la.la_reduce_segments(dst_a.data_ptr(), srcs, offs, seg_len, NAME[x.dtype], la.OPS[op], stream)
    la.la_reduce_segments_static(dst_b.data_ptr(), srcs, offs, seg_len, NAME[x.dtype], la.OPS[op], stream)
    torch.cuda.synchronize()
    a, b = to_host(dst_a), to_host(dst_b)
    assert np.array_equal(a.view(np.uint8), b.view(np.uint8)), "static entry point differs from la_reduce_segments"
    ref = oracle.reduce_segments(rows[0], rows[1:], offs, seg_len, op=op)
    assert np.array_equal(b.view(np.uint8), ref.view(np.uint8)), "static entry point differs from the oracle"


@pytest.mark.parametrize("kind", ["i32", "f32", "bf16"])
def test_static_entry_point_two_calls_second_smaller(oracle, kind):
    # first call: 700 segments (two fill launches), fan-in 9, ragged lengths, several tiles per segment
    n = 700 * 6000 + 100
    run_both(oracle, kind, 8, n, [i * 6000 + (i % 7) for i in range(700)], 5003)
    # second call, smaller in every respect: 3 segments, fan-in 3, short; the array still holds call one's tables
    run_both(oracle, kind, 2, 40000, [5, 9001, 30000], 777)
    # and a third with operands that disagree modulo 16 bytes (unaligned path) and another operation
    run_both(oracle, kind, 3, 50000, [0, 20000], 12345, shifts=[0, 1, 2, 3], op="max")


def test_static_entry_point_limits_and_errors():
    if not torch.cuda.is_available():
        pytest.fail("this test needs a GPU")
    d = torch.zeros(1 << 16, dtype=torch.float32, device="cuda")
    s = [torch.ones(1 << 16, dtype=torch.float32, device="cuda") for _ in range(65)]
    ptrs = [t.data_ptr() for t in s]
    with pytest.raises(la.LaError) as ei:  # more sources than the limit
        la.la_reduce_segments_static(d.data_ptr(), ptrs, [0], 16, "float32")
    assert ei.value.status == la.LA_ERR_INVALID_ARG and "64" in str(ei.value)
    with pytest.raises(la.LaError) as ei:  # more segments than the limit
        la.la_reduce_segments_static(d.data_ptr(), ptrs[:1], list(range(0, 8193 * 4, 4)), 4, "float32")
    assert ei.value.status == la.LA_ERR_INVALID_ARG
    with pytest.raises(la.LaError) as ei:  # tables beyond the static array: 8192 * (32 + 8 * 33) > 1 MiB
        la.la_reduce_segments_static(d.data_ptr(), ptrs[:32], list(range(0, 8192 * 4, 4)), 4, "float32")
    assert ei.value.status == la.LA_ERR_INVALID_ARG and "static scratch" in str(ei.value)
    with pytest.raises(la.LaError):  # overlapping segments
        la.la_reduce_segments_static(d.data_ptr(), ptrs[:1], [0, 8], 16, "float32")
    with pytest.raises(la.LaError):  # a source that is the destination
        la.la_reduce_segments_static(d.data_ptr(), [d.data_ptr()], [0], 16, "float32")
    torch.cuda.synchronize()
    assert float(d.abs().sum()) == 0.0  # nothing ran
    # the largest accepted table: 8192 segments, fan-in 11 + the owned range (8192 * (32 + 8 * 12) = 1 MiB exactly)
    la.la_reduce_segments_static(d.data_ptr(), ptrs[:11], list(range(0, 8192 * 8, 8)), 8, "float32")
    torch.cuda.synchronize()
    assert float(d.min()) == 11.0 and float(d.max()) == 11.0


def test_static_entry_point_recorded_into_a_callers_graph(oracle):
    """What the entry point is for: a caller under graph capture.  After one eager call (which
    looks up the array's device address), a call is recorded with torch.cuda.graph together with
    the copy that restores dst, and replayed three times with eager calls of other shapes (which
    rewrite the shared array) in between: every replay must give the oracle's bits."""
    if not torch.cuda.is_available():
        pytest.fail("this test needs a GPU")
    k, n, seg_len = 5, 300000, 4001
    offs = [i * 5000 + (i % 5) for i in range(55)]
    x = inputs("f32", k + 1, n, seed=3)
    ref = oracle.reduce_segments(x[0], list(x[1:]), offs, seg_len)
    dev = [to_dev(x[t]) for t in range(k + 1)]
    dst0 = dev[0].clone()
    srcs = [t.data_ptr() for t in dev[1:]]
    run_both(oracle, "f32", 2, 40000, [5, 9001, 30000], 777)  # eager: the symbol lookup happens here
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        dev[0].copy_(dst0)
        la.la_reduce_segments_static(dev[0].data_ptr(), srcs, offs, seg_len, "float32", la.LA_SUM,
                                     torch.cuda.current_stream().cuda_stream)
    for replay in range(3):
        run_both(oracle, "i32", 3, 50000, [0, 20000], 1234 + replay)  # other tables pass through the array
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(to_host(dev[0]).view(np.uint8), ref.view(np.uint8)), replay
