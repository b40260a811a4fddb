"""CPU oracle for the emulated lane-aware all-reduce (ctypes wrapper around la_oracle.c).

TEST INFRASTRUCTURE ONLY: the tests, the smoke check and the benchmark's CPU-baseline leg
import this package; the product package never does.  Nothing here touches a GPU.

`build()` compiles la_oracle.c with gcc; the functions below load the built library lazily.
Buffers are numpy arrays: int32, float32, or uint16 holding bf16 bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "la_oracle.c")
_LIB = os.path.join(_HERE, "libla_oracle.so")

I32, F32, BF16, F16, F64 = 0, 1, 2, 3, 4
OPS = {"sum": 0, "prod": 1, "max": 2, "min": 3}
RING, LANE, LANE_MULTIPROC, LANE_RING, LANE_MULTIPROC_RING = 0, 1, 2, 3, 4
RECURSIVE_DOUBLING, RABENSEIFNER = 5, 6
ALGOS = {"ring": RING, "lane": LANE, "lane_multiproc": LANE_MULTIPROC, "lane_ring": LANE_RING,
         "lane_multiproc_ring": LANE_MULTIPROC_RING, "recursive_doubling": RECURSIVE_DOUBLING,
         "rabenseifner": RABENSEIFNER}

# phases in the message trace
PH_LANE_S1, PH_LANE_S2A, PH_LANE_S2B, PH_LANE_S3, PH_RING_RS, PH_RING_AG = 1, 2, 3, 4, 10, 11
PH_LANE_S2_RING_RS, PH_LANE_S2_RING_AG = 5, 6
PH_RECURSIVE_DOUBLING, PH_RABENSEIFNER_RS, PH_RABENSEIFNER_AG = 20, 21, 22

MSG_DTYPE = np.dtype(
    [("phase", "<i4"), ("step", "<i4"), ("src", "<i4"), ("dst", "<i4"), ("off", "<u8"), ("cnt", "<u8")]
)


def build(force: bool = True, src: str = _SRC, lib: str = _LIB) -> str:
    """Compile the oracle (plain C, no fast-math, no contraction)."""
    if force or not os.path.exists(lib) or os.path.getmtime(lib) < os.path.getmtime(src):
        cmd = ["gcc", "-O2", "-std=c99", "-fno-fast-math", "-ffp-contract=off", "-fopenmp",
               "-fPIC", "-shared", "-Wall", "-Wextra", "-o", lib, src]
        subprocess.run(cmd, check=True)
    return lib


def dtype_code(arr: np.ndarray) -> int:
    table = {np.dtype(np.int32): I32, np.dtype(np.float32): F32, np.dtype(np.uint16): BF16,
             np.dtype(np.float16): F16, np.dtype(np.float64): F64}
    if arr.dtype not in table:
        raise TypeError("oracle buffers must be int32, float32, float16, float64 or uint16 (bf16 bits), "
                        f"not {arr.dtype}")
    return table[arr.dtype]


def _row_ptrs(rows):
    arr = (ctypes.c_void_p * len(rows))()
    for i, r in enumerate(rows):
        assert r.flags["C_CONTIGUOUS"] and r.ndim == 1
        arr[i] = r.ctypes.data
    return arr


class Oracle:
    """The functions of one built oracle library.  The module-level functions below use the
    library built from la_oracle.c; tests that plant mistakes load their own build."""

    I32, F32, BF16 = I32, F32, BF16
    PH_LANE_S1, PH_LANE_S2A, PH_LANE_S2B, PH_LANE_S3 = PH_LANE_S1, PH_LANE_S2A, PH_LANE_S2B, PH_LANE_S3
    PH_RING_RS, PH_RING_AG = PH_RING_RS, PH_RING_AG
    PH_LANE_S2_RING_RS, PH_LANE_S2_RING_AG = PH_LANE_S2_RING_RS, PH_LANE_S2_RING_AG
    PH_RECURSIVE_DOUBLING, PH_RABENSEIFNER_RS, PH_RABENSEIFNER_AG = 20, 21, 22

    def __init__(self, libpath: str):
        lib = ctypes.CDLL(libpath)
        u64, i32, vp = ctypes.c_uint64, ctypes.c_int, ctypes.c_void_p
        lib.oracle_allreduce.argtypes = [i32, i32, i32, i32, u64, i32, ctypes.POINTER(vp), i32,
                                         vp, u64, ctypes.POINTER(u64)]
        lib.oracle_allreduce.restype = i32
        lib.oracle_allreduce_shared.argtypes = lib.oracle_allreduce.argtypes
        lib.oracle_allreduce_shared.restype = i32
        lib.oracle_allreduce_op.argtypes = [i32, i32] + list(lib.oracle_allreduce.argtypes)
        lib.oracle_allreduce_op.restype = i32
        lib.oracle_definition_reduce.argtypes = [i32, i32, i32, u64, ctypes.POINTER(vp), vp]
        lib.oracle_definition_reduce.restype = i32
        lib.oracle_reduce_segments_op.argtypes = [i32, i32, vp, ctypes.POINTER(vp), i32, vp, u64, u64]
        lib.oracle_reduce_segments_op.restype = i32
        lib.oracle_f16_round.argtypes = [vp, vp, u64]
        lib.oracle_f16_widen.argtypes = [vp, vp, u64]
        lib.oracle_bf16_round.argtypes = [vp, vp, u64]
        lib.oracle_bf16_widen.argtypes = [vp, vp, u64]
        lib.oracle_part.argtypes = [u64, u64, u64, ctypes.POINTER(u64), ctypes.POINTER(u64)]
        lib.oracle_set_threads.argtypes = [i32]
        lib.oracle_max_threads.restype = i32
        self.lib = lib

    def set_threads(self, t: int) -> None:
        self.lib.oracle_set_threads(int(t))

    def max_threads(self) -> int:
        return int(self.lib.oracle_max_threads())

    def allreduce(self, algo, N: int, G: int, Q: int, inputs, max_rounds: int = -1,
                  want_trace: bool = False, in_place: bool = False, shared: bool = False, op="sum"):
        """Simulate a schedule over the rank buffers `inputs` (a 2-D array or a list of 1-D
        arrays): P = N*G*Q private buffers, or with shared=True the N*G per-GPU buffers that the
        Q processes of a GPU share.  Returns the result (and the message trace when asked)."""
        algo = ALGOS[algo] if isinstance(algo, str) else int(algo)
        P = N * G * (1 if shared else Q)
        if isinstance(inputs, np.ndarray):
            assert inputs.ndim == 2 and inputs.shape[0] == P
            work = inputs if in_place else inputs.copy()
            rows = [work[r] for r in range(P)]
        else:
            assert len(inputs) == P
            rows = list(inputs) if in_place else [np.array(r, copy=True) for r in inputs]
            work = rows
        n = rows[0].shape[0]
        assert all(r.shape[0] == n and r.dtype == rows[0].dtype for r in rows)
        ptrs = _row_ptrs(rows)
        tlen = ctypes.c_uint64(0)
        trace, cap = None, 0
        if want_trace:
            # generous bound: ring sends 2(P-1)P messages, lane fewer than 4 P max(R, N)
            cap = 4 * (N * G * Q) * max(N * G * Q, 2) + 16
            trace = np.zeros(cap, dtype=MSG_DTYPE)
        opc = OPS[op] if isinstance(op, str) else int(op)
        rc = self.lib.oracle_allreduce_op(1 if shared else 0, opc, algo, N, G, Q, n, dtype_code(rows[0]), ptrs,
                                          int(max_rounds), trace.ctypes.data if want_trace else None, cap,
                                          ctypes.byref(tlen))
        if rc != 0:
            raise RuntimeError(f"oracle_allreduce failed with code {rc}")
        if want_trace:
            assert tlen.value <= cap
            return work, trace[: tlen.value]
        return work

    def definition_reduce(self, inputs, op="sum"):
        """The all-reduce by its definition: int32 -> int32 (exact, wrapped); floats -> float64."""
        rows = [np.ascontiguousarray(inputs[r]) for r in range(len(inputs))]
        n = rows[0].shape[0]
        code = dtype_code(rows[0])
        out = np.empty(n, dtype=np.int32 if code == I32 else np.float64)
        opc = OPS[op] if isinstance(op, str) else int(op)
        rc = self.lib.oracle_definition_reduce(code, opc, len(rows), n, _row_ptrs(rows), out.ctypes.data)
        if rc != 0:
            raise RuntimeError(f"oracle_definition_reduce failed with code {rc}")
        return out

    def definition_sum(self, inputs):
        return self.definition_reduce(inputs, "sum")

    def reduce_segments(self, dst: np.ndarray, srcs, seg_offsets, seg_len: int, op="sum") -> np.ndarray:
        """dst[o] = ((dst[o] + srcs[0][o]) + srcs[1][o]) + ... over every segment; a copy."""
        out = dst.copy()
        offs = np.ascontiguousarray(seg_offsets, dtype=np.uint64)
        srcs = [np.ascontiguousarray(s) for s in srcs]
        ptrs = _row_ptrs(srcs) if srcs else (ctypes.c_void_p * 1)()
        opc = OPS[op] if isinstance(op, str) else int(op)
        rc = self.lib.oracle_reduce_segments_op(dtype_code(out), opc, out.ctypes.data, ptrs, len(srcs),
                                                offs.ctypes.data, len(offs), int(seg_len))
        if rc != 0:
            raise RuntimeError(f"oracle_reduce_segments failed with code {rc}")
        return out

    def bf16_round(self, x: np.ndarray) -> np.ndarray:
        x = np.ascontiguousarray(x, dtype=np.float32)
        out = np.empty(x.shape, dtype=np.uint16)
        self.lib.oracle_bf16_round(x.ctypes.data, out.ctypes.data, x.size)
        return out

    def bf16_widen(self, h: np.ndarray) -> np.ndarray:
        h = np.ascontiguousarray(h, dtype=np.uint16)
        out = np.empty(h.shape, dtype=np.float32)
        self.lib.oracle_bf16_widen(h.ctypes.data, out.ctypes.data, h.size)
        return out

    def f16_round(self, x: np.ndarray) -> np.ndarray:
        x = np.ascontiguousarray(x, dtype=np.float32)
        out = np.empty(x.shape, dtype=np.uint16)
        self.lib.oracle_f16_round(x.ctypes.data, out.ctypes.data, x.size)
        return out

    def f16_widen(self, h: np.ndarray) -> np.ndarray:
        h = np.ascontiguousarray(h, dtype=np.uint16)
        out = np.empty(h.shape, dtype=np.float32)
        self.lib.oracle_f16_widen(h.ctypes.data, out.ctypes.data, h.size)
        return out

    def part(self, length: int, m: int, i: int):
        off, cnt = ctypes.c_uint64(), ctypes.c_uint64()
        self.lib.oracle_part(length, m, i, ctypes.byref(off), ctypes.byref(cnt))
        return off.value, cnt.value


_default = None


def default() -> Oracle:
    global _default
    if _default is None:
        build(force=False)
        _default = Oracle(_LIB)
    return _default


def set_threads(t):
    default().set_threads(t)


def max_threads():
    return default().max_threads()


def allreduce(*a, **k):
    return default().allreduce(*a, **k)


def definition_sum(inputs):
    return default().definition_sum(inputs)


def reduce_segments(dst, srcs, seg_offsets, seg_len, op="sum"):
    return default().reduce_segments(dst, srcs, seg_offsets, seg_len, op)


def definition_reduce(inputs, op="sum"):
    return default().definition_reduce(inputs, op)


def bf16_round(x):
    return default().bf16_round(x)


def bf16_widen(h):
    return default().bf16_widen(h)


def part(length, m, i):
    return default().part(length, m, i)
