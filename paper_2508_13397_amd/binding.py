"""ctypes binding of liblaneallreduce.so: the same names as include/lane_allreduce.h, argument
marshalling only.  Every step of the all-reduce runs in the library's HIP kernels; there is no
fallback: if the library has not been built, or a call fails, an exception is raised."""
from __future__ import annotations

import ctypes
import importlib.util
import os
import sys
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblaneallreduce.so")

LA_OK, LA_ERR_INVALID_ARG, LA_ERR_UNSUPPORTED, LA_ERR_OUT_OF_MEMORY, LA_ERR_DEVICE = range(5)
LA_ALGO_RING, LA_ALGO_LANE, LA_ALGO_LANE_MULTIPROC = 0, 1, 2
LA_ALGO_RECURSIVE_DOUBLING, LA_ALGO_RABENSEIFNER = 3, 4
LA_I32, LA_F32, LA_BF16, LA_F16, LA_F64 = 0, 1, 2, 3, 4
LA_SUM, LA_PROD, LA_MAX, LA_MIN = 0, 1, 2, 3
OPS = {"sum": LA_SUM, "prod": LA_PROD, "max": LA_MAX, "min": LA_MIN}
LA_SCHED_DEFAULT, LA_SCHED_P2P_GATHER, LA_SCHED_STAGED, LA_SCHED_INNER_RING = 0, 1, 2, 4
LA_SCHED_SHARED_BUFFERS, LA_SCHED_OUT_OF_PLACE = 8, 16
LA_SCHED_ONLY_REDUCE_SCATTER, LA_SCHED_ONLY_ALLGATHER = 32, 64
LA_SCHED_FUSED_GATHER, LA_SCHED_SINGLE_LAUNCH = 128, 256
LA_STEP_REDUCE, LA_STEP_COPY = 0, 1
LA_STAGE_S1, LA_STAGE_S2A, LA_STAGE_S2B, LA_STAGE_S3, LA_STAGE_S2 = 1, 2, 3, 4, 5
LA_STAGE_RING_RS, LA_STAGE_RING_AG, LA_STAGE_PACK = 10, 11, 20
LA_STAGE_S2_RING_RS, LA_STAGE_S2_RING_AG = 6, 7
LA_STAGE_S2_S3, LA_STAGE_S1_S3, LA_STAGE_S1_S2_S3 = 8, 9, 15
LA_STAGE_COPY_INPUT = 21
LA_STAGE_RECURSIVE_DOUBLING, LA_STAGE_RABENSEIFNER_RS, LA_STAGE_RABENSEIFNER_AG = 12, 13, 14

ALGOS = {"ring": LA_ALGO_RING, "lane": LA_ALGO_LANE, "lane_multiproc": LA_ALGO_LANE_MULTIPROC,
         "recursive_doubling": LA_ALGO_RECURSIVE_DOUBLING, "rabenseifner": LA_ALGO_RABENSEIFNER}
DTYPES = {"int32": LA_I32, "float32": LA_F32, "bfloat16": LA_BF16, "float16": LA_F16, "float64": LA_F64}
ELEM_SIZE = {LA_I32: 4, LA_F32: 4, LA_BF16: 2, LA_F16: 2, LA_F64: 8}
STAGE_NAMES = {21: "copy-input", 12: "rec-doubling", 13: "rabenseifner-RS", 14: "rabenseifner-AG", 1: "S1", 2: "S2a", 3: "S2b", 4: "S3", 5: "S2", 6: "S2-ring-RS", 7: "S2-ring-AG", 8: "S2+S3", 9: "S1+S3", 15: "S1+S2+S3", 10: "ring-RS",
               11: "ring-AG", 20: "pack"}

# every symbol include/lane_allreduce.h declares
EXPORTS = (
    "la_topology_create", "la_topology_destroy", "la_topology_num_ranks",
    "la_schedule_build", "la_schedule_build_ex", "la_schedule_destroy", "la_schedule_num_steps",
    "la_schedule_num_buffers", "la_schedule_owned_ranges", "la_schedule_step_group",
    "la_schedule_staging_elems", "la_schedule_step_info", "la_schedule_step_table",
    "la_allreduce_emulated", "la_allreduce_emulated_out_of_place", "la_schedule_run_step", "la_schedule_run_steps", "la_reduce_segments",
    "la_reduce_segments_static",
    "la_schedule_launch_plan", "la_schedule_launch_segments", "la_schedule_fusion_runs", "la_schedule_fusion_info",
    "la_schedule_fusion_table",
    "la_status_string", "la_last_error", "la_tuning_set", "la_tuning_get",
)


class LaunchPlan(ctypes.Structure):
    """la_launch_plan_t"""
    _fields_ = [("block", ctypes.c_int), ("unroll", ctypes.c_int), ("cache_policy", ctypes.c_int),
                ("tiling", ctypes.c_int), ("tiles_per_segment", ctypes.c_uint32),
                ("edge_workgroups", ctypes.c_uint32), ("workgroups", ctypes.c_uint64)]


class LaError(RuntimeError):
    def __init__(self, status: int, where: str, detail: str):
        super().__init__(f"{where}: {detail}")
        self.status = status


_lib = None


def _share_hip_runtime_with_torch() -> None:
    """PyTorch-ROCm ships a HIP runtime of its own under the system runtime's soname.  Whichever of
    the two is loaded first serves every later user of that soname; if this library pulled in the
    system's and torch then brought its own (with its own HSA runtime), the process would hold two,
    and the second finds no device.  So where torch is installed it is imported before the library
    is loaded, and both use torch's."""
    if "torch" not in sys.modules and importlib.util.find_spec("torch") is not None:
        import torch  # noqa: F401


def lib() -> ctypes.CDLL:
    """Load the built library; raise loudly when it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} has not been built; run `python -m paper_2508_13397_amd.build` "
            "(hipcc, gfx950). There is no CPU fallback.")
    _share_hip_runtime_with_torch()
    L = ctypes.CDLL(LIB_PATH)
    vp, i32, u32, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_uint, ctypes.c_size_t
    pp = ctypes.POINTER
    L.la_topology_create.argtypes = [i32, i32, i32, pp(vp)]
    L.la_topology_destroy.argtypes = [vp]
    L.la_topology_num_ranks.argtypes = [vp]
    L.la_schedule_build.argtypes = [vp, i32, sz, i32, pp(vp)]
    L.la_schedule_build_ex.argtypes = [vp, i32, sz, i32, u32, pp(vp)]
    L.la_schedule_destroy.argtypes = [vp]
    L.la_schedule_num_steps.argtypes = [vp]
    L.la_schedule_num_buffers.argtypes = [vp]
    L.la_schedule_owned_ranges.argtypes = [vp, i32, i32, vp, vp]
    L.la_schedule_step_group.argtypes = [vp, i32]
    L.la_schedule_step_group.restype = i32
    L.la_schedule_staging_elems.argtypes = [vp]
    L.la_schedule_staging_elems.restype = sz
    L.la_schedule_step_info.argtypes = [vp, i32, pp(i32), pp(i32), pp(sz), pp(sz), pp(i32), pp(i32), pp(sz), pp(sz)]
    L.la_schedule_step_table.argtypes = [vp, i32, vp, vp, vp, vp, vp]
    L.la_allreduce_emulated.argtypes = [vp, pp(vp), sz, i32, i32, vp]
    L.la_allreduce_emulated_out_of_place.argtypes = [vp, pp(vp), pp(vp), sz, i32, i32, vp]
    L.la_schedule_run_step.argtypes = [vp, i32, pp(vp), vp]
    L.la_schedule_launch_plan.argtypes = [vp, i32, pp(vp), pp(vp), vp, pp(LaunchPlan)]
    L.la_schedule_launch_segments.argtypes = [vp, i32, pp(vp), pp(vp), vp, sz, pp(sz), vp, vp, vp]
    L.la_schedule_fusion_runs.argtypes = [vp]
    L.la_schedule_fusion_info.argtypes = [vp, i32, pp(i32), pp(i32), pp(ctypes.c_uint64), pp(ctypes.c_uint64), pp(i32),
                                          pp(sz), pp(sz)]
    L.la_schedule_run_steps.argtypes = [vp, i32, i32, pp(vp), i32, vp]
    L.la_schedule_fusion_table.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp, vp]
    L.la_reduce_segments.argtypes = [vp, pp(vp), i32, pp(sz), sz, sz, i32, i32, vp]
    L.la_reduce_segments_static.argtypes = L.la_reduce_segments.argtypes
    L.la_status_string.argtypes = [i32]
    L.la_status_string.restype = ctypes.c_char_p
    L.la_last_error.restype = ctypes.c_char_p
    L.la_tuning_set.argtypes = [ctypes.c_char_p, i32]
    L.la_tuning_get.argtypes = [ctypes.c_char_p]
    _lib = L
    return L


def _check(status: int, where: str) -> None:
    if status != LA_OK:
        L = lib()
        name = L.la_status_string(status).decode()
        raise LaError(status, where, f"{name}: {L.la_last_error().decode()}")


def ptr_array(ptrs):
    """A C array of device addresses; build it once when the same buffers are used repeatedly."""
    if isinstance(ptrs, ctypes.Array):
        return ptrs
    arr = (ctypes.c_void_p * max(len(ptrs), 1))()
    for i, p in enumerate(ptrs):
        arr[i] = p
    return arr


_ptr_array = ptr_array


def la_status_string(status: int) -> str:
    return lib().la_status_string(status).decode()


def la_last_error() -> str:
    return lib().la_last_error().decode()


def la_tuning_set(key: str, value: int) -> None:
    _check(lib().la_tuning_set(key.encode(), int(value)), "la_tuning_set")


def la_tuning_get(key: str) -> int:
    return int(lib().la_tuning_get(key.encode()))


class Topology:
    """la_topology_t"""

    def __init__(self, nodes: int, gpus_per_node: int, procs_per_gpu: int):
        self.handle = ctypes.c_void_p()
        _check(lib().la_topology_create(nodes, gpus_per_node, procs_per_gpu, ctypes.byref(self.handle)),
               "la_topology_create")
        self.nodes, self.gpus_per_node, self.procs_per_gpu = nodes, gpus_per_node, procs_per_gpu

    @property
    def num_ranks(self) -> int:
        return int(lib().la_topology_num_ranks(self.handle))

    def close(self) -> None:
        if self.handle:
            lib().la_topology_destroy(self.handle)
            self.handle = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def la_topology_create(nodes: int, gpus_per_node: int, procs_per_gpu: int) -> Topology:
    return Topology(nodes, gpus_per_node, procs_per_gpu)


class Schedule:
    """la_schedule_t"""

    def __init__(self, topo: Topology, algo, n: int, dtype, flags: int = LA_SCHED_DEFAULT):
        self.algo = ALGOS[algo] if isinstance(algo, str) else int(algo)
        self.dtype = DTYPES[dtype] if isinstance(dtype, str) else int(dtype)
        self.n, self.flags, self.topo = int(n), int(flags), topo
        self.handle = ctypes.c_void_p()
        _check(lib().la_schedule_build_ex(topo.handle, self.algo, self.n, self.dtype, self.flags,
                                          ctypes.byref(self.handle)), "la_schedule_build")

    @property
    def num_steps(self) -> int:
        return int(lib().la_schedule_num_steps(self.handle))

    @property
    def num_buffers(self) -> int:
        return int(lib().la_schedule_num_buffers(self.handle))

    def owned_ranges(self, buffer: int):
        """[(offset, length), ...] that `buffer` holds fully reduced between the two halves"""
        count = lib().la_schedule_owned_ranges(self.handle, buffer, 0, None, None)
        if count < 0:
            raise LaError(LA_ERR_INVALID_ARG, "la_schedule_owned_ranges", "bad buffer index")
        offs = np.zeros(max(count, 1), dtype=np.uint64)
        lens = np.zeros(max(count, 1), dtype=np.uint64)
        lib().la_schedule_owned_ranges(self.handle, buffer, count, offs.ctypes.data, lens.ctypes.data)
        return [(int(offs[i]), int(lens[i])) for i in range(count)]

    @property
    def staging_elems(self) -> int:
        return int(lib().la_schedule_staging_elems(self.handle))

    def step_info(self, step: int) -> dict:
        i32, sz = ctypes.c_int, ctypes.c_size_t
        kind, stage, k, m = i32(), i32(), i32(), i32()
        S, longest, rd, wr = sz(), sz(), sz(), sz()
        _check(lib().la_schedule_step_info(self.handle, step, ctypes.byref(kind), ctypes.byref(stage),
                                           ctypes.byref(S), ctypes.byref(longest), ctypes.byref(k),
                                           ctypes.byref(m), ctypes.byref(rd), ctypes.byref(wr)),
               "la_schedule_step_info")
        return dict(kind=kind.value, stage=stage.value, stage_name=STAGE_NAMES.get(stage.value, "?"),
                    num_segments=S.value, seg_len_max=longest.value, fan_in=k.value, fan_out=m.value,
                    bytes_read=rd.value, bytes_written=wr.value,
                    group=int(lib().la_schedule_step_group(self.handle, step)))

    def step_table(self, step: int) -> dict:
        info = self.step_info(step)
        S, k, m = info["num_segments"], info["fan_in"], info["fan_out"]
        seg_len = np.zeros(S, dtype=np.uint64)
        src_buf = np.zeros((S, k), dtype=np.int32)
        src_off = np.zeros((S, k), dtype=np.uint64)
        dst_buf = np.zeros((S, m), dtype=np.int32)
        dst_off = np.zeros((S, m), dtype=np.uint64)
        _check(lib().la_schedule_step_table(self.handle, step, seg_len.ctypes.data, src_buf.ctypes.data,
                                            src_off.ctypes.data, dst_buf.ctypes.data, dst_off.ctypes.data),
               "la_schedule_step_table")
        info.update(seg_len=seg_len, src_buf=src_buf, src_off=src_off, dst_buf=dst_buf, dst_off=dst_off)
        return info

    def steps(self):
        return [self.step_info(i) for i in range(self.num_steps)]

    def close(self) -> None:
        if self.handle:
            lib().la_schedule_destroy(self.handle)
            self.handle = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def la_schedule_build(topo: Topology, algo, n: int, dtype, flags: int = LA_SCHED_DEFAULT) -> Schedule:
    return Schedule(topo, algo, n, dtype, flags)


def la_allreduce_emulated(sched: Schedule, bufs: Sequence[int], n: int, dtype, op: int = LA_SUM,
                          stream: int = 0) -> None:
    """bufs: P device addresses (e.g. tensor.data_ptr()); stream: a hipStream_t as integer."""
    dtype = DTYPES[dtype] if isinstance(dtype, str) else int(dtype)
    _check(lib().la_allreduce_emulated(sched.handle, _ptr_array(bufs), int(n), dtype, int(op),
                                       ctypes.c_void_p(stream)), "la_allreduce_emulated")


def la_allreduce_emulated_out_of_place(sched: Schedule, sendbufs: Sequence[int], recvbufs: Sequence[int], n: int, dtype,
                                       op: int = LA_SUM, stream: int = 0) -> None:
    dtype = DTYPES[dtype] if isinstance(dtype, str) else int(dtype)
    _check(lib().la_allreduce_emulated_out_of_place(sched.handle, _ptr_array(sendbufs), _ptr_array(recvbufs), int(n),
                                                    dtype, int(op), ctypes.c_void_p(stream)),
           "la_allreduce_emulated_out_of_place")


def la_schedule_run_step(sched: Schedule, step: int, bufs: Sequence[int], stream: int = 0) -> None:
    _check(lib().la_schedule_run_step(sched.handle, int(step), _ptr_array(bufs), ctypes.c_void_p(stream)),
           "la_schedule_run_step")


def la_schedule_run_steps(sched: Schedule, first_step: int, num_steps: int, bufs: Sequence[int], op: int = LA_SUM,
                          stream: int = 0) -> None:
    _check(lib().la_schedule_run_steps(sched.handle, int(first_step), int(num_steps), _ptr_array(bufs), int(op),
                                       ctypes.c_void_p(stream)), "la_schedule_run_steps")


def la_schedule_launch_plan(sched: Schedule, step: int, bufs: Sequence[int], sendbufs: Optional[Sequence[int]] = None,
                            staging: int = 0) -> dict:
    """Host only: how `step` would be launched for buffers at these addresses (never dereferenced)."""
    plan = LaunchPlan()
    _check(lib().la_schedule_launch_plan(sched.handle, int(step), _ptr_array(bufs),
                                         _ptr_array(sendbufs) if sendbufs is not None else None,
                                         ctypes.c_void_p(staging), ctypes.byref(plan)), "la_schedule_launch_plan")
    return {name: int(getattr(plan, name)) for name, _ in LaunchPlan._fields_}


def la_schedule_launch_segments(sched: Schedule, step: int, bufs: Sequence[int],
                                sendbufs: Optional[Sequence[int]] = None, staging: int = 0) -> dict:
    """Host only: the segments of `step` as launched for buffers at these addresses (after merging)."""
    info = sched.step_info(step)
    k, m, cap = info["fan_in"], info["fan_out"], info["num_segments"]
    count = ctypes.c_size_t()
    seg_len = np.zeros(max(cap, 1), dtype=np.uint64)
    src = np.zeros((max(cap, 1), k), dtype=np.uint64)
    dst = np.zeros((max(cap, 1), m), dtype=np.uint64)
    _check(lib().la_schedule_launch_segments(sched.handle, int(step), _ptr_array(bufs),
                                             _ptr_array(sendbufs) if sendbufs is not None else None,
                                             ctypes.c_void_p(staging), cap, ctypes.byref(count), seg_len.ctypes.data,
                                             src.ctypes.data, dst.ctypes.data), "la_schedule_launch_segments")
    c = int(count.value)
    return dict(count=c, seg_len=seg_len[:c], src_addr=src[:c], dst_addr=dst[:c])


def la_schedule_fusion_runs(sched: Schedule) -> int:
    """Host only: how many runs of steps the schedule has that can execute as one launch each."""
    r = int(lib().la_schedule_fusion_runs(sched.handle))
    if r < 0:
        raise LaError(LA_ERR_OUT_OF_MEMORY, "la_schedule_fusion_runs", la_last_error())
    return r


def la_schedule_fusion_table(sched: Schedule, run: int) -> dict:
    """Host only: the chains of one run and their operations."""
    first, steps, auto = ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
    C, O = ctypes.c_uint64(), ctypes.c_uint64()
    rd, wr = ctypes.c_size_t(), ctypes.c_size_t()
    _check(lib().la_schedule_fusion_info(sched.handle, int(run), ctypes.byref(first), ctypes.byref(steps), ctypes.byref(C),
                                         ctypes.byref(O), ctypes.byref(auto), ctypes.byref(rd), ctypes.byref(wr)),
           "la_schedule_fusion_info")
    c, o = int(C.value), int(O.value)
    lo, ln, first_op = np.zeros(c, np.uint64), np.zeros(c, np.uint64), np.zeros(c + 1, np.uint64)
    step, seg, pf, fw = np.zeros(o, np.uint32), np.zeros(o, np.uint32), np.zeros(o, np.int32), np.zeros(o, np.int32)
    _check(lib().la_schedule_fusion_table(sched.handle, int(run), lo.ctypes.data, ln.ctypes.data, first_op.ctypes.data,
                                          step.ctypes.data, seg.ctypes.data, pf.ctypes.data, fw.ctypes.data),
           "la_schedule_fusion_table")
    return dict(first_step=first.value, num_steps=steps.value, automatic=bool(auto.value), bytes_read=rd.value,
                bytes_written=wr.value, chain_lo=lo, chain_len=ln,
                chain_first_op=first_op, op_step=step, op_segment=seg, op_prefetch_source=pf, op_forward_source=fw)


def la_reduce_segments(dst: int, srcs: Sequence[int], seg_offsets: Sequence[int], seg_len: int, dtype,
                       op: int = LA_SUM, stream: int = 0) -> None:
    dtype = DTYPES[dtype] if isinstance(dtype, str) else int(dtype)
    offs = (ctypes.c_size_t * max(len(seg_offsets), 1))(*[int(o) for o in seg_offsets])
    _check(lib().la_reduce_segments(ctypes.c_void_p(dst), _ptr_array(srcs), len(srcs), offs, len(seg_offsets),
                                    int(seg_len), dtype, int(op), ctypes.c_void_p(stream)),
           "la_reduce_segments")


def la_reduce_segments_static(dst: int, srcs: Sequence[int], seg_offsets: Sequence[int], seg_len: int, dtype,
                              op: int = LA_SUM, stream: int = 0) -> None:
    """la_reduce_segments without any allocation (tables in the library's static device array)."""
    dtype = DTYPES[dtype] if isinstance(dtype, str) else int(dtype)
    offs = (ctypes.c_size_t * max(len(seg_offsets), 1))(*[int(o) for o in seg_offsets])
    _check(lib().la_reduce_segments_static(ctypes.c_void_p(dst), _ptr_array(srcs), len(srcs), offs, len(seg_offsets),
                                           int(seg_len), dtype, int(op), ctypes.c_void_p(stream)),
           "la_reduce_segments_static")
