"""MI355X-native emulated lane-aware all-reduce: segmented k-way reduce schedules on one GPU.

The arithmetic lives in liblaneallreduce.so (HIP, gfx950; C ABI in include/lane_allreduce.h);
`binding` mirrors that ABI with ctypes.  PyTorch is used by callers only to allocate device
memory and to provide a stream."""
from .binding import (  # noqa: F401
    ALGOS, DTYPES, ELEM_SIZE, EXPORTS, LA_ALGO_LANE, LA_ALGO_LANE_MULTIPROC, LA_ALGO_RABENSEIFNER, LA_ALGO_RECURSIVE_DOUBLING, LA_ALGO_RING, LA_BF16, LA_F16, LA_F64, LA_MAX, LA_MIN, LA_PROD, OPS,
    LA_ERR_DEVICE, LA_ERR_INVALID_ARG, LA_ERR_OUT_OF_MEMORY, LA_ERR_UNSUPPORTED, LA_F32, LA_I32, LA_OK,
    LA_SCHED_DEFAULT, LA_SCHED_FUSED_GATHER, LA_SCHED_INNER_RING, LA_SCHED_ONLY_ALLGATHER, LA_SCHED_ONLY_REDUCE_SCATTER, LA_SCHED_OUT_OF_PLACE, LA_SCHED_P2P_GATHER, LA_SCHED_SHARED_BUFFERS, LA_SCHED_SINGLE_LAUNCH, LA_SCHED_STAGED, LA_STAGE_COPY_INPUT, LA_STAGE_PACK, LA_STAGE_RABENSEIFNER_AG, LA_STAGE_RABENSEIFNER_RS,
    LA_STAGE_RECURSIVE_DOUBLING, LA_STAGE_RING_AG,
    LA_STAGE_RING_RS, LA_STAGE_S1, LA_STAGE_S2, LA_STAGE_S2_RING_AG, LA_STAGE_S2_RING_RS, LA_STAGE_S2A, LA_STAGE_S2B, LA_STAGE_S3, LA_STEP_COPY,
    LA_STEP_REDUCE, LA_SUM, LIB_PATH, LaError, Schedule, Topology, la_allreduce_emulated, la_allreduce_emulated_out_of_place, la_last_error,
    la_reduce_segments, la_reduce_segments_static, la_schedule_build, la_schedule_fusion_runs, la_schedule_fusion_table, la_schedule_launch_plan, la_schedule_launch_segments, la_schedule_run_step, la_schedule_run_steps, la_status_string, la_topology_create,
    la_tuning_get, la_tuning_set, lib, ptr_array,
)


def torch_dtype_code(t) -> int:
    """la_dtype_t of a torch tensor (int32, float32, bfloat16)."""
    import torch

    table = {torch.int32: LA_I32, torch.float32: LA_F32, torch.bfloat16: LA_BF16, torch.float16: LA_F16,
             torch.float64: LA_F64}
    if t.dtype not in table:
        raise TypeError(f"unsupported tensor dtype {t.dtype}")
    return table[t.dtype]


def allreduce_tensors(sched: Schedule, tensors, stream=None, op=LA_SUM) -> None:
    """In-place emulated all-reduce over P contiguous 1-D device tensors on torch's current (or
    the given) stream.  Marshals pointers only."""
    import torch

    if len(tensors) != sched.num_buffers:
        raise ValueError(f"the schedule works on {sched.num_buffers} buffers, got {len(tensors)}")
    for t in tensors:
        if not (t.is_cuda and t.is_contiguous() and t.numel() == sched.n):
            raise ValueError("every rank buffer must be a contiguous device tensor of n elements")
    s = stream if stream is not None else torch.cuda.current_stream()
    la_allreduce_emulated(sched, [t.data_ptr() for t in tensors], sched.n, torch_dtype_code(tensors[0]),
                          OPS[op] if isinstance(op, str) else op, s.cuda_stream)
