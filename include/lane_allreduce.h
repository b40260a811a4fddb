/*
 * lane_allreduce.h -- C ABI of the emulated lane-aware all-reduce for one MI355X (gfx950).
 *
 * P = nodes * gpus_per_node * procs_per_gpu virtual ranks each own a private buffer of n
 * elements; all P buffers live in the HBM of the one GPU.  A schedule turns a topology into a
 * list of steps; every step is a table of segments, and a segment says "add these k source
 * ranges element by element, in this order, and store the sum to these m destination ranges".
 * Message exchanges of the distributed algorithm become reads of a peer's buffer; all
 * arithmetic runs in HIP kernels, one launch per step (or one per run of consecutive two-operand
 * steps, see la_schedule_fusion_runs).
 *
 * Rank numbering follows l_r = r mod PPG ("Multiple Processes Per GPU" subsection):
 *   r = (node * gpus_per_node + gpu) * procs_per_gpu + proc.
 *
 * Pointer arguments marked [host] are read by the CPU before the call returns (the caller may
 * free them at once); arguments marked [device] are HIP device pointers owned by the caller.
 * The library never frees or reallocates caller memory.  Handles are owned by the library and
 * released by their *_destroy call; destroying NULL is a no-op.
 *
 * Every function returns LA_OK or an error; after an error nothing has been enqueued.
 * la_last_error() gives a thread-local description of the most recent failure.
 */
#ifndef LANE_ALLREDUCE_H
#define LANE_ALLREDUCE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct la_topology la_topology_t; /* opaque, host only */
typedef struct la_schedule la_schedule_t; /* opaque; owns host tables and (once run) device tables */

typedef enum {
    LA_OK = 0,
    LA_ERR_INVALID_ARG = 1,   /* null pointer, dimension <= 0, n == 0, mismatch with the schedule,
                                 misaligned or overlapping buffers */
    LA_ERR_UNSUPPORTED = 2,   /* unknown dtype / algorithm / flag / operation, or a combination that is not built */
    LA_ERR_OUT_OF_MEMORY = 3, /* host or device allocation failed */
    LA_ERR_DEVICE = 4         /* a HIP call failed (no GPU, launch error, ...) */
} la_status_t;

typedef enum {
    LA_ALGO_RING = 0,          /* Algorithm 1, ring_allreduce, over all P ranks */
    LA_ALGO_LANE = 1,          /* Algorithm 2, lane_allreduce: one lane per GPU, owned by the GPU's
                                  leader process (local rank 0) */
    LA_ALGO_LANE_MULTIPROC = 2, /* Algorithm 2 run per process ("Multi-lane Approach"): each lane
                                   is split again into one sub-chunk per process of the GPU */
    /* The small- and medium-size algorithms of the Background section, flat over all P ranks; P
     * must be a power of two (else LA_ERR_UNSUPPORTED).  Not available with
     * LA_SCHED_SHARED_BUFFERS. */
    LA_ALGO_RECURSIVE_DOUBLING = 3, /* log2 P launches; ranks that differ in one bit exchange and
                                       add their whole buffers */
    LA_ALGO_RABENSEIFNER = 4        /* reduce-scatter by recursive halving (log2 P launches, the
                                       data halving each time) + all-gather by recursive doubling */
} la_algo_t;

/* Element types.  The paper reduces 32-bit floats; the others follow the same schedules.  The
 * 16-bit types are widened exactly to fp32, combined in fp32 and rounded to nearest-even once
 * per reduce step. */
typedef enum { LA_I32 = 0, LA_F32 = 1, LA_BF16 = 2, LA_F16 = 3, LA_F64 = 4 } la_dtype_t;
/* Operations.  LA_SUM is MPI_SUM, the one the paper uses.  Floating-point maximum / minimum: a
 * NaN loses against a number, +0 is larger than -0; int32 sum and product wrap. */
typedef enum { LA_SUM = 0, LA_PROD = 1, LA_MAX = 2, LA_MIN = 3 } la_op_t;

/* Flags of la_schedule_build_ex (bit set). */
enum {
    LA_SCHED_DEFAULT = 0u,
    /* All-gather stages as one copy segment per (source, destination) pair, and the inter-node
     * all-reduce as two steps (reduce-scatter of pieces, then all-gather of pieces).  Without
     * it a reduced piece is written to all its destinations by the launch that produces or
     * first reads it (multi-destination store), so it is read from HBM once.  Schedules without
     * an all-gather of that kind (ring, recursive doubling, Rabenseifner) ignore the flag. */
    LA_SCHED_P2P_GATHER = 1u,
    /* Staged exchange: before every reduce step the incoming segments are first copied into a
     * contiguous staging area owned by the library ("the message"), and the reduce reads them
     * from there and stores into the rank buffer.  This is the copy to and from a private
     * device buffer that the GPUDirect runs needed (Results, "GPUDirect RDMA Analysis").
     * Without it the reduce reads the peers' segments in place (fused pack + reduce). */
    LA_SCHED_STAGED = 2u,
    /* Lane schedules only: the inter-node all-reduce of every part is Algorithm 1 run on the lane
     * communicator (the inter-node ring variant that the Results section measures): 2(N-1) steps,
     * each one ring iteration of all lane communicators, instead of the direct N-way exchange.
     * Ignored by the algorithms that have no inter-node stage (ring, recursive doubling,
     * Rabenseifner). */
    LA_SCHED_INNER_RING = 4u,
    /* The shared-buffer model of "Multiple Processes Per GPU": one buffer per GPU (bufs holds
     * nodes * gpus_per_node pointers, index node * gpus_per_node + gpu); the procs_per_gpu
     * processes of a GPU work on it, process q on part q of a balanced split of n.  The result in
     * every buffer is the sum of the nodes * gpus_per_node buffers.
     *   LA_ALGO_RING            the "Standard Approach": one all-reduce per local rank over the
     *                           processes with that local rank (new_comm), all running at once;
     *                           each is Algorithm 1 over nodes * gpus_per_node members.
     *   LA_ALGO_LANE_MULTIPROC  the "Multi-lane Approach": Algorithm 2 per process on its slice
     *                           (S1 fan-in = gpus_per_node).  LA_ALGO_LANE: the same with one
     *                           process per GPU.
     * With LA_SCHED_STAGED every process first copies its slice into a private staging slot, the
     * all-reduce runs on the private copies, and the result is copied back (the copy to and from
     * a buffer allocated by the calling process of the GPUDirect runs).  LA_SCHED_INNER_RING is
     * not available in this model. */
    LA_SCHED_SHARED_BUFFERS = 8u,
    /* Separate send and receive buffers, as Algorithm 1 is printed (buf_send, buf_recv): the
     * schedule is run with la_allreduce_emulated_out_of_place; original inputs are read from the
     * send buffers, which are never written, and every result lands in the receive buffers. */
    LA_SCHED_OUT_OF_PLACE = 16u,
    /* Stand-alone halves of an all-reduce.  Every schedule here is a reduce-scatter followed by
     * an all-gather (MPI_Reduce_scatter ... MPI_Allgatherv of Algorithm 2, the two loops of
     * Algorithm 1, the two phases of Rabenseifner's algorithm).  ONLY_REDUCE_SCATTER keeps the
     * first half: afterwards buffer b holds the complete reduction on the ranges
     * la_schedule_owned_ranges(b) reports, and partial sums elsewhere.  ONLY_ALLGATHER keeps the
     * second half: it expects those ranges to be valid and copies them to every buffer.  Running
     * the two one after the other is the all-reduce, bit for bit.  Lane schedules: the first
     * half is S1 + the inter-node reduce-scatter, the second the inter-node all-gather + S3.
     * Not available for recursive doubling, nor for shared buffers with copy-in / copy-out. */
    LA_SCHED_ONLY_REDUCE_SCATTER = 32u,
    LA_SCHED_ONLY_ALLGATHER = 64u,
    /* Lane schedules: fold both all-gathers of Algorithm 2 (the one inside the lane all-reduce and
     * MPI_Allgatherv on the node group) into the store of the inter-node reduce, which then writes
     * each reduced piece to all N * R rank buffers (k = N, m = N * R; with one node the intra-node
     * reduce does it: k = R, m = R).  Same sums in the same order, so the result is bit-identical
     * to the unfused schedule; the launch that re-reads every owner's part to copy it is gone
     * (N * n elements less to read; the writes are the same).  An emulation-level fusion: between
     * real ranks the two all-gathers use different networks.  Excludes P2P_GATHER, INNER_RING and
     * the halves. */
    LA_SCHED_FUSED_GATHER = 128u,
    /* Lane schedules: the whole of Algorithm 2 as ONE launch.  Piece v of part j is computed as a
     * two-level sum straight from the inputs: for every node, its R rank buffers in ascending
     * node-local index (what MPI_Reduce_scatter on the node group leaves at the owner, rounded to
     * the element type as that result is when it is stored), then the node results in ascending
     * node order (the lane all-reduce); the result is stored to all N * R rank buffers (both
     * all-gathers).  k = m = N * R, la_schedule_step_group() = R.  Bit-identical to the three-stage
     * schedule; every input is read once and every output written once, the lower bound of the
     * definition.  Like LA_SCHED_FUSED_GATHER a fusion of the emulation, not of the algorithm.
     * Combines only with LA_SCHED_SHARED_BUFFERS and LA_SCHED_OUT_OF_PLACE. */
    LA_SCHED_SINGLE_LAUNCH = 256u
};

/* Step kinds and stage labels reported by la_schedule_step_info. */
enum { LA_STEP_REDUCE = 0, LA_STEP_COPY = 1 };
enum {
    LA_STAGE_S1 = 1,       /* intra-node reduce-scatter (MPI_Reduce_scatter of Algorithm 2) */
    LA_STAGE_S2A = 2,      /* inter-node reduce-scatter of the N pieces of each part */
    LA_STAGE_S2B = 3,      /* inter-node all-gather of the pieces */
    LA_STAGE_S3 = 4,       /* intra-node all-gather (MPI_Allgatherv of Algorithm 2) */
    LA_STAGE_S2 = 5,       /* S2A and S2B in one launch (multi-destination store) */
    LA_STAGE_S2_RING_RS = 6, /* LA_SCHED_INNER_RING: one reduce iteration of the inter-node rings */
    LA_STAGE_S2_RING_AG = 7, /* LA_SCHED_INNER_RING: one gather iteration of the inter-node rings */
    LA_STAGE_S2_S3 = 8,    /* LA_SCHED_FUSED_GATHER: inter-node reduce storing to every rank */
    LA_STAGE_S1_S3 = 9,    /* LA_SCHED_FUSED_GATHER on one node: intra-node reduce storing to every rank */
    LA_STAGE_RING_RS = 10, /* one iteration of the first loop of Algorithm 1 */
    LA_STAGE_RING_AG = 11, /* one iteration of the second loop of Algorithm 1 */
    LA_STAGE_RECURSIVE_DOUBLING = 12, /* one round of recursive doubling */
    LA_STAGE_RABENSEIFNER_RS = 13,    /* one halving round of Rabenseifner's reduce-scatter */
    LA_STAGE_RABENSEIFNER_AG = 14,    /* one doubling round of Rabenseifner's all-gather */
    LA_STAGE_S1_S2_S3 = 15, /* LA_SCHED_SINGLE_LAUNCH: Algorithm 2 as one two-level reduce */
    LA_STAGE_PACK = 20,    /* staged exchange: copy of incoming segments into the staging area */
    LA_STAGE_COPY_INPUT = 21 /* out-of-place: ranges that no step reduces, copied from send to receive */
};

/* ---- topology ------------------------------------------------------------------------- */

/* All three counts must be >= 1 and their product must fit in 2^20. */
la_status_t la_topology_create(int nodes, int gpus_per_node, int procs_per_gpu, la_topology_t** out);
la_status_t la_topology_destroy(la_topology_t* topo);
int la_topology_num_ranks(const la_topology_t* topo); /* P, or -1 for NULL */

/* ---- schedules ------------------------------------------------------------------------ */

/*
 * Build the per-step segment tables of an all-reduce over n elements per rank (host work only;
 * device tables are created by the first run).  n need not be divisible: every split is
 * balanced (part i of m gets floor(len/m) elements, plus one if i < len mod m); parts of length
 * zero produce no segment.
 *
 *   ring            Algorithm 1: P chunks; P-1 reduce steps (rank r adds the chunk it receives
 *                   from r-1 to its own copy) and P-1 copy steps.
 *   lane, lane_multiproc
 *                   Algorithm 2: S1 reduce-scatter inside each node (fan-in = ranks per node),
 *                   S2 all-reduce of each part across the nodes (fan-in = nodes), S3 all-gather
 *                   inside each node.  Operands are added in ascending communicator rank.
 *
 * Every schedule is checked at build time: no step reads a range that another segment of the
 * same step writes.
 */
la_status_t la_schedule_build(const la_topology_t* topo, la_algo_t algo, size_t n, la_dtype_t dtype,
                              la_schedule_t** out);
la_status_t la_schedule_build_ex(const la_topology_t* topo, la_algo_t algo, size_t n, la_dtype_t dtype,
                                 unsigned flags, la_schedule_t** out);
la_status_t la_schedule_destroy(la_schedule_t* sched);

int la_schedule_num_steps(const la_schedule_t* sched);       /* -1 for NULL */
int la_schedule_num_buffers(const la_schedule_t* sched);     /* entries of bufs: P, or nodes * gpus_per_node
                                                                with LA_SCHED_SHARED_BUFFERS; -1 for NULL */
size_t la_schedule_staging_elems(const la_schedule_t* sched); /* elements of library-owned staging */
/* The element ranges that buffer `buffer` holds fully reduced after the reduce-scatter half (and
 * must provide to the all-gather half).  Writes up to `capacity` (offset, length) pairs [host]
 * and returns how many there are (one per rank; one per process with shared buffers; none for a
 * rank that owns nothing, such as a non-leader in LA_ALGO_LANE); -1 for bad arguments. */
int la_schedule_owned_ranges(const la_schedule_t* sched, int buffer, int capacity, uint64_t* offsets, uint64_t* lengths);

/* Shape of one step.  Any out pointer may be NULL.  bytes_* are the algorithmic bytes of the
 * step: sum over segments of len * fan_in (resp. fan_out) * element size. */
la_status_t la_schedule_step_info(const la_schedule_t* sched, int step, int* kind, int* stage,
                                  size_t* num_segments, size_t* seg_len_max, int* fan_in, int* fan_out,
                                  size_t* bytes_read, size_t* bytes_written);

/* Sources per first-level sum of a step: the fan-in for an ordinary step; for the two-level step
 * of LA_SCHED_SINGLE_LAUNCH the sources are added in runs of this many, each run rounded to the
 * element type, and the run results are then added in order.  -1 for bad arguments. */
int la_schedule_step_group(const la_schedule_t* sched, int step);

/* Copy out the table of one step [host arrays sized from la_schedule_step_info]:
 * seg_len[S]; src_buf/src_off[S*fan_in]; dst_buf/dst_off[S*fan_out].  A buffer index below
 * la_schedule_num_buffers() is a caller buffer (the receive buffer in an out-of-place schedule);
 * that number itself is the staging area; that number + 1 + b is send buffer b of an
 * out-of-place schedule.  Offsets are in elements. */
la_status_t la_schedule_step_table(const la_schedule_t* sched, int step, uint64_t* seg_len, int32_t* src_buf,
                                   uint64_t* src_off, int32_t* dst_buf, uint64_t* dst_off);

/* ---- execution ------------------------------------------------------------------------ */

/*
 * In-place all-reduce: on return of the enqueued work every bufs[r] holds the element-wise SUM
 * of the P input buffers (the MPI_Allreduce(..., MPI_SUM, ...) of the "Standard Approach"
 * listing, with send and receive buffer the same).
 *   bufs        [host] array of la_schedule_num_buffers() [device] pointers (P unless the schedule
 *               was built with LA_SCHED_SHARED_BUFFERS), each to n elements of dtype, aligned to
 *               the element size, pairwise disjoint.  128-bit accesses are used when all
 *               buffers share the same address modulo 16 bytes; otherwise a slower
 *               element-wise path runs.
 *   n, dtype    must equal the values the schedule was built with.
 *   hip_stream  a hipStream_t (NULL = the default stream).  The call enqueues one kernel per
 *               step and returns without synchronising.
 * A schedule remembers the last 8 buffer sets it was run with (1 if it owns a staging area) and
 * keeps their resolved tables on the device; a call with a set it does not remember uploads
 * tables with a synchronous copy, after waiting for the work of the set it forgets in exchange.
 * Runs of steps with at most two sources and destinations per segment (the ring forms) go out as
 * one launch each (see la_schedule_fusion_runs); a schedule of 16 or more launches without such a
 * run is recorded once per buffer set into a HIP graph of kernel nodes and replayed.  A call with
 * a remembered set allocates nothing and enqueues kernel launches only (no copy, memset, event or
 * synchronisation), so it may be recorded into a caller's own graph, provided the library does
 * not replay a graph of its own for the schedule ("graph" knob 0, or fewer than 16 launches).
 * Calls on one schedule are serialised by the library; different schedules can be used from
 * different host threads at the same time.
 * int32 wraps; fp32 adds are IEEE, in the fixed operand order of the tables; bf16 operands are
 * widened to fp32, summed in fp32 and rounded to nearest-even once per reduce step.
 */
la_status_t la_allreduce_emulated(const la_schedule_t* sched, void* const* bufs, size_t n, la_dtype_t dtype,
                                  la_op_t op, void* hip_stream);

/* The same all-reduce with separate buffers: sendbufs[b] is read only, recvbufs[b] receives the
 * result; all 2 * la_schedule_num_buffers() buffers must be pairwise disjoint.  The schedule must
 * have been built with LA_SCHED_OUT_OF_PLACE (and la_allreduce_emulated refuses such a schedule). */
la_status_t la_allreduce_emulated_out_of_place(const la_schedule_t* sched, const void* const* sendbufs,
                                               void* const* recvbufs, size_t n, la_dtype_t dtype, la_op_t op,
                                               void* hip_stream);

/* Enqueue a single step of the schedule (same conventions, LA_SUM): for per-step timing and for
 * tests that look at intermediate states. */
la_status_t la_schedule_run_step(const la_schedule_t* sched, int step, void* const* bufs, void* hip_stream);
/* Enqueue steps [first_step, first_step + num_steps) with the given operation, launched as
 * la_allreduce_emulated launches them (a run of steps that lies inside the range goes out as one
 * fused launch if the "fuse" knob selects it).  Not for out-of-place schedules. */
la_status_t la_schedule_run_steps(const la_schedule_t* sched, int first_step, int num_steps, void* const* bufs,
                                  la_op_t op, void* hip_stream);

/* Host only, for tests and for reading the launch heuristics: how one step would be launched for
 * buffers at the given addresses.  The addresses are never dereferenced and no device call is
 * made.  sendbufs is NULL unless the schedule is out-of-place; staging is the address to assume
 * for the library-owned staging area of a LA_SCHED_STAGED schedule (ignored otherwise).  Honours
 * the la_tuning_set knobs like a real launch. */
typedef struct la_launch_plan {
    int block;                  /* lanes per workgroup */
    int unroll;                 /* 16-byte vectors per lane and operand: a tile is block * unroll vectors */
    int cache_policy;           /* 0..7, see la_tuning_set */
    int tiling;                 /* 0: full tiles from the segment's start; 1: a short first tile, the others
                                   start where destination 0's address is a multiple of the tile size;
                                   2: as few tiles as 0, all of one size */
    uint32_t tiles_per_segment; /* workgroups per segment (those beyond a short segment's end exit at once) */
    uint32_t edge_workgroups;   /* workgroups for the elements outside the segments' whole 16-byte vectors */
    uint64_t workgroups;        /* edge_workgroups + segments * tiles_per_segment */
} la_launch_plan_t;
la_status_t la_schedule_launch_plan(const la_schedule_t* sched, int step, const void* const* bufs,
                                    const void* const* sendbufs, const void* staging, la_launch_plan_t* out);

/*
 * Column analysis of a schedule (host only).  Algorithms 1 and 2 exchange chunks that sit at the same
 * element offset in every rank's buffer, so element i of a buffer only ever meets element i of other
 * buffers.  Cutting the element axis wherever a segment of a step starts or ends gives column ranges
 * ("chains") that never exchange data; a chain's operations are the (step, segment) pairs that cover
 * it, in step order (Algorithm 1 over P ranks: P chains, one per chunk, of 2(P - 1) operations).  A
 * "run" is a maximal sequence of two or more consecutive steps whose segments have at most two
 * sources and two destinations each (the two loops of Algorithm 1, the ring form of the inter-node
 * stage, recursive halving and doubling, point-to-point copies).  la_allreduce_emulated executes a
 * run as ONE launch in which a wave takes its piece of a chain through all the run's steps (same
 * sums in the same order, every store of every step made, no synchronisation between workgroups),
 * instead of one launch per step; which runs, see the "fuse" knob of la_tuning_set.  Steps outside
 * runs (the fan-in and fan-out steps of Algorithm 2) keep their own launches.
 *   la_schedule_fusion_runs   number of runs (0: none; -1: NULL schedule or out of memory)
 *   la_schedule_fusion_info   first step and number of steps of a run, its chains and operations, and
 *                             whether it is fused without being asked (four steps or more, and the
 *                             longest chain has fewer than 8 operations per step); bytes_read and
 *                             bytes_written are what the fused launch moves with the current "forward"
 *                             setting: every destination is stored, a source is loaded unless it is
 *                             taken from registers (the steps' own figures, la_schedule_step_info,
 *                             count every source); any out pointer may be NULL
 *   la_schedule_fusion_table  [host arrays sized from la_schedule_fusion_info; any may be NULL]
 *     chain_lo[C], chain_len[C]    the chain's elements; chain_first_op[C + 1] prefix sums into the ops
 *     op_step[ops], op_segment[ops]   the operation: that segment of that step, restricted to the chain
 *     op_prefetch_source[ops]      a source no earlier operation of the chain has written (it may be
 *                                  loaded ahead of time), or -1
 *     op_forward_source[ops]       a source that is exactly what the previous operation of the chain
 *                                  stored (taken from registers, see the "forward" knob), or -1
 */
int la_schedule_fusion_runs(const la_schedule_t* sched);
la_status_t la_schedule_fusion_info(const la_schedule_t* sched, int run, int* first_step, int* num_steps,
                                    uint64_t* num_chains, uint64_t* num_ops, int* automatic, size_t* bytes_read,
                                    size_t* bytes_written);
la_status_t la_schedule_fusion_table(const la_schedule_t* sched, int run, uint64_t* chain_lo, uint64_t* chain_len,
                                     uint64_t* chain_first_op, uint32_t* op_step, uint32_t* op_segment,
                                     int32_t* op_prefetch_source, int32_t* op_forward_source);

/* Host only, like la_schedule_launch_plan: the segments of one step as they are launched.  A table
 * segment whose source ranges start where those of the segment before it end, and whose destination
 * ranges do too (as a set: the order of a destination list does not matter, every destination
 * receives the same value), is launched as part of that segment: the N pieces of a part in the
 * inter-node step, every segment of the one-launch form.  The sums and their order are unchanged,
 * and la_schedule_step_info / la_schedule_step_table keep reporting the segments as generated.
 * Writes the number of launch segments to *count and, for the first min(capacity, *count) of them,
 * seg_len[g] (elements), src_addr[g * fan_in + t] and dst_addr[g * fan_out + d] (byte addresses;
 * any of the three arrays may be NULL) [host]. */
la_status_t la_schedule_launch_segments(const la_schedule_t* sched, int step, const void* const* bufs,
                                        const void* const* sendbufs, const void* staging, size_t capacity,
                                        size_t* count, uint64_t* seg_len, uint64_t* src_addr, uint64_t* dst_addr);

/*
 * k incoming segments summed into the owned segment (the local reduction that follows each
 * received message, "GPU-Aware All-Reduce Operations" subsection), for num_segments segments
 * in one launch.  For every segment s and i < seg_len, with o = seg_offsets[s] + i:
 *     dst[o] = ((dst[o] + srcs[0][o]) + srcs[1][o]) + ... + srcs[k-1][o]
 *   dst          [device] owned buffer
 *   srcs         [host] array of k [device] pointers (k >= 0; k == 0 leaves dst unchanged)
 *   seg_offsets  [host] array of num_segments element offsets, applied to dst and every src;
 *                segments must not overlap each other
 * dst and srcs must be aligned to the element size and srcs must not overlap the written
 * ranges of dst.  Enqueues on hip_stream, no synchronisation.
 */
la_status_t la_reduce_segments(void* dst, const void* const* srcs, int k, const size_t* seg_offsets,
                               size_t num_segments, size_t seg_len, la_dtype_t dtype, la_op_t op,
                               void* hip_stream);

/*
 * la_reduce_segments for callers that cannot allocate: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, same result, bit for bit; the
 * call makes no allocation of any kind on the device or in pinned host memory and no copy: the
 * per-call tables that la_reduce_segments keeps in a stream-ordered allocation live in a static
 * device array of 1 MiB (held by every GPU the library runs on until the process ends) and are
 * written there by a small kernel launched on hip_stream ahead of the reduce kernel.
 * Limits: k <= 64, num_segments <= 8192, and num_segments * (32 + 8 * (k + 1)) bytes (each of the
 * three tables rounded up to 256) <= 1 MiB; beyond them LA_ERR_INVALID_ARG, nothing enqueued.
 * All calls on one GPU share the one array: calls on the same stream are ordered and safe, calls
 * that may overlap on the GPU (different streams, or host threads on different streams) race and
 * must be ordered by the caller.  The array's device address is looked up on the first call on a
 * device; make that call outside a graph capture.
 */
la_status_t la_reduce_segments_static(void* dst, const void* const* srcs, int k, const size_t* seg_offsets,
                                      size_t num_segments, size_t seg_len, la_dtype_t dtype, la_op_t op,
                                      void* hip_stream);

/* ---- diagnostics and tuning ----------------------------------------------------------- */

const char* la_status_string(la_status_t status);
const char* la_last_error(void);

/* Launch-shape knobs for measurements (process-wide, read when a schedule is bound or a
 * la_reduce_segments call is made).  By default every step picks its own shape from its fan-in,
 * fan-out and segment length (schedules whose buffers together are at most 96 MiB keep one workgroup
 * size for all steps); a knob set to a fixed value overrides that choice for all steps.
 *   "unroll"      16-byte vectors per lane and operand: 1, 2, 4, 8 (8: only with workgroups of
 *                 1024 lanes, else 4 is used); 0 = automatic
 *   "cache_policy" 0..7: which of {loads of pure sources, loads of sources the segment also
 *                 overwrites, stores} are plain (P), non-temporal (N) or scope-1 (S):
 *                 0 PPP, 1 NPP, 2 NPS, 3 NNN, 4 PPN, 5 NNP, 6 NNS, 7 PPS; -1 = automatic.
 *                 A three-digit value abc sets policy a for pure reduce steps, b for reduce
 *                 steps with several destinations and c for copy / broadcast steps.
 *   "block"       lanes per workgroup: 256, 1024; 0 = automatic
 *   "merge"       1 (default): table-adjacent segments that continue each other are launched as one
 *                 (see la_schedule_launch_segments); 0: every table segment is a launch segment
 *   "fuse"        which runs of steps (see la_schedule_fusion_runs) la_allreduce_emulated executes as
 *                 one launch each: -1 (default): those of four steps or more whose longest chain has
 *                 fewer than 8 operations per step (the ring forms; recursive halving on up to 32
 *                 ranks); 1: every run; 0: none.
 *                 A run is fused only if all buffers share their address modulo 16 bytes.
 *   "forward"     fused launches only.  1 (default): a source that is exactly what the previous
 *                 operation of its chain stored (the chunk a rank has just received from its
 *                 predecessor) is taken from the registers of the lane that stored it; the store to the
 *                 rank buffer is made all the same.  0: every source is loaded from memory
 *                 (la_tuning_get("fused_launches") counts the fused launches made so far; read-only)
 *   "graph"       1: la_allreduce_emulated replays the schedule as one HIP graph of kernel nodes,
 *                 0: it launches step by step, -1 (default): graph for schedules of 16+ launches
 * la_tuning_set returns LA_ERR_INVALID_ARG for an unknown key or value; la_tuning_get returns
 * the current setting, or -2 for an unknown key. */
la_status_t la_tuning_set(const char* key, int value);
int la_tuning_get(const char* key);

#ifdef __cplusplus
}
#endif
#endif /* LANE_ALLREDUCE_H */
