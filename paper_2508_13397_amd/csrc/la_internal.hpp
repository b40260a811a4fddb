// Internal declarations shared by the host-side sources of liblaneallreduce.
#pragma once

#include <cstdarg>
#include <cstdint>
#include <mutex>
#include <vector>

#include "lane_allreduce.h"

namespace la {

// Balanced split of `len` into `m` parts: part i has floor(len/m) elements plus one if
// i < len mod m; offsets are the exclusive prefix sums of the counts (the counts and
// displacement arrays c_on_chunk / D of Algorithms 1 and 2, without dropping a remainder).
struct Part {
    uint64_t off, cnt;
};
inline Part split_part(uint64_t len, uint64_t m, uint64_t i)
{
    const uint64_t q = len / m, rem = len % m;
    return Part{i * q + (i < rem ? i : rem), q + (i < rem ? 1u : 0u)};
}

inline size_t dtype_size(la_dtype_t d)
{
    if (d == LA_BF16 || d == LA_F16) return 2;
    return d == LA_F64 ? 8 : 4;
}
inline bool known_dtype(int d)
{
    return d == LA_I32 || d == LA_F32 || d == LA_BF16 || d == LA_F16 || d == LA_F64;
}
inline bool known_op(int op)
{
    return op == LA_SUM || op == LA_PROD || op == LA_MAX || op == LA_MIN;
}

struct Operand {
    int32_t buf;  // rank index, or P for the staging area
    uint64_t off; // elements
};

// One launch: S segments, each with k sources and m destinations.
struct Step {
    int kind = LA_STEP_REDUCE;
    int stage = 0;
    int k = 0, m = 0;
    int group = 0;             // > 0: the k sources are added in runs of `group`, each run rounded to
                               // the element type, then the run results in order (two-level sum)
    std::vector<uint64_t> len; // [S]
    std::vector<Operand> src;  // [S*k]
    std::vector<Operand> dst;  // [S*m]
    size_t num_segments() const { return len.size(); }
};

// Per-segment record the kernels read.
struct SegInfo {
    uint64_t len;        // elements
    uint32_t head;       // elements before the vector body: up to the first 16-byte, or if all operands
                         // agree modulo 128 bytes the first 128-byte boundary (vector path only)
    uint32_t vec_ok;     // 1: all operands of the segment share the address modulo 16
    uint64_t alias_mask; // bit t: source t (t < 64) is also a destination of the segment
};

// Host and device code share the arithmetic that describes a segment.
#if defined(__HIPCC__) || defined(__HIP__)
#define LA_HOST_DEVICE __host__ __device__
#else
#define LA_HOST_DEVICE
#endif

inline LA_HOST_DEVICE uint64_t align_up(uint64_t x, uint64_t a)
{
    return (x + a - 1) / a * a;
}

// Complete the record of a segment of `len` elements whose first operand starts at byte address
// `first`, given whether all its operands agree modulo 16 bytes (`congruent`) and the largest of
// 16 and 128 bytes modulo which they all agree (`align`); returns the segment's length in 16-byte
// units as the launch sees it.  The vector body starts at the first 16-byte boundary -- or, when
// all operands also agree modulo a cache line (the usual case: an odd element offset into
// 256-byte aligned buffers), at the first 128-byte boundary, so that every wave's 1 KiB access
// covers whole lines (otherwise each touches nine lines instead of eight and stores partial
// lines: an odd n cost 14 to 26 % of the whole all-reduce).  The elements before it are done one
// per lane.
inline LA_HOST_DEVICE uint64_t finish_segment(SegInfo& si, uint64_t len, uint64_t first, uint32_t esize, bool congruent,
                                              uint32_t align)
{
    const uint64_t vec = 16 / esize;
    si.len = len;
    if (!congruent) {
        si.head = 0;
        si.vec_ok = 0;
        return (len + vec - 1) / vec;
    }
    uint64_t head = ((align - (first & (align - 1))) & (align - 1)) / esize;
    if (head > len) head = len;
    si.head = (uint32_t)head;
    si.vec_ok = 1;
    return (len - head) / vec;
}

// How the kernel cuts the 16-byte vectors of a segment into tiles of at most block * unroll.
enum : uint32_t {
    TILING_PLAIN = 0,   // full tiles from the segment's start, the last one ragged
    TILING_ALIGNED = 1, // a short first tile, so that the others start where destination 0's address is a
                        // multiple of the tile size
    TILING_EQUAL = 2,   // as few tiles as TILING_PLAIN, all of one size (a multiple of 128 bytes)
};

// The elements of a segment before its first and after its last whole 16-byte vector are done one
// per lane by separate "edge" workgroups at the front of the grid, EDGE_LANES lanes per segment
// (enough for the longest head plus tail: 63 + 7 two-byte elements).
constexpr uint32_t EDGE_LANES = 128;

// Device view of one step, passed to the kernels by value.
struct StepTable {
    const SegInfo* seg;      // [S]
    const uint64_t* src_ptr; // [S*k] byte addresses
    const uint64_t* dst_ptr; // [S*m]
    uint32_t k, m;
    uint32_t tiles_per_seg;  // grid = S * tiles_per_seg blocks
    uint32_t num_segments;
    uint32_t op = 0;         // la_op_t of the launch
    uint32_t group = 0;      // 0 or k: one level; else sources per first-level run
    uint32_t tiling = 0;     // TILING_*: how a segment's vectors are cut into workgroup tiles
    uint32_t edge_blocks = 0; // leading workgroups that do the elements outside the whole vectors (0: there are none)
};

// ---- column-fused execution of runs of steps in one launch ---------------------------------------
// Every step of the schedules here is element-wise at one element offset: all operands of a
// segment start at the same offset of their buffers.  Element i of any buffer therefore only ever
// meets element i of other buffers, and the element axis can be cut, at every offset where some
// segment of some step starts or ends, into column ranges that never exchange data.  A "chain" is
// one column range with the ordered list of (step, segment) pairs that cover it; chains are
// independent of each other, so one wave can run all steps of its piece of a chain, in step order,
// without waiting for any other wave: the launches of a run of steps (2(P - 1) for Algorithm 1)
// collapse into one, and every store of every step is still performed.  A run is a maximal sequence
// of consecutive steps whose segments have at most two sources and two destinations (the ring forms,
// recursive halving and doubling, point-to-point copies); the fan-in and fan-out steps of Algorithm 2
// keep their own launches, whose large tiles suit them better.
struct FusionRun {
    int first_step = 0, num_steps = 0;
    uint64_t max_chain_ops = 0;                // operations of the longest chain
    // Fused without being asked?  A wave executes its chain's operations one after the other, about
    // half a microsecond each when an operand has to come back from the L2, while a launch costs
    // about 4 us whatever it carries: worth it when the longest chain has fewer than 8 operations per
    // step saved (Algorithm 1: one per step; recursive halving over 16 ranks: 30 in 8 steps; recursive
    // doubling over 16 ranks, 32 in 4 steps, measured 17 % slower fused at small sizes).
    bool automatic() const { return num_steps >= 4 && max_chain_ops < 8 * (uint64_t)num_steps; }
    std::vector<uint64_t> chain_lo, chain_len; // [C] column range in elements
    std::vector<uint64_t> chain_first;         // [C + 1] first op of each chain (prefix sums)
    std::vector<uint32_t> op_step, op_seg;     // [ops] chain-major, in step order (absolute step index)
    // a source of the op that no earlier op of the chain has written (an original input of the run),
    // which the kernel may load ahead of time; -1: none
    std::vector<int32_t> op_prefetch;
    // a source that is exactly what the previous op of the chain stored (the message a rank has just
    // received and now passes on, or adds to): the lane that stored it still holds it; -1: none
    std::vector<int32_t> op_forward;
};
struct FusionPlan {
    bool analysed = false;
    std::vector<FusionRun> runs;
};
constexpr int FUSED_MAX_FAN = 2;      // sources, and destinations, of a segment that can run fused

struct ChainInfo { // device record of one chain
    uint64_t first_op;
    uint64_t nvec;     // whole 16-byte vectors of the column range
    uint32_t num_ops;
    uint32_t head;     // elements before the first whole vector
    uint32_t tail;     // elements after the last one
    uint32_t pad;
};

// Device record of one operation of a chain: one 64-byte line that holds everything the operation
// needs, so that a wave fetches it with one load.
struct FusedOp {
    uint32_t reserved;  // zero
    uint32_t live;      // bit 0: 1 = an operation, 0 = padding behind a chain's last operation (chains are
                        // padded to a multiple of eight records, so that the kernel's loop needs no test
                        // per operation); bits 8 and up, in the first record of every eight: FUSED_BLOCK_*
    uint16_t k, m;
    int16_t prefetch;   // a source that is an original input of the run (loadable ahead), or -1
    int16_t forward;    // a source that is what the previous op of the chain stored (still in registers), or -1
    // byte address of the chain's first element in each operand: k sources, then m destinations
    uint64_t addr[2 * FUSED_MAX_FAN];
    uint64_t pad1[2];
};
static_assert(sizeof(FusedOp) == 64, "one cache line per operation");

constexpr uint32_t FUSED_LANES = 64; // one wave per workgroup: no barrier anywhere in the kernel
constexpr uint32_t FUSED_CHAIN_PAD = 8;            // records per chain: a multiple of this
// Shape of eight consecutive operations (the records [8b, 8b + 8) of a chain), see ring_block in fused.hip
enum : uint32_t { FUSED_BLOCK_GENERAL = 0, FUSED_BLOCK_ADD = 1, FUSED_BLOCK_COPY = 2 };
constexpr uint32_t FUSED_EDGE_TILE = 0xffffffffu;  // wg_tile of the workgroup that does a chain's elements
                                                   // outside its whole 16-byte vectors

struct FusedTable { // passed to the kernel by value
    const ChainInfo* chain;
    const FusedOp* op;
    const uint32_t* wg_chain; // [workgroups] chain of each workgroup
    const uint32_t* wg_tile;  // [workgroups] which tile of FUSED_LANES * unroll vectors of the chain
    uint32_t workgroups;
    uint32_t op_code = 0;     // la_op_t
};

// Launch shape of one step.  In the process-wide setting 0 (unroll, block) and -1 (cache_policy)
// mean "choose per step from its fan-in, fan-out and segment length".
struct Tuning {
    int unroll = 0;       // 16-byte vectors per lane and operand: 1, 2, 4, 8
    int cache_policy = -1; // 0..7, see Policy<> in kernels.hip
    int block = 0;        // lanes per workgroup: 256, 1024
    int merge = 1;        // launch table-adjacent segments that continue each other as one
    int forward = 1;      // fused launch: take what the previous op of a chain stored from registers
    bool operator==(const Tuning& o) const
    {
        return unroll == o.unroll && block == o.block && cache_policy == o.cache_policy && merge == o.merge &&
               forward == o.forward;
    }
};
Tuning current_tuning();
// Fill the automatic fields of `requested` for a step with k sources, m destinations, a longest
// segment of `longest_units` 16-byte vectors and `bytes_per_operand` bytes summed over its
// segments (the size of the step's result, and of its source when k == 1).  all_inputs: the step
// is the whole all-reduce (every source an original input, every rank a destination).
// working_set: bytes of all buffers the schedule works on (what a loop of all-reduces keeps touching).
Tuning resolve_tuning(const Tuning& requested, uint32_t k, uint32_t m, uint64_t longest_units,
                      uint64_t bytes_per_operand, bool all_inputs, size_t esize, uint64_t working_set);

// runtime.cpp: a segment's record from its resolved operand addresses (ptrs = k sources followed by
// the destinations; returns its length in 16-byte units), and the grid of a launch: edge
// workgroups, workgroups per segment, tiling.  dp = destination addresses, m per segment.
uint64_t describe_segment(SegInfo& si, uint64_t len, const uint64_t* ptrs, size_t count, size_t esize, size_t k);
uint32_t plan_edges(const SegInfo* seg, size_t S, size_t esize, const Tuning& shape);
uint32_t plan_tiles(const SegInfo* seg, const uint64_t* dp, size_t S, size_t m, size_t esize, const Tuning& shape,
                    uint64_t longest, uint32_t* tiling);

// kernels.hip
la_status_t launch_step(const StepTable& t, la_dtype_t dtype, const Tuning& tune, void* hip_stream);
la_status_t check_launch(const StepTable& t, la_dtype_t dtype, const Tuning& tune); // what launch_step would refuse
uint32_t tiles_for(uint64_t max_units, const Tuning& tune); // units = 16-byte vectors per operand

// runtime.cpp: the argument checks common to la_reduce_segments and its allocation-free variant
// (everything but the overlap of segments); *nothing is set when the call has no work to do.
la_status_t check_reduce_segments_args(const char* who, const void* dst, const void* const* srcs, int k,
                                       const size_t* seg_offsets, size_t num_segments, size_t seg_len, la_dtype_t dtype,
                                       la_op_t op, bool* nothing);

// error reporting
la_status_t fail(la_status_t st, const char* fmt, ...);

} // namespace la

struct la_topology {
    int nodes, gpus, procs;
    int ranks() const { return nodes * gpus * procs; }
    int per_node() const { return gpus * procs; }
    int rank_of(int node, int local) const { return node * gpus * procs + local; }
};

struct la_binding; // runtime.cpp

struct la_schedule {
    la_topology topo;
    la_algo_t algo;
    la_dtype_t dtype;
    uint64_t n;
    unsigned flags;
    int nbuf = 0; // caller buffers: one per rank, or one per GPU with LA_SCHED_SHARED_BUFFERS;
                  // buffer index nbuf in the tables is the staging area
    uint64_t staging_elems = 0;
    std::vector<la::Step> steps;
    std::vector<std::vector<la::Part>> owned; // per buffer: ranges it holds fully reduced between the halves
    // device-side state, created by the first run
    mutable std::mutex mu;
    mutable la::FusionPlan fusion; // built on first use (under mu)
    // the buffer sets the schedule has been run on lately, most recent first (a few, so that a
    // caller that alternates between buffer sets does not re-upload tables on every call)
    mutable std::vector<la_binding*> bound;
};

namespace la {
// fusion.cpp: fills s.fusion (once) with the runs of steps that can execute column-fused
void analyse_fusion(const la_schedule& s);
// fused.hip
la_status_t launch_fused(const FusedTable& t, la_dtype_t dtype, int unroll, void* hip_stream);
la_status_t generate_steps(la_schedule& s);
la_status_t validate_hazards(const la_schedule& s);
void release_binding(la_binding* b);
} // namespace la
