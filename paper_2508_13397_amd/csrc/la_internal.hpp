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

// Launch shape of one step.  In the process-wide setting 0 (unroll, block) and -1 (cache_policy)
// mean "choose per step from its fan-in, fan-out and segment length".
struct Tuning {
    int unroll = 0;       // 16-byte vectors per lane and operand: 1, 2, 4, 8
    int cache_policy = -1; // 0..7, see Policy<> in kernels.hip
    int block = 0;        // lanes per workgroup: 256, 1024
    int merge = 1;        // launch table-adjacent segments that continue each other as one
    bool operator==(const Tuning& o) const
    {
        return unroll == o.unroll && block == o.block && cache_policy == o.cache_policy && merge == o.merge;
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
    // the buffer sets the schedule has been run on lately, most recent first (a few, so that a
    // caller that alternates between buffer sets does not re-upload tables on every call)
    mutable std::vector<la_binding*> bound;
};

namespace la {
la_status_t generate_steps(la_schedule& s);
la_status_t validate_hazards(const la_schedule& s);
void release_binding(la_binding* b);
} // namespace la
