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
    bool operator==(const Tuning& o) const
    {
        return unroll == o.unroll && block == o.block && cache_policy == o.cache_policy;
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

// kernels.hip
la_status_t launch_step(const StepTable& t, la_dtype_t dtype, const Tuning& tune, void* hip_stream);
uint32_t tiles_for(uint64_t max_units, const Tuning& tune); // units = 16-byte vectors per operand

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
