// Execution side of the C ABI: binds a schedule to device addresses, uploads the per-step
// tables, and enqueues one kernel per step.
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <atomic>
#include <cstring>
#include <new>
#include <string>

#include "la_internal.hpp"

using namespace la;

#define LA_HIP(call)                                                                                  \
    do {                                                                                              \
        hipError_t e_ = (call);                                                                       \
        if (e_ != hipSuccess) return fail(LA_ERR_DEVICE, "%s failed: %s", #call, hipGetErrorString(e_)); \
    } while (0)

// ---- tuning ---------------------------------------------------------------------------------

namespace la {
static std::atomic<int> g_unroll{0};
static std::atomic<int> g_cache_policy{-1};
static std::atomic<int> g_block{0};
static std::atomic<int> g_merge{1};
static std::atomic<int> g_forward{1};
static std::atomic<int> g_graph{-1};
static std::atomic<int> g_fused_launches{0}; // column-fused launches made so far (read-only knob, for tests)
// -1: fuse the runs that FusionRun::automatic() selects (the ring forms, recursive halving on few ranks);
// 1: every run of two steps or more; 0: never
static std::atomic<int> g_fuse{-1}; // -1: graphs for schedules of GRAPH_MIN_STEPS launches or more
// Measured: a graph launch costs the host about 15 us whatever it holds, a stream launch 2.5 to 3 us;
// on the GPU a kernel node and a stream launch take the same time.  Below 16 launches the stream wins.
constexpr int GRAPH_MIN_STEPS = 16;

Tuning current_tuning()
{
    Tuning t;
    t.unroll = g_unroll.load();
    t.cache_policy = g_cache_policy.load();
    t.block = g_block.load();
    t.merge = g_merge.load();
    t.forward = g_forward.load();
    return t;
}

// Launch shapes and cache policies measured on MI355X (every step is HBM-bound):
//  - pure reduce (k >= 2, one destination): every pure source is read once, so its loads are
//    non-temporal; large tiles keep each workgroup on long contiguous runs of every operand,
//    which matters more as k grows.  The result is what the next launch reads: if it fits the
//    last-level cache it is stored with scope-1 stores (it stays resident), else streamed out;
//  - copy / broadcast (k == 1): the source was produced by the previous launch.  If it fits the
//    last-level cache it is read with ordinary loads and the destinations are written with
//    non-temporal stores, so that the written stream does not evict it;
//  - tiles: an operand stream that exceeds the last-level cache comes from DRAM and wants long
//    contiguous runs per workgroup (64..128 KiB); one that the previous launch left in the cache
//    is served faster in small tiles (16 KiB) by many workgroups;
//  - reduce with multi-destination store: every source is overwritten in place; ordinary loads,
//    scope-1 stores.  With many more destinations than sources (LA_SCHED_FUSED_GATHER) the step
//    behaves like a broadcast and takes its shape: 128 KiB tiles, streaming stores.
constexpr uint64_t LAST_LEVEL_CACHE_BYTES = 256ull << 20;
constexpr uint64_t L2_TOTAL_BYTES = 32ull << 20; // 8 XCDs x 4 MiB
constexpr uint64_t SMALL_SCHEDULE_BYTES = 96ull << 20; // all buffers of a schedule together

Tuning resolve_tuning(const Tuning& req, uint32_t k, uint32_t m, uint64_t longest_units, uint64_t bytes_per_operand,
                      bool all_inputs, size_t esize, uint64_t working_set)
{
    Tuning t;
    bool store_bound = false; // many more stores than loads per workgroup: the workgroup count matters little
    int cls; // step class: 0 pure reduce, 1 reduce + multi-destination store, 2 copy / broadcast
    // measured on 16 ranks: the cache-resident shapes win up to about 1.25 times the cache (a result of
    // 320 MiB: 0.575 against 0.590 ms), and lose from 1.5 times on (0.738 against 0.709 ms)
    const bool fits = bytes_per_operand <= LAST_LEVEL_CACHE_BYTES + LAST_LEVEL_CACHE_BYTES / 4;
    // Everything the schedule touches is more than the L2s hold and fits the last-level cache (with
    // the same margins as above): the few-operand steps then do better with ordinary loads or
    // stores, which leave their lines where the next launch finds them.
    const bool resident = working_set >= L2_TOTAL_BYTES + L2_TOTAL_BYTES / 2 &&
                          working_set <= LAST_LEVEL_CACHE_BYTES + LAST_LEVEL_CACHE_BYTES / 4;
    if (k >= 2 && m == 1) {
        cls = 0;
        t.cache_policy = fits ? 6 : 3;
        // Fan-in 2 to 4 with 64 to 256 MiB in all: NPP (results stored write-back, the operand that is
        // overwritten loaded normally) is 3 to 14 % faster for the whole all-reduce than NNS: ring on
        // 8 to 32 ranks (with PPS on its copy steps) -6 / -10 / -8 % at 64 / 128 / 256 MiB, lane on
        // 4 x 4 x 1, 2 x 2 x 2, 4 x 2 x 1 and 8 x 2 x 1 -3 to -9 %, Rabenseifner -3 %.  At 32 MiB and
        // from 384 MiB on the streaming policies win.
        if (k < 8 && resident) t.cache_policy = 1;
        if (k >= 16) {
            t.block = 1024;
            t.unroll = 4;
        } else if (k >= 8) {
            t.block = 1024;
            t.unroll = 8;
        } else if (k >= 3) {
            // Operands that stream from DRAM want long runs; cache-resident ones small tiles.  What
            // decides is what the step READS: k operands of the result's size.  C2 S1 (k = 4, result
            // 256 MiB, inputs 1 GiB) streams its inputs whatever the loop before it left in the cache:
            // from a cold cache 128 KiB tiles give 6.10 TB/s against 5.65 with 16 KiB tiles; in a loop
            // over the same buffers, where a quarter of the inputs is still cache-resident, they cost
            // 5 % of the step (201 against 191 us).
            const bool reads_fit = (uint64_t)k * bytes_per_operand <= LAST_LEVEL_CACHE_BYTES + LAST_LEVEL_CACHE_BYTES / 4;
            t.block = 1024;
            t.unroll = reads_fit ? 1 : 8;
        } else {
            t.block = fits ? 256 : 1024; // short launches start and drain faster with small workgroups
            t.unroll = 4;
        }
    } else if (k == 1) {
        cls = 2;
        // A broadcast whose copies all fit the last-level cache stores them scope-1, so that whoever
        // reads them next finds them there (the next all-reduce's first step: 16 to 1024 ranks, 64 to
        // 384 MiB in all, -3 to -12 % time against non-temporal stores; from 512 MiB on non-temporal
        // stores win again by 1 to 5 %, and so they do, by 5 to 10 %, when everything fits the L2s).
        // Segments under 64 KiB do not take non-temporal stores well at any size measured (1024
        // ranks, 16 and 32 KiB segments, 0.5 and 1 GiB in all: -7 to -10 % time with scope-1).
        const uint64_t written = (uint64_t)m * bytes_per_operand;
        const bool beyond_l2 = written >= L2_TOTAL_BYTES + L2_TOTAL_BYTES / 2; // 45 MiB: -9 % with scope-1, 48 MiB: +2 %
        // (up to 4 copies: 288 MiB written still gains 2 %, 336 MiB loses 1.5 %, 384 MiB loses 7 %;
        // 15 and 31 copies: 360 MiB gains 8 %, 480 MiB still 3 %)
        const uint64_t most = LAST_LEVEL_CACHE_BYTES + LAST_LEVEL_CACHE_BYTES / (m <= 4 ? 8 : 2);
        const bool keep = beyond_l2 && (written <= most || longest_units < 4096);
        if (m == 1) {
            t.cache_policy = resident ? 7 : 6;
            t.block = fits ? 256 : 1024;
            t.unroll = 4;
        } else if (m <= 4) {
            t.cache_policy = keep ? 7 : fits ? 4 : 7;
            t.block = fits ? 256 : 1024;
            t.unroll = fits ? 1 : 4;
        } else {
            t.cache_policy = keep ? 7 : fits ? 4 : 7;
            t.block = 1024;
            t.unroll = 8;
        }
    } else {
        cls = 1;
        // sources that the previous launch left in the cache: ordinary loads; streamed from DRAM
        // and then overwritten: non-temporal loads (16 MiB pieces of 512 MiB buffers: 5.85 -> 6.3 TB/s)
        t.cache_policy = fits ? 7 : 6;
        if (all_inputs) {
            // the whole all-reduce in one launch: every source is an original input, read once
            // and overwritten; as many stores as loads.  16-bit types keep two sets of eight
            // fp32 accumulators per vector: 64 KiB tiles fit the register file, 128 KiB do not.
            t.cache_policy = fits ? 6 : 3;
            t.block = 1024;
            t.unroll = esize < 4 ? 4 : 8;
        } else if (m >= 8 && m > k) {
            // The all-gathers folded into the reduce: store-dominated, like a broadcast.  A workgroup
            // streams its tile to m destinations, so few large workgroups do better than one per
            // compute unit: C3 (k = 8, m = 128, 1 MiB segments) 128 workgroups of 128 KiB 342 us, 256 of
            // 64 KiB 364; C5 (k = 32, m = 1024, 128 KiB segments) 64 workgroups of 64 KiB 706 us, 256 of
            // 16 KiB 825, 32 of 128 KiB 1162 (with a fan-in of 32 the loads of a 128 KiB tile take too long).
            t.cache_policy = fits ? 4 : 6;
            t.block = 1024;
            t.unroll = k >= 16 ? 4 : 8;
            store_bound = true;
        } else if (k < 8) {
            t.block = 1024;
            t.unroll = 1;
        } else {
            t.block = fits ? 256 : 1024;
            t.unroll = 4;
        }
    }
    if (req.unroll > 0) t.unroll = req.unroll;
    if (req.block > 0) t.block = req.block;
    if (req.cache_policy >= 100) {
        // one digit per step class: reduce, reduce + multi-destination, copy / broadcast
        const int digit[3] = {req.cache_policy / 100, (req.cache_policy / 10) % 10, req.cache_policy % 10};
        t.cache_policy = digit[cls];
    } else if (req.cache_policy >= 0) {
        t.cache_policy = req.cache_policy;
    }
    // a tile should not be much longer than the longest segment of the step
    if (req.unroll <= 0)
        while (t.unroll > 1 && (uint64_t)t.block * t.unroll > longest_units) t.unroll /= 2;
    if (req.block <= 0)
        if (t.block > 256 && (uint64_t)t.block * t.unroll > longest_units) t.block = 256;
    // ... nor so long that the step has fewer workgroups than the GPU has compute units
    const uint64_t vectors = bytes_per_operand / 16;
    constexpr uint64_t COMPUTE_UNITS = 256;
    if (req.unroll <= 0 && !store_bound)
        while (t.unroll > 1 && vectors / ((uint64_t)t.block * t.unroll) < COMPUTE_UNITS) t.unroll /= 2;
    if (req.block <= 0 && !store_bound)
        if (t.block > 256 && vectors / ((uint64_t)t.block * t.unroll) < COMPUTE_UNITS) t.block = 256;
    if (t.unroll == 8 && t.block != 1024) t.unroll = 4; // 128 KiB tiles exist for 1024 lanes only
    return t;
}
} // namespace la

// ---- a schedule bound to device addresses -------------------------------------------------------

struct la_binding {
    std::vector<uint64_t> bufs; // the P device addresses the tables were resolved with
    int device = -1;
    Tuning requested;           // the process-wide setting the launch shapes were derived from
    std::vector<Tuning> shape;  // per step
    void* tables = nullptr;     // one device allocation holding every step's tables
    size_t tables_bytes = 0;
    void* staging = nullptr;    // library-owned staging area (LA_SCHED_STAGED)
    bool used = false;
    std::vector<StepTable> step; // device views
    // the whole schedule as one executable graph of kernel nodes (launch-bound schedules)
    hipStream_t capture_stream = nullptr;
    hipGraph_t graph = nullptr;
    hipGraphExec_t graph_exec = nullptr;
    uint32_t graph_op = 0;       // the operation recorded in the graph's kernel arguments
    bool graph_failed = false;
    // the runs of steps that execute as one column-fused launch each (fused.hip), built on first use
    struct FusedRun {
        void* tables = nullptr;
        FusedTable table;
        int unroll = 0;
        bool ready = false, impossible = false;
    };
    std::vector<FusedRun> fused; // one per run of the schedule's fusion plan
    // which runs the last call launched fused, kept so that a repeat call decides (and allocates) nothing
    struct Selection {
        int fuse = 0, first = -1, last = -1; // the "fuse" knob and the range of steps it was made for
        std::vector<int> run_at;             // per step: the fused run that starts there, or -1
        bool any = false;
    };
    Selection selection;
};

namespace la {

static void drop_graph(la_binding* b)
{
    if (b->graph_exec) (void)hipGraphExecDestroy(b->graph_exec);
    if (b->graph) (void)hipGraphDestroy(b->graph);
    b->graph_exec = nullptr;
    b->graph = nullptr;
    b->graph_failed = false;
}

// Work that a binding's tables serve may still be in flight on whatever streams the caller used.
// Nothing is recorded per call to track it (an event record per all-reduce costs the stream about
// as much as a short kernel); the rare operations that free or rewrite a used binding's tables
// wait for the whole device instead.
static void wait_for_device(int device)
{
    int cur = -1;
    if (hipGetDevice(&cur) != hipSuccess) return;
    if (cur != device && hipSetDevice(device) != hipSuccess) return;
    (void)hipDeviceSynchronize();
    if (cur != device) (void)hipSetDevice(cur);
}

void release_binding(la_binding* b)
{
    if (!b) return;
    if (b->used) wait_for_device(b->device);
    drop_graph(b);
    if (b->capture_stream) (void)hipStreamDestroy(b->capture_stream);
    if (b->tables) (void)hipFree(b->tables);
    for (la_binding::FusedRun& r : b->fused)
        if (r.tables) (void)hipFree(r.tables);
    if (b->staging) (void)hipFree(b->staging);
    delete b;
}

// Fill SegInfo for one segment from its resolved operand addresses; returns its length in
// 16-byte units as the launch sees it.
uint64_t describe_segment(SegInfo& si, uint64_t len, const uint64_t* ptrs, size_t count, size_t esize, size_t k)
{
    // ptrs = k sources followed by the destinations
    si.alias_mask = 0;
    for (size_t t = 0; t < k && t < 64; ++t)
        for (size_t d = k; d < count; ++d)
            if (ptrs[d] == ptrs[t]) si.alias_mask |= uint64_t(1) << t;
    bool congruent = true;
    uint32_t align = 128;
    for (size_t i = 1; i < count; ++i) {
        if (((ptrs[i] ^ ptrs[0]) & 15u) != 0) congruent = false;
        if (((ptrs[i] ^ ptrs[0]) & 127u) != 0) align = 16;
    }
    return finish_segment(si, len, ptrs[0], (uint32_t)esize, congruent, align);
}

// Workgroups per segment of a launch and how the kernel cuts a segment into tiles.
//
// Full tiles counted from a segment's own start suit segments that start and end on multiples of
// the tile size (buffer lengths that are powers of two).  Other lengths ran 3 to 13 % below their
// power-of-two neighbours (measured over 16 to 1024 ranks, 3 to 360 MB each), for two reasons with
// two remedies:
//  * long segments: the tiles straddle the multiples of the tile size in memory.  With the first
//    tile of a segment cut short, so that every later one starts on such a multiple of destination
//    0's address, these lengths run like their neighbours (+5 to +10 %).  The price is up to one
//    more, partly empty workgroup per segment, which costs more than it gains when segments are a
//    few tiles long (up to -5 % below 4 tiles, nothing from 8): aligned from ALIGN_MIN_TILES tiles
//    in the longest segment.  The kernel derives the same lead from the same table entry.
//  * short segments: a ragged last tile among two to seven leaves workgroups of unequal work; the
//    same number of tiles, all of one size, gained 0 to 6 %.
constexpr uint64_t ALIGN_MIN_TILES = 8;

// Edge workgroups of a launch: enough for every segment if any segment has elements outside its
// whole vectors, else none (buffers and partitions that are multiples of 128 bytes: the usual case).
uint32_t plan_edges(const SegInfo* seg, size_t S, size_t esize, const Tuning& shape)
{
    const uint64_t vec = 16 / esize;
    bool any = false;
    for (size_t g = 0; g < S && !any; ++g) any = seg[g].head != 0 || (seg[g].len - seg[g].head) % vec != 0;
    if (!any) return 0;
    const uint64_t per_block = (uint64_t)shape.block / EDGE_LANES;
    return (uint32_t)((S + per_block - 1) / per_block);
}

uint32_t plan_tiles(const SegInfo* seg, const uint64_t* dp, size_t S, size_t m, size_t esize, const Tuning& shape,
                    uint64_t longest, uint32_t* tiling)
{
    const uint64_t tile = (uint64_t)shape.block * (uint64_t)shape.unroll; // 16-byte vectors
    if (longest < ALIGN_MIN_TILES * tile) {
        *tiling = TILING_EQUAL;
        return tiles_for(longest, shape);
    }
    *tiling = TILING_PLAIN;
    const uint64_t vec = 16 / esize;
    uint64_t most = 1;
    bool any_lead = false;
    for (size_t g = 0; g < S; ++g) {
        uint64_t units, lead = 0;
        if (seg[g].vec_ok) {
            units = (seg[g].len - seg[g].head) / vec;
            lead = ((dp[g * m] + (uint64_t)seg[g].head * esize) & (tile * 16u - 1u)) / 16u;
        } else {
            units = (seg[g].len + vec - 1) / vec; // the unaligned path counts from the segment's start
        }
        any_lead = any_lead || lead != 0;
        most = std::max(most, (lead + units + tile - 1) / tile);
    }
    if (!any_lead) return tiles_for(longest, shape);
    *tiling = TILING_ALIGNED;
    return (uint32_t)most;
}

namespace {

struct HostTables {
    std::vector<unsigned char> blob;
    std::vector<StepTable> view; // pointers are offsets until relocated
};

// Resolve every (buffer, offset) operand of `steps` against `base` addresses and lay the tables
// out in one blob.  base[P] is the staging area.
void resolve_tables(const std::vector<Step>& steps, const std::vector<uint64_t>& base, size_t esize, const Tuning& tune,
                    uint64_t working_set, HostTables& out, std::vector<Tuning>& shapes)
{
    uint64_t total = 0;
    std::vector<uint64_t> seg_at(steps.size()), src_at(steps.size()), dst_at(steps.size());
    for (size_t i = 0; i < steps.size(); ++i) {
        const Step& p = steps[i];
        const size_t S = p.num_segments();
        seg_at[i] = total;
        total = align_up(total + S * sizeof(SegInfo), 256);
        src_at[i] = total;
        total = align_up(total + S * p.k * sizeof(uint64_t), 256);
        dst_at[i] = total;
        total = align_up(total + S * p.m * sizeof(uint64_t), 256);
    }
    out.blob.assign(total ? total : 256, 0);
    out.view.resize(steps.size());
    shapes.resize(steps.size());
    // Small schedules run every step with one workgroup size.  A launch whose workgroup size differs
    // from the previous launch's starts about 1.6 us later than one of the same size (plain HIP
    // launches of trivial dependent kernels on one stream: 2.8 us per launch with one size, 4.4 us
    // alternating 256 and 1024 lanes; a change of the register count costs nothing), which long
    // launches hide and short ones do not: 16 ranks x 1 / 2 / 4 MiB 19.4 / 26.1 / 35.4 -> 14.1 / 18.7 /
    // 32.3 us per all-reduce, 64 ranks x 256 KiB and 1 MiB 20.5 -> 15.6 and 41.3 -> 33.0, 8 ranks x
    // 4 MiB 26.0 -> 18.9.  The vectors per lane stay each step's own.  At 80 MiB in all one size still
    // gains 5 to 19 %, at 96 MiB nothing, beyond that it is +-2 % either way.
    Tuning request = tune;
    if (working_set <= SMALL_SCHEDULE_BYTES && request.block <= 0) request.block = 256;
    std::vector<uint64_t> all, cur_dst, cand_dst;
    for (size_t i = 0; i < steps.size(); ++i) {
        const Step& p = steps[i];
        const size_t S = p.num_segments(), k = (size_t)p.k, m = (size_t)p.m;
        SegInfo* seg = reinterpret_cast<SegInfo*>(out.blob.data() + seg_at[i]);
        uint64_t* sp = reinterpret_cast<uint64_t*>(out.blob.data() + src_at[i]);
        uint64_t* dp = reinterpret_cast<uint64_t*>(out.blob.data() + dst_at[i]);
        // Launch segments: a table segment continues the one before it when every source range starts
        // where that one's ended and the destination ranges do too, as a set (a piece is stored to the
        // same buffers whoever reduces it; only the order of the list differs, and every destination
        // receives the same value).  Such runs are launched as one segment: the pieces of a part in the
        // inter-node step (C5: 1024 segments of 4 KiB become 32 of 128 KiB), every segment of the
        // one-launch form.  Same sums in the same order; the logical tables stay as generated.
        size_t launched = 0; // segments written so far
        uint64_t step_elems = 0;
        bool cur_dst_valid = false;
        for (size_t g = 0; g < S; ++g) {
            step_elems += p.len[g];
            uint64_t* s_new = sp + launched * k;
            uint64_t* d_new = dp + launched * m;
            for (size_t t = 0; t < k; ++t) s_new[t] = base[p.src[g * k + t].buf] + p.src[g * k + t].off * esize;
            for (size_t d = 0; d < m; ++d) d_new[d] = base[p.dst[g * m + d].buf] + p.dst[g * m + d].off * esize;
            if (tune.merge && launched > 0) {
                const uint64_t shift = seg[launched - 1].len * esize;
                const uint64_t* s_old = s_new - k;
                const uint64_t* d_old = d_new - m;
                bool same = true;
                for (size_t t = 0; t < k && same; ++t) same = s_new[t] == s_old[t] + shift;
                if (same && m == 1) same = d_new[0] == d_old[0] + shift;
                if (same && m > 1) {
                    if (!cur_dst_valid) {
                        cur_dst.assign(d_old, d_old + m);
                        std::sort(cur_dst.begin(), cur_dst.end());
                        cur_dst_valid = true;
                    }
                    cand_dst.assign(d_new, d_new + m);
                    std::sort(cand_dst.begin(), cand_dst.end());
                    for (size_t d = 0; d < m && same; ++d) same = cand_dst[d] == cur_dst[d] + shift;
                }
                if (same) {
                    seg[launched - 1].len += p.len[g];
                    continue;
                }
            }
            seg[launched].len = p.len[g];
            cur_dst_valid = false;
            ++launched;
        }
        uint64_t longest = 0;
        for (size_t g = 0; g < launched; ++g) {
            all.assign(sp + g * k, sp + (g + 1) * k);
            all.insert(all.end(), dp + g * m, dp + (g + 1) * m);
            longest = std::max(longest, describe_segment(seg[g], seg[g].len, all.data(), all.size(), esize, k));
        }
        StepTable& v = out.view[i];
        v.seg = reinterpret_cast<const SegInfo*>(seg_at[i]);
        v.src_ptr = reinterpret_cast<const uint64_t*>(src_at[i]);
        v.dst_ptr = reinterpret_cast<const uint64_t*>(dst_at[i]);
        v.k = (uint32_t)p.k;
        v.m = (uint32_t)p.m;
        v.group = (uint32_t)p.group;
        v.num_segments = (uint32_t)launched;
        shapes[i] = resolve_tuning(request, v.k, v.m, longest, step_elems * esize,
                                   p.stage == LA_STAGE_S1_S2_S3 && p.k > 1 && p.m > 1, esize, working_set);
        v.tiles_per_seg = plan_tiles(seg, dp, launched, m, esize, shapes[i], longest, &v.tiling);
        v.edge_blocks = plan_edges(seg, launched, esize, shapes[i]);
    }
}

void relocate(std::vector<StepTable>& view, const void* device_base)
{
    const uint64_t b = reinterpret_cast<uint64_t>(device_base);
    for (StepTable& v : view) {
        v.seg = reinterpret_cast<const SegInfo*>(b + reinterpret_cast<uint64_t>(v.seg));
        v.src_ptr = reinterpret_cast<const uint64_t*>(b + reinterpret_cast<uint64_t>(v.src_ptr));
        v.dst_ptr = reinterpret_cast<const uint64_t*>(b + reinterpret_cast<uint64_t>(v.dst_ptr));
    }
}

// addr layout: [0, P) the (receive) buffers, [P] the staging area (filled by bind), and for an
// out-of-place schedule [P + 1, 2P + 1) the send buffers.
la_status_t check_buffers(const la_schedule& s, void* const* bufs, const void* const* sendbufs,
                          std::vector<uint64_t>& addr)
{
    const int P = s.nbuf;
    const size_t e = dtype_size(s.dtype);
    const bool oop = (s.flags & LA_SCHED_OUT_OF_PLACE) != 0;
    if (oop != (sendbufs != nullptr))
        return fail(LA_ERR_INVALID_ARG, oop ? "the schedule is out-of-place: use la_allreduce_emulated_out_of_place"
                                            : "the schedule was not built with LA_SCHED_OUT_OF_PLACE");
    addr.assign(oop ? 2 * P + 1 : P + 1, 0);
    std::vector<uint64_t> sorted;
    for (int r = 0; r < P; ++r) {
        if (!bufs[r]) return fail(LA_ERR_INVALID_ARG, "bufs[%d] is NULL", r);
        addr[r] = reinterpret_cast<uint64_t>(bufs[r]);
        if (addr[r] % e) return fail(LA_ERR_INVALID_ARG, "bufs[%d] is not aligned to the element size", r);
        sorted.push_back(addr[r]);
        if (oop) {
            if (!sendbufs[r]) return fail(LA_ERR_INVALID_ARG, "sendbufs[%d] is NULL", r);
            addr[P + 1 + r] = reinterpret_cast<uint64_t>(sendbufs[r]);
            if (addr[P + 1 + r] % e) return fail(LA_ERR_INVALID_ARG, "sendbufs[%d] is not aligned to the element size", r);
            sorted.push_back(addr[P + 1 + r]);
        }
    }
    std::sort(sorted.begin(), sorted.end());
    for (size_t r = 1; r < sorted.size(); ++r)
        if (sorted[r] < sorted[r - 1] + s.n * e)
            return fail(LA_ERR_INVALID_ARG, "buffers overlap (or one pointer was passed twice)");
    return LA_OK;
}

// Serialises the library's synchronous device calls (allocation, table upload) with its graph
// captures, across all schedules of the process.
std::mutex g_device_mu;

constexpr size_t MAX_BINDINGS = 8;

// Make sched.bound.front() describe `addr` on the current device with the current tile shape.
la_status_t bind(const la_schedule& s, std::vector<uint64_t>& addr, const Tuning& tune)
{
    int dev = -1;
    LA_HIP(hipGetDevice(&dev));
    const int P = s.nbuf;
    const std::vector<uint64_t> key = addr; // caller addresses only: the staging slot is still 0
    for (size_t i = 0; i < s.bound.size(); ++i) {
        la_binding* c = s.bound[i];
        if (c->device == dev && c->requested == tune && c->bufs == key) {
            if (i) std::rotate(s.bound.begin(), s.bound.begin() + i, s.bound.begin() + i + 1); // to the front
            return LA_OK;
        }
    }
    std::lock_guard<std::mutex> device_lock(g_device_mu); // not while another schedule records its graph
    la_binding* b = nullptr;
    // a staged schedule owns a staging area per binding, which can be large: keep one
    const size_t keep = s.staging_elems ? 1 : MAX_BINDINGS;
    if (s.bound.size() >= keep) {
        // recycle the least recently used one (its allocations are reused when it is on this device)
        b = s.bound.back();
        s.bound.pop_back();
        if (b->used) wait_for_device(b->device); // earlier work still reads its tables
        if (b->device != dev) {
            release_binding(b);
            b = nullptr;
        }
    }
    if (!b) {
        b = new (std::nothrow) la_binding;
        if (!b) return fail(LA_ERR_OUT_OF_MEMORY, "out of host memory");
        b->device = dev;
    }
    s.bound.insert(s.bound.begin(), b);
    b->bufs.clear(); // not a match for anything until it is complete
    const size_t e = dtype_size(s.dtype);
    if (s.staging_elems && !b->staging) {
        if (hipMalloc(&b->staging, s.staging_elems * e) != hipSuccess) {
            b->staging = nullptr;
            return fail(LA_ERR_OUT_OF_MEMORY, "cannot allocate %llu bytes of staging",
                        (unsigned long long)(s.staging_elems * e));
        }
    }
    addr[P] = reinterpret_cast<uint64_t>(b->staging);
    HostTables ht;
    std::vector<Tuning> shapes;
    try {
        resolve_tables(s.steps, addr, e, tune, (uint64_t)s.nbuf * s.n * e, ht, shapes);
    } catch (const std::bad_alloc&) {
        return fail(LA_ERR_OUT_OF_MEMORY, "out of host memory");
    }
    if (b->tables && b->tables_bytes != ht.blob.size()) {
        LA_HIP(hipFree(b->tables));
        b->tables = nullptr;
    }
    if (!b->tables) {
        if (hipMalloc(&b->tables, ht.blob.size()) != hipSuccess) {
            b->tables = nullptr;
            return fail(LA_ERR_OUT_OF_MEMORY, "cannot allocate %zu bytes of device tables", ht.blob.size());
        }
        b->tables_bytes = ht.blob.size();
    }
    LA_HIP(hipMemcpy(b->tables, ht.blob.data(), ht.blob.size(), hipMemcpyHostToDevice));
    relocate(ht.view, b->tables);
    b->step = std::move(ht.view);
    b->bufs = key;
    drop_graph(b); // recorded launches point at the old tables
    for (la_binding::FusedRun& r : b->fused)
        if (r.tables) (void)hipFree(r.tables);
    b->fused.clear();
    b->selection = la_binding::Selection();
    b->requested = tune;
    b->shape = std::move(shapes);
    b->used = false;
    return LA_OK;
}

// Record every launch of the schedule into a graph of kernel nodes.  Only kernel launches are
// captured (no memset or copy nodes).  On failure the binding falls back to stream launches.
la_status_t capture_graph(const la_schedule_t* sched, la_binding* b, uint32_t op)
{
    // Relaxed mode: the capture holds nothing but this library's kernel launches on a private
    // stream, so other threads (the caller's allocator, another schedule's table upload) need not
    // be kept from synchronous calls while it runs; in the stricter modes such a call in another
    // thread was seen to fail and to invalidate the capture.  The library's own synchronous device
    // calls are kept out of the window by g_device_mu as well.
    std::lock_guard<std::mutex> device_lock(g_device_mu);
    if (!b->capture_stream) LA_HIP(hipStreamCreateWithFlags(&b->capture_stream, hipStreamNonBlocking));
    LA_HIP(hipStreamBeginCapture(b->capture_stream, hipStreamCaptureModeRelaxed));
    la_status_t st = LA_OK;
    for (size_t i = 0; i < b->step.size() && st == LA_OK; ++i) {
        StepTable t = b->step[i];
        t.op = op;
        st = launch_step(t, sched->dtype, b->shape[i], b->capture_stream);
    }
    hipGraph_t g = nullptr;
    const hipError_t e = hipStreamEndCapture(b->capture_stream, &g);
    if (st != LA_OK || e != hipSuccess || !g) {
        if (g) (void)hipGraphDestroy(g);
        return st != LA_OK ? st : fail(LA_ERR_DEVICE, "hipStreamEndCapture failed: %s", hipGetErrorString(e));
    }
    hipGraphExec_t x = nullptr;
    if (hipGraphInstantiate(&x, g, nullptr, nullptr, 0) != hipSuccess) {
        (void)hipGraphDestroy(g);
        return fail(LA_ERR_DEVICE, "hipGraphInstantiate failed");
    }
    b->graph = g;
    b->graph_exec = x;
    b->graph_op = op;
    return LA_OK;
}

// Device tables of one column-fused run for the binding's addresses.  Sets `impossible` when the
// addresses do not allow it (then its steps are launched one by one).
la_status_t build_fused(const la_schedule& s, la_binding* b, size_t run, const std::vector<uint64_t>& addr)
{
    const FusionRun& f = s.fusion.runs[run];
    la_binding::FusedRun& out = b->fused[run];
    out.impossible = true;
    const size_t e = dtype_size(s.dtype);
    for (size_t i = 0; i < addr.size(); ++i)
        if (i != (size_t)s.nbuf && ((addr[i] ^ addr[0]) & 15u) != 0) return LA_OK; // no common 16-byte phase
    const size_t C = f.chain_lo.size();
    const uint64_t vec = 16 / e;
    std::vector<ChainInfo> chain(C);
    uint64_t O = 0; // records, every chain padded to a multiple of FUSED_CHAIN_PAD
    for (size_t c = 0; c < C; ++c) {
        const uint64_t first = (addr[0] + f.chain_lo[c] * e) & 15u;
        uint64_t head = ((16 - first) & 15u) / e;
        if (head > f.chain_len[c]) head = f.chain_len[c];
        chain[c].first_op = O;
        chain[c].num_ops = (uint32_t)align_up(f.chain_first[c + 1] - f.chain_first[c], FUSED_CHAIN_PAD);
        chain[c].head = (uint32_t)head;
        chain[c].nvec = (f.chain_len[c] - head) / vec;
        chain[c].tail = (uint32_t)((f.chain_len[c] - head) % vec);
        chain[c].pad = 0;
        O += chain[c].num_ops;
    }
    // One vector per lane: a wave takes 1 KiB of its chain through all operations.
    // One more workgroup per chain that has elements outside its whole vectors.
    auto workgroups_for = [&](uint64_t unroll) {
        uint64_t w = 0;
        for (size_t c = 0; c < C; ++c) w += (chain[c].nvec + FUSED_LANES * unroll - 1) / (FUSED_LANES * unroll);
        return w;
    };
    const uint64_t unroll = 1;
    uint64_t W = workgroups_for(unroll);
    for (size_t c = 0; c < C; ++c) W += chain[c].head + chain[c].tail > 0 ? 1 : 0;
    if (W > 0x7fffffffull || C > 0xffffffffull) return LA_OK;
    const uint64_t chain_at = 0;
    const uint64_t op_at = align_up(chain_at + C * sizeof(ChainInfo), 256);
    const uint64_t wgc_at = align_up(op_at + O * sizeof(FusedOp), 256);
    const uint64_t wgt_at = align_up(wgc_at + W * sizeof(uint32_t), 256);
    const uint64_t total = align_up(wgt_at + W * sizeof(uint32_t), 256);
    std::vector<unsigned char> blob(total, 0); // padding records are all zeros
    std::copy(chain.begin(), chain.end(), reinterpret_cast<ChainInfo*>(blob.data() + chain_at));
    FusedOp* op = reinterpret_cast<FusedOp*>(blob.data() + op_at);
    for (size_t c = 0; c < C; ++c) {
        FusedOp* to_op = op + chain[c].first_op;
        for (uint64_t o = f.chain_first[c]; o < f.chain_first[c + 1]; ++o, ++to_op) {
            const Step& p = s.steps[f.op_step[o]];
            const size_t g = f.op_seg[o];
            to_op->live = 1;
            to_op->k = (uint16_t)p.k;
            to_op->m = (uint16_t)p.m;
            to_op->prefetch = (int16_t)f.op_prefetch[o];
            to_op->forward = b->requested.forward ? (int16_t)f.op_forward[o] : (int16_t)-1;
            // a source that comes from registers is not also requested ahead of time
            if (to_op->forward >= 0 && to_op->forward == to_op->prefetch) to_op->prefetch = -1;
            // the chain's first element in every operand (all operands of a segment share its offset)
            uint64_t* to = to_op->addr;
            for (int t = 0; t < p.k; ++t) *to++ = addr[p.src[g * p.k + t].buf] + f.chain_lo[c] * e;
            for (int d = 0; d < p.m; ++d) *to++ = addr[p.dst[g * p.m + d].buf] + f.chain_lo[c] * e;
        }
    }
    // blocks of eight operations that are all "add what I hold to a prefetched input" or all "store
    // what I hold", with the four operations behind them wanting a prefetch (resp. none): the kernel
    // runs these without a branch
    for (size_t c = 0; c < C; ++c) {
        FusedOp* o = op + chain[c].first_op;
        const uint32_t count = chain[c].num_ops;
        auto at = [&](uint32_t i) -> const FusedOp* { return i < count ? o + i : nullptr; };
        for (uint32_t j = 0; j < count; j += FUSED_CHAIN_PAD) {
            bool add = true, copy = true;
            for (uint32_t i = j; i < j + FUSED_CHAIN_PAD; ++i) {
                const FusedOp& x = o[i];
                add = add && x.live == 1 && x.k == 2 && x.m == 1 && x.prefetch == 0 && x.forward == 1;
                copy = copy && x.live == 1 && x.k == 1 && x.m == 1 && x.forward == 0;
            }
            for (uint32_t i = j + 4; i < j + FUSED_CHAIN_PAD + 4; ++i) {
                const FusedOp* x = at(i);
                const bool wants = x && (x->live & 1u) && x->prefetch >= 0;
                add = add && wants && x->prefetch == 0;
                copy = copy && !wants;
            }
            o[j].live |= (add ? FUSED_BLOCK_ADD : copy ? FUSED_BLOCK_COPY : FUSED_BLOCK_GENERAL) << 8;
        }
    }
    uint32_t* wgc = reinterpret_cast<uint32_t*>(blob.data() + wgc_at);
    uint32_t* wgt = reinterpret_cast<uint32_t*>(blob.data() + wgt_at);
    uint64_t w = 0;
    for (size_t c = 0; c < C; ++c) {
        const uint64_t tiles = (chain[c].nvec + FUSED_LANES * unroll - 1) / (FUSED_LANES * unroll);
        for (uint64_t t = 0; t < tiles; ++t, ++w) {
            wgc[w] = (uint32_t)c;
            wgt[w] = (uint32_t)t;
        }
    }
    for (size_t c = 0; c < C; ++c)
        if (chain[c].head + chain[c].tail > 0) {
            wgc[w] = (uint32_t)c;
            wgt[w++] = FUSED_EDGE_TILE;
        }
    std::lock_guard<std::mutex> device_lock(g_device_mu);
    if (hipMalloc(&out.tables, total) != hipSuccess) {
        out.tables = nullptr;
        (void)hipGetLastError();
        return LA_OK; // no room for the fused tables: launch step by step
    }
    LA_HIP(hipMemcpy(out.tables, blob.data(), total, hipMemcpyHostToDevice));
    const uint64_t base = reinterpret_cast<uint64_t>(out.tables);
    out.table.chain = reinterpret_cast<const ChainInfo*>(base + chain_at);
    out.table.op = reinterpret_cast<const FusedOp*>(base + op_at);
    out.table.wg_chain = reinterpret_cast<const uint32_t*>(base + wgc_at);
    out.table.wg_tile = reinterpret_cast<const uint32_t*>(base + wgt_at);
    out.table.workgroups = (uint32_t)W;
    out.unroll = (int)unroll;
    out.ready = true;
    out.impossible = false;
    return LA_OK;
}

// A binding that was made for exactly these pointers (in this order) on this device with this
// tuning: the set was validated when it was bound.  No allocation, no sort: a repeat call costs one
// comparison of P addresses.
la_binding* find_binding(const la_schedule& s, void* const* bufs, const void* const* sendbufs, int dev,
                         const Tuning& tune)
{
    const size_t P = (size_t)s.nbuf;
    const bool oop = (s.flags & LA_SCHED_OUT_OF_PLACE) != 0;
    if (oop != (sendbufs != nullptr)) return nullptr;
    for (size_t i = 0; i < s.bound.size(); ++i) {
        la_binding* c = s.bound[i];
        if (c->device != dev || !(c->requested == tune) || c->bufs.size() != (oop ? 2 * P + 1 : P + 1)) continue;
        bool same = true;
        for (size_t r = 0; r < P && same; ++r) same = c->bufs[r] == reinterpret_cast<uint64_t>(bufs[r]);
        for (size_t r = 0; oop && r < P && same; ++r) same = c->bufs[P + 1 + r] == reinterpret_cast<uint64_t>(sendbufs[r]);
        if (!same) continue;
        if (i) std::rotate(s.bound.begin(), s.bound.begin() + i, s.bound.begin() + i + 1); // to the front
        return c;
    }
    return nullptr;
}

la_status_t run_steps(const la_schedule_t* sched, void* const* bufs, const void* const* sendbufs, int first,
                      int last, uint32_t op, void* hip_stream)
{
    la_status_t st = LA_OK;
    std::lock_guard<std::mutex> lock(sched->mu);
    const Tuning tune = current_tuning();
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) dev = -1; // reported below, after the arguments have been checked
    la_binding* b = dev >= 0 ? find_binding(*sched, bufs, sendbufs, dev, tune) : nullptr;
    if (!b) {
        try {
            std::vector<uint64_t> fresh;
            st = check_buffers(*sched, bufs, sendbufs, fresh);
            if (st != LA_OK) return st;
            st = bind(*sched, fresh, tune);
            if (st != LA_OK) return st;
        } catch (const std::bad_alloc&) {
            return fail(LA_ERR_OUT_OF_MEMORY, "out of host memory");
        }
        b = sched->bound.front();
    }
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const int mode = g_graph.load();
    const bool whole = first == 0 && last == (int)sched->steps.size();
    const bool want_graph = whole && last > 0 && (mode == 1 || (mode < 0 && last >= GRAPH_MIN_STEPS));
    // which runs of steps go out as one column-fused launch each
    const int fuse = g_fuse.load();
    la_binding::Selection& sel = b->selection;
    if (fuse == 0 || last - first < 2) {
        sel.any = false;
        sel.first = -1;
    } else if (sel.fuse != fuse || sel.first != first || sel.last != last) {
        sel.first = -1; // not valid until complete
        sel.any = false;
        try {
            analyse_fusion(*sched);
            const std::vector<FusionRun>& runs = sched->fusion.runs;
            if (b->fused.size() != runs.size()) b->fused.resize(runs.size());
            sel.run_at.assign(sched->steps.size(), -1);
            for (size_t r = 0; r < runs.size(); ++r) {
                const FusionRun& f = runs[r];
                if (f.first_step < first || f.first_step + f.num_steps > last) continue;
                if (fuse < 0 && !f.automatic()) continue;
                if (!b->fused[r].ready && !b->fused[r].impossible) {
                    std::vector<uint64_t> addr = b->bufs; // the caller's addresses; the staging slot is not used by a run
                    st = build_fused(*sched, b, r, addr);
                    if (st != LA_OK) return st;
                }
                if (b->fused[r].ready) {
                    sel.run_at[f.first_step] = (int)r;
                    sel.any = true;
                }
            }
            sel.fuse = fuse;
            sel.first = first;
            sel.last = last;
        } catch (const std::bad_alloc&) {
            sched->fusion = FusionPlan();
            sel.any = false;
        }
    }
    const bool any_fused = sel.any;
    const std::vector<int>& run_at = sel.run_at;
    bool launched = false;
    if (!any_fused && want_graph && !b->graph_failed) {
        if (b->graph_exec && b->graph_op != op) drop_graph(b);
        if (!b->graph_exec && capture_graph(sched, b, op) != LA_OK) b->graph_failed = true;
        if (b->graph_exec) {
            if (hipGraphLaunch(b->graph_exec, stream) == hipSuccess) {
                launched = true;
            } else {
                (void)hipGetLastError(); // the graph is given up; the steps are launched one by one
                drop_graph(b);
                b->graph_failed = true;
            }
        }
    }
    if (!launched) {
        for (int i = first; i < last;) {
            if (any_fused && run_at[i] >= 0) {
                const la_binding::FusedRun& r = b->fused[run_at[i]];
                FusedTable t = r.table;
                t.op_code = op;
                st = launch_fused(t, sched->dtype, r.unroll, hip_stream);
                if (st != LA_OK) return st;
                g_fused_launches.fetch_add(1);
                i += sched->fusion.runs[run_at[i]].num_steps;
                continue;
            }
            StepTable t = b->step[i];
            t.op = op;
            st = launch_step(t, sched->dtype, b->shape[i], hip_stream);
            if (st != LA_OK) return st;
            ++i;
        }
    }
    b->used = true;
    return LA_OK;
}

} // namespace
} // namespace la

namespace la {
la_status_t check_reduce_segments_args(const char* who, const void* dst, const void* const* srcs, int k,
                                       const size_t* seg_offsets, size_t num_segments, size_t seg_len, la_dtype_t dtype,
                                       la_op_t op, bool* nothing)
{
    *nothing = false;
    if (!known_op((int)op)) return fail(LA_ERR_UNSUPPORTED, "%s: unknown operation %d", who, (int)op);
    if (!known_dtype((int)dtype)) return fail(LA_ERR_UNSUPPORTED, "%s: unknown dtype %d", who, (int)dtype);
    if (k < 0) return fail(LA_ERR_INVALID_ARG, "%s: k is negative", who);
    if (!dst) return fail(LA_ERR_INVALID_ARG, "%s: dst is NULL", who);
    if (k > 0 && !srcs) return fail(LA_ERR_INVALID_ARG, "%s: srcs is NULL", who);
    if (num_segments > 0 && !seg_offsets) return fail(LA_ERR_INVALID_ARG, "%s: seg_offsets is NULL", who);
    const size_t e = dtype_size(dtype);
    if (reinterpret_cast<uint64_t>(dst) % e) return fail(LA_ERR_INVALID_ARG, "%s: dst is not aligned to the element size", who);
    for (int t = 0; t < k; ++t) {
        if (!srcs[t]) return fail(LA_ERR_INVALID_ARG, "%s: srcs[%d] is NULL", who, t);
        if (reinterpret_cast<uint64_t>(srcs[t]) % e)
            return fail(LA_ERR_INVALID_ARG, "%s: srcs[%d] is not aligned to the element size", who, t);
        if (srcs[t] == dst) return fail(LA_ERR_INVALID_ARG, "%s: srcs[%d] aliases dst", who, t);
    }
    if (k == 0 || num_segments == 0 || seg_len == 0) {
        *nothing = true; // nothing to add
        return LA_OK;
    }
    if (num_segments > 0xffffffffull) return fail(LA_ERR_INVALID_ARG, "%s: too many segments", who);
    return LA_OK;
}
} // namespace la

// ---- pinned upload chunks for one-shot tables ----------------------------------------------------
// la_reduce_segments builds its tables in pinned host memory so that the upload is a true
// asynchronous copy and the call never waits for the GPU.  A chunk is reused once the copy that
// read it has completed (its event has fired).

namespace la {
namespace {

struct PinnedChunk {
    void* host = nullptr;
    uint64_t bytes = 0;
    hipEvent_t done = nullptr;
    bool in_flight = false;
    int device = -1;
};

std::mutex g_pool_mu;
std::vector<PinnedChunk*> g_pool;

la_status_t acquire_pinned(uint64_t bytes, PinnedChunk** out)
{
    int dev = -1;
    LA_HIP(hipGetDevice(&dev));
    for (PinnedChunk* c : g_pool) {
        if (c->device != dev || c->bytes < bytes) continue;
        if (c->in_flight) {
            if (hipEventQuery(c->done) != hipSuccess) continue;
            c->in_flight = false;
        }
        *out = c;
        return LA_OK;
    }
    PinnedChunk* c = new (std::nothrow) PinnedChunk;
    if (!c) return fail(LA_ERR_OUT_OF_MEMORY, "out of host memory");
    c->bytes = std::max<uint64_t>(align_up(bytes, 4096), 64 * 1024);
    c->device = dev;
    if (hipHostMalloc(&c->host, c->bytes, hipHostMallocDefault) != hipSuccess) {
        delete c;
        return fail(LA_ERR_OUT_OF_MEMORY, "cannot allocate %llu bytes of pinned host memory",
                    (unsigned long long)bytes);
    }
    if (hipEventCreateWithFlags(&c->done, hipEventDisableTiming) != hipSuccess) {
        (void)hipHostFree(c->host);
        delete c;
        return fail(LA_ERR_DEVICE, "hipEventCreate failed");
    }
    g_pool.push_back(c);
    *out = c;
    return LA_OK;
}

} // namespace
} // namespace la

// ---- C ABI --------------------------------------------------------------------------------------

extern "C" {

la_status_t la_allreduce_emulated(const la_schedule_t* sched, void* const* bufs, size_t n, la_dtype_t dtype,
                                  la_op_t op, void* hip_stream)
{
    if (!sched) return fail(LA_ERR_INVALID_ARG, "la_allreduce_emulated: schedule is NULL");
    if (!bufs) return fail(LA_ERR_INVALID_ARG, "la_allreduce_emulated: bufs is NULL");
    if (!known_op((int)op)) return fail(LA_ERR_UNSUPPORTED, "la_allreduce_emulated: unknown operation %d", (int)op);
    if (!known_dtype((int)dtype))
        return fail(LA_ERR_UNSUPPORTED, "la_allreduce_emulated: unknown dtype %d", (int)dtype);
    if (n != sched->n || dtype != sched->dtype)
        return fail(LA_ERR_INVALID_ARG, "la_allreduce_emulated: n/dtype differ from the schedule's (%llu, %d)",
                    (unsigned long long)sched->n, (int)sched->dtype);
    return run_steps(sched, bufs, nullptr, 0, (int)sched->steps.size(), (uint32_t)op, hip_stream);
}

la_status_t la_allreduce_emulated_out_of_place(const la_schedule_t* sched, const void* const* sendbufs,
                                               void* const* recvbufs, size_t n, la_dtype_t dtype, la_op_t op,
                                               void* hip_stream)
{
    if (!sched) return fail(LA_ERR_INVALID_ARG, "la_allreduce_emulated_out_of_place: schedule is NULL");
    if (!sendbufs || !recvbufs) return fail(LA_ERR_INVALID_ARG, "la_allreduce_emulated_out_of_place: a buffer array is NULL");
    if (!known_op((int)op)) return fail(LA_ERR_UNSUPPORTED, "la_allreduce_emulated_out_of_place: unknown operation %d", (int)op);
    if (!known_dtype((int)dtype))
        return fail(LA_ERR_UNSUPPORTED, "la_allreduce_emulated_out_of_place: unknown dtype %d", (int)dtype);
    if (n != sched->n || dtype != sched->dtype)
        return fail(LA_ERR_INVALID_ARG, "la_allreduce_emulated_out_of_place: n/dtype differ from the schedule's (%llu, %d)",
                    (unsigned long long)sched->n, (int)sched->dtype);
    return run_steps(sched, recvbufs, sendbufs, 0, (int)sched->steps.size(), (uint32_t)op, hip_stream);
}

la_status_t la_schedule_run_steps(const la_schedule_t* sched, int first_step, int num_steps, void* const* bufs,
                                  la_op_t op, void* hip_stream)
{
    if (!sched) return fail(LA_ERR_INVALID_ARG, "la_schedule_run_steps: schedule is NULL");
    if (!bufs) return fail(LA_ERR_INVALID_ARG, "la_schedule_run_steps: bufs is NULL");
    if (!known_op((int)op)) return fail(LA_ERR_UNSUPPORTED, "la_schedule_run_steps: unknown operation %d", (int)op);
    if (first_step < 0 || num_steps < 0 || first_step > (int)sched->steps.size() ||
        num_steps > (int)sched->steps.size() - first_step)
        return fail(LA_ERR_INVALID_ARG, "la_schedule_run_steps: steps [%d, %d + %d) out of range", first_step, first_step,
                    num_steps);
    if (num_steps == 0) return LA_OK;
    return run_steps(sched, bufs, nullptr, first_step, first_step + num_steps, (uint32_t)op, hip_stream);
}

la_status_t la_schedule_run_step(const la_schedule_t* sched, int step, void* const* bufs, void* hip_stream)
{
    if (!sched) return fail(LA_ERR_INVALID_ARG, "la_schedule_run_step: schedule is NULL");
    if (!bufs) return fail(LA_ERR_INVALID_ARG, "la_schedule_run_step: bufs is NULL");
    if (step < 0 || step >= (int)sched->steps.size())
        return fail(LA_ERR_INVALID_ARG, "la_schedule_run_step: step %d out of range", step);
    return run_steps(sched, bufs, nullptr, step, step + 1, (uint32_t)LA_SUM, hip_stream);
}

// the launch tables of one step for buffers at the given addresses (host only)
static la_status_t plan_one_step(const char* who, const la_schedule_t* sched, int step, const void* const* bufs,
                                 const void* const* sendbufs, const void* staging, HostTables& ht,
                                 std::vector<Tuning>& shapes)
{
    if (!sched) return fail(LA_ERR_INVALID_ARG, "%s: schedule is NULL", who);
    if (!bufs) return fail(LA_ERR_INVALID_ARG, "%s: bufs is NULL", who);
    if (step < 0 || step >= (int)sched->steps.size()) return fail(LA_ERR_INVALID_ARG, "%s: step %d out of range", who, step);
    try {
        std::vector<uint64_t> addr;
        la_status_t st = check_buffers(*sched, const_cast<void* const*>(bufs), sendbufs, addr);
        if (st != LA_OK) return st;
        const size_t e = dtype_size(sched->dtype);
        addr[sched->nbuf] = reinterpret_cast<uint64_t>(staging);
        if (sched->staging_elems > 0 && (addr[sched->nbuf] == 0 || addr[sched->nbuf] % 16))
            return fail(LA_ERR_INVALID_ARG, "%s: the schedule is staged: pass a 16-byte aligned staging address", who);
        const std::vector<Step> one(1, sched->steps[step]);
        resolve_tables(one, addr, e, current_tuning(), (uint64_t)sched->nbuf * sched->n * e, ht, shapes);
    } catch (const std::bad_alloc&) {
        return fail(LA_ERR_OUT_OF_MEMORY, "%s: out of host memory", who);
    }
    return LA_OK;
}

la_status_t la_schedule_launch_plan(const la_schedule_t* sched, int step, const void* const* bufs,
                                    const void* const* sendbufs, const void* staging, la_launch_plan_t* out)
{
    if (!out) return fail(LA_ERR_INVALID_ARG, "la_schedule_launch_plan: out is NULL");
    HostTables ht;
    std::vector<Tuning> shapes;
    const la_status_t st = plan_one_step("la_schedule_launch_plan", sched, step, bufs, sendbufs, staging, ht, shapes);
    if (st != LA_OK) return st;
    const StepTable& v = ht.view[0];
    out->block = shapes[0].block;
    out->unroll = shapes[0].unroll;
    out->cache_policy = shapes[0].cache_policy;
    out->tiling = (int)v.tiling;
    out->tiles_per_segment = v.tiles_per_seg;
    out->edge_workgroups = v.edge_blocks;
    out->workgroups = (uint64_t)v.edge_blocks + (uint64_t)v.num_segments * v.tiles_per_seg;
    return LA_OK;
}

la_status_t la_schedule_launch_segments(const la_schedule_t* sched, int step, const void* const* bufs,
                                        const void* const* sendbufs, const void* staging, size_t capacity,
                                        size_t* count, uint64_t* seg_len, uint64_t* src_addr, uint64_t* dst_addr)
{
    if (!count) return fail(LA_ERR_INVALID_ARG, "la_schedule_launch_segments: count is NULL");
    HostTables ht;
    std::vector<Tuning> shapes;
    const la_status_t st = plan_one_step("la_schedule_launch_segments", sched, step, bufs, sendbufs, staging, ht, shapes);
    if (st != LA_OK) return st;
    const StepTable& v = ht.view[0];
    const unsigned char* blob = ht.blob.data(); // the views hold offsets into the blob until they are relocated
    const SegInfo* seg = reinterpret_cast<const SegInfo*>(blob + reinterpret_cast<uint64_t>(v.seg));
    const uint64_t* sp = reinterpret_cast<const uint64_t*>(blob + reinterpret_cast<uint64_t>(v.src_ptr));
    const uint64_t* dp = reinterpret_cast<const uint64_t*>(blob + reinterpret_cast<uint64_t>(v.dst_ptr));
    *count = v.num_segments;
    const size_t take = std::min<size_t>(capacity, v.num_segments);
    for (size_t g = 0; g < take; ++g) {
        if (seg_len) seg_len[g] = seg[g].len;
        if (src_addr) std::copy(sp + g * v.k, sp + (g + 1) * v.k, src_addr + g * v.k);
        if (dst_addr) std::copy(dp + g * v.m, dp + (g + 1) * v.m, dst_addr + g * v.m);
    }
    return LA_OK;
}

la_status_t la_reduce_segments(void* dst, const void* const* srcs, int k, const size_t* seg_offsets,
                               size_t num_segments, size_t seg_len, la_dtype_t dtype, la_op_t op,
                               void* hip_stream)
{
    bool nothing = false;
    la_status_t vst = check_reduce_segments_args("la_reduce_segments", dst, srcs, k, seg_offsets, num_segments, seg_len,
                                                 dtype, op, &nothing);
    if (vst != LA_OK || nothing) return vst;
    try {
        std::vector<size_t> sorted(seg_offsets, seg_offsets + num_segments);
        std::sort(sorted.begin(), sorted.end());
        for (size_t s = 1; s < num_segments; ++s)
            if (sorted[s] < sorted[s - 1] + seg_len)
                return fail(LA_ERR_INVALID_ARG, "la_reduce_segments: segments overlap");
    } catch (const std::bad_alloc&) {
        return fail(LA_ERR_OUT_OF_MEMORY, "la_reduce_segments: out of host memory");
    }
    const size_t e = dtype_size(dtype);
    const uint64_t d = reinterpret_cast<uint64_t>(dst);

    // Tables for one step with k+1 sources (dst first) and one destination.
    const size_t K = (size_t)k + 1;
    const uint64_t seg_bytes = align_up(num_segments * sizeof(SegInfo), 256);
    const uint64_t src_bytes = align_up(num_segments * K * sizeof(uint64_t), 256);
    const uint64_t dst_bytes = align_up(num_segments * sizeof(uint64_t), 256);
    const uint64_t total_bytes = seg_bytes + src_bytes + dst_bytes;
    std::lock_guard<std::mutex> lock(g_pool_mu);
    PinnedChunk* chunk = nullptr;
    la_status_t pst = acquire_pinned(total_bytes, &chunk);
    if (pst != LA_OK) return pst;
    unsigned char* blob = static_cast<unsigned char*>(chunk->host);
    SegInfo* seg = reinterpret_cast<SegInfo*>(blob);
    uint64_t* sp = reinterpret_cast<uint64_t*>(blob + seg_bytes);
    uint64_t* dp = reinterpret_cast<uint64_t*>(blob + seg_bytes + src_bytes);
    uint64_t longest = 0;
    uint64_t all_small[66];
    std::vector<uint64_t> all_big;
    uint64_t* all = all_small;
    try {
        if (K + 1 > 66) {
            all_big.resize(K + 1);
            all = all_big.data();
        }
    } catch (const std::bad_alloc&) {
        return fail(LA_ERR_OUT_OF_MEMORY, "la_reduce_segments: out of host memory");
    }
    for (size_t s = 0; s < num_segments; ++s) {
        const uint64_t byte_off = (uint64_t)seg_offsets[s] * e;
        sp[s * K] = d + byte_off;
        for (int t = 0; t < k; ++t) sp[s * K + 1 + t] = reinterpret_cast<uint64_t>(srcs[t]) + byte_off;
        dp[s] = d + byte_off;
        std::copy(sp + s * K, sp + (s + 1) * K, all);
        all[K] = dp[s];
        longest = std::max(longest, describe_segment(seg[s], seg_len, all, K + 1, e, K));
    }
    // the launch is planned, and everything that can refuse it is checked, before anything is enqueued
    StepTable t;
    t.k = (uint32_t)K;
    t.m = 1;
    t.op = (uint32_t)op;
    t.num_segments = (uint32_t)num_segments;
    const Tuning tune = resolve_tuning(current_tuning(), t.k, t.m, longest, (uint64_t)num_segments * seg_len * e, false, e,
                                       (uint64_t)(K + 1) * num_segments * seg_len * e);
    t.tiles_per_seg = plan_tiles(seg, dp, num_segments, 1, e, tune, longest, &t.tiling);
    t.edge_blocks = plan_edges(seg, num_segments, e, tune);
    la_status_t st = check_launch(t, dtype, tune);
    if (st != LA_OK) return st;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    void* dev = nullptr;
    if (hipMallocAsync(&dev, total_bytes, stream) != hipSuccess)
        return fail(LA_ERR_OUT_OF_MEMORY, "la_reduce_segments: cannot allocate %llu bytes of device tables",
                    (unsigned long long)total_bytes);
    hipError_t he = hipMemcpyAsync(dev, chunk->host, total_bytes, hipMemcpyHostToDevice, stream);
    if (he == hipSuccess) he = hipEventRecord(chunk->done, stream); // the chunk is free again after the copy
    if (he != hipSuccess) {
        (void)hipFreeAsync(dev, stream);
        return fail(LA_ERR_DEVICE, "la_reduce_segments: table upload failed: %s", hipGetErrorString(he));
    }
    chunk->in_flight = true;
    const uint64_t b = reinterpret_cast<uint64_t>(dev);
    t.seg = reinterpret_cast<const SegInfo*>(b);
    t.src_ptr = reinterpret_cast<const uint64_t*>(b + seg_bytes);
    t.dst_ptr = reinterpret_cast<const uint64_t*>(b + seg_bytes + src_bytes);
    st = launch_step(t, dtype, tune, hip_stream);
    (void)hipFreeAsync(dev, stream); // stream-ordered: freed after the kernel has run
    return st;
}

la_status_t la_tuning_set(const char* key, int value)
{
    if (!key) return fail(LA_ERR_INVALID_ARG, "la_tuning_set: key is NULL");
    const std::string k(key);
    if (k == "unroll") {
        if (value != 0 && value != 1 && value != 2 && value != 4 && value != 8)
            return fail(LA_ERR_INVALID_ARG, "la_tuning_set: unroll must be 0 (auto), 1, 2, 4 or 8");
        g_unroll.store(value);
        return LA_OK;
    }
    if (k == "cache_policy") {
        const bool one = value >= -1 && value <= 7;
        const bool three = value >= 100 && value / 100 <= 7 && (value / 10) % 10 <= 7 && value % 10 <= 7;
        if (!one && !three)
            return fail(LA_ERR_INVALID_ARG, "la_tuning_set: cache_policy must be -1 (auto), 0..7, or three digits 0..7");
        g_cache_policy.store(value);
        return LA_OK;
    }
    if (k == "graph") {
        if (value < -1 || value > 1) return fail(LA_ERR_INVALID_ARG, "la_tuning_set: graph must be -1 (auto), 0 or 1");
        g_graph.store(value);
        return LA_OK;
    }
    if (k == "merge") {
        if (value != 0 && value != 1) return fail(LA_ERR_INVALID_ARG, "la_tuning_set: merge must be 0 or 1");
        g_merge.store(value);
        return LA_OK;
    }
    if (k == "forward") {
        if (value != 0 && value != 1) return fail(LA_ERR_INVALID_ARG, "la_tuning_set: forward must be 0 or 1");
        g_forward.store(value);
        return LA_OK;
    }
    if (k == "fuse") {
        if (value < -1 || value > 1) return fail(LA_ERR_INVALID_ARG, "la_tuning_set: fuse must be -1 (auto), 0 or 1");
        g_fuse.store(value);
        return LA_OK;
    }
    if (k == "block") {
        if (value != 0 && value != 256 && value != 1024)
            return fail(LA_ERR_INVALID_ARG, "la_tuning_set: block must be 0 (auto), 256 or 1024");
        g_block.store(value);
        return LA_OK;
    }
    return fail(LA_ERR_INVALID_ARG, "la_tuning_set: unknown key '%s'", key);
}

int la_tuning_get(const char* key)
{
    if (!key) return -2;
    const std::string k(key);
    if (k == "unroll") return g_unroll.load();
    if (k == "cache_policy") return g_cache_policy.load();
    if (k == "block") return g_block.load();
    if (k == "graph") return g_graph.load();
    if (k == "merge") return g_merge.load();
    if (k == "fuse") return g_fuse.load();
    if (k == "forward") return g_forward.load();
    if (k == "fused_launches") return g_fused_launches.load();
    return -2;
}

} // extern "C"
