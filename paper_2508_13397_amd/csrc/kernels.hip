// gfx950 kernels of the segmented k-way reduce / multi-destination copy.
//
// One launch executes one step: S segments, each "sum k source ranges element by element, in
// table order, and store the result to m destination ranges".  k == 1 is a copy or broadcast;
// m > 1 writes the same result to several rank buffers.  This is the local reduction that
// follows every received message in Algorithms 1 and 2, generalised from two operands to k,
// with the message transfer itself folded in as a read of the peer's buffer.
//
// The work is HBM-bound (at most k-1 adds per (k+m) elements moved), so the kernel is built
// around 16-byte coalesced accesses with many independent loads in flight per lane; no LDS and
// no matrix cores.  A workgroup of BLOCK lanes owns a tile of UNROLL*BLOCK vectors of one segment;
// consecutive workgroups own consecutive tiles, so the eight XCDs (which receive workgroups
// round-robin) stream disjoint, adjacent 4-128 KiB pieces of the same operand rows at once.  The
// elements outside a segment's whole vectors go to a few edge workgroups at the front of the grid.
#include <hip/hip_runtime.h>

#include "kernel_common.hpp"
#include "la_internal.hpp"

namespace la {

namespace {

template <typename T, int U, int POLICY, int BLOCK, int MODE>
__global__ __launch_bounds__(BLOCK) void seg_reduce_kernel(StepTable tab)
{
    using P = Policy<POLICY>;
    const uint32_t k = tab.k, m = tab.m, op = MODE == MODE_SUM ? (uint32_t)LA_SUM : tab.op;
    const uint32_t group = MODE == MODE_GROUPED ? tab.group : k;
    const uint32_t tid = threadIdx.x;

    if (blockIdx.x < tab.edge_blocks) {
        // Edge workgroup: the elements outside the whole vectors of BLOCK / EDGE_LANES segments,
        // one per lane.  Each is a chain of memory latencies (k loads, a few at a time); in
        // workgroups of their own these chains run beside the tiles instead of prolonging every
        // segment's first tile (128 ranks, 1.4 and 2.8 MiB each: 9 and 6 % of the all-reduce).
        static_assert(128 / sizeof(typename T::elem) - 1 + T::VEC - 1 <= EDGE_LANES, "head + tail lanes");
        const uint32_t seg = __builtin_amdgcn_readfirstlane(blockIdx.x * (BLOCK / EDGE_LANES) + tid / EDGE_LANES);
        if (seg >= tab.num_segments) return;
        const uint32_t l = tid % EDGE_LANES;
        const table_seg sg = as_table(tab.seg) + seg;
        const uint64_t len = sg->len;
        const uint32_t head = sg->head;
        const table_u64 sp = as_table(tab.src_ptr) + (uint64_t)seg * k;
        const table_u64 dp = as_table(tab.dst_ptr) + (uint64_t)seg * m;
        // without a vector phase common to all operands the vectors count from the segment's start (head 0)
        const uint64_t whole = (len - head) / T::VEC;
        const uint32_t tail = (uint32_t)((len - head) % T::VEC);
        if (l < head + tail) {
            const uint64_t e = l < head ? l : head + whole * T::VEC + (l - head);
            reduce_one<T>(sp, dp, k, m, group, e, op);
        }
        return;
    }
    const uint32_t tile_block = blockIdx.x - tab.edge_blocks;
    const uint32_t seg = tile_block / tab.tiles_per_seg;
    const uint32_t tile = tile_block - seg * tab.tiles_per_seg;
    const table_seg sg = as_table(tab.seg) + seg;
    SegInfo si;
    si.len = sg->len;
    si.head = sg->head;
    si.vec_ok = sg->vec_ok;
    si.alias_mask = sg->alias_mask;
    const table_u64 sp = as_table(tab.src_ptr) + (uint64_t)seg * k;
    const table_u64 dp = as_table(tab.dst_ptr) + (uint64_t)seg * m;
    const uint64_t dst0 = dp[0]; // fetched with the segment record: the tiling and the lane rotation need it
    constexpr uint64_t TILE = (uint64_t)BLOCK * U; // vectors per tile

    if (!si.vec_ok) {
        // operands disagree on their 16-byte phase: 16-byte vectors counted from the start of the
        // segment, every access unaligned (the last len % VEC elements: edge workgroups)
        const uint64_t whole = si.len / T::VEC;
        const uint64_t v_lo = (uint64_t)tile * TILE;
        uint64_t v_hi = v_lo + TILE;
        if (v_hi > whole) v_hi = whole;
        for (uint64_t v = v_lo + tid; v < v_hi; v += BLOCK) reduce_vector_unaligned<T>(sp, dp, k, m, group, v * 16u, op);
        return;
    }

    const uint64_t body = si.len - si.head;    // elements from the first 16-byte boundary on
    const uint64_t nvec = body / T::VEC;       // whole vectors (the elements around them: edge workgroups)

    // Tile t covers the vectors [t*per - lead, (t+1)*per - lead) of the body.  Plain: per = TILE,
    // lead = 0.  Aligned: lead is the distance of the body's start from the previous multiple of
    // the tile size in destination 0's address, so every tile but the first starts on such a
    // multiple.  Equal: the tiles that TILE would need, all of one size (whole 128-byte lines).
    uint64_t per = TILE, lead = 0;
    if (tab.tiling == TILING_ALIGNED) {
        lead = ((dst0 + (uint64_t)si.head * sizeof(typename T::elem)) & (TILE * 16u - 1u)) / 16u;
    } else if (tab.tiling == TILING_EQUAL && nvec > TILE) {
        const uint64_t count = (nvec + TILE - 1) / TILE;
        per = ((nvec + count - 1) / count + 7u) & ~uint64_t(7);
    }
    const uint64_t lo = (uint64_t)tile * per;
    if (nvec == 0 || lo >= lead + nvec) return; // uniform: nothing left for this workgroup
    const uint64_t tile_v0 = lo > lead ? lo - lead : 0;
    const uint64_t tile_v1 = lo + per < lead + nvec ? lo + per - lead : nvec;
    const uint32_t tile_bytes = (uint32_t)(tile_v1 - tile_v0) * 16u;
    const uint64_t tile_off = (uint64_t)si.head * sizeof(typename T::elem) + tile_v0 * 16u;
    const uint64_t in_place = si.alias_mask;

    // Lane j of the workgroup takes the vector of the tile whose address (in destination 0) is
    // j * 16 modulo the tile size: whatever the tile's start, a wave's 64 vectors are 1 KiB on a
    // 1 KiB boundary, the waves of a workgroup follow each other as in a tile that starts on a
    // multiple of the tile size, and the vectors before that start wrap to the tile's end (any
    // rotation of the lanes covers a tile once; offsets beyond its bytes are dropped by the range
    // check).  1024 ranks x 4 MiB viewed at +128 B ... +512 B: the broadcast step lost 5 to 8 %.
    const uint32_t phase = (uint32_t)((dst0 + tile_off) & (TILE * 16u - 1u));
    uint32_t off[U];
#pragma unroll
    for (int u = 0; u < U; ++u) off[u] = ((tid + (uint32_t)u * BLOCK) * 16u - phase) & (uint32_t)(TILE * 16u - 1u);

    u32x4 out[U];
    if (k == 1) {
        // copy / broadcast: the bits are moved as they are (no widening and narrowing, which would
        // quiet a signalling NaN of the 16-bit types)
        const __amdgpu_buffer_rsrc_t r = tile_rsrc(sp[0], tile_off, tile_bytes);
#pragma unroll
        for (int u = 0; u < U; ++u) out[u] = load_src<P>(r, off[u], (in_place & 1u) != 0);
    } else if constexpr (MODE != MODE_GROUPED) {
        typename T::Acc acc[U];
        reduce_run<T, U, P>(acc, sp, 0, k, in_place, tile_off, tile_bytes, off, op);
#pragma unroll
        for (int u = 0; u < U; ++u) out[u] = T::narrow(acc[u]);
    } else {
        // first level: runs of `group` sources, each rounded as a stored result would be;
        // second level: the run results in order
        typename T::Acc acc[U];
        for (uint32_t t0 = 0; t0 < k; t0 += group) {
            const uint32_t t1 = t0 + group < k ? t0 + group : k;
            typename T::Acc run[U];
            reduce_run<T, U, P>(run, sp, t0, t1, in_place, tile_off, tile_bytes, off, op);
            if (t0 == 0) {
#pragma unroll
                for (int u = 0; u < U; ++u) acc[u] = T::widen(T::narrow(run[u]));
            } else {
#pragma unroll
                for (int u = 0; u < U; ++u) T::add(acc[u], T::narrow(run[u]), op);
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) out[u] = T::narrow(acc[u]);
    }
    for (uint32_t d = 0; d < m; ++d) {
        const __amdgpu_buffer_rsrc_t r = tile_rsrc(dp[d], tile_off, tile_bytes);
#pragma unroll
        for (int u = 0; u < U; ++u) store16<P::ST>(r, off[u], out[u]);
    }
}

template <typename T, int U, int POLICY, int BLOCK>
void launch_op(const StepTable& t, dim3 grid, hipStream_t s)
{
    if (t.group > 0 && t.group < t.k)
        hipLaunchKernelGGL((seg_reduce_kernel<T, U, POLICY, BLOCK, MODE_GROUPED>), grid, dim3(BLOCK), 0, s, t);
    else if (t.op == (uint32_t)LA_SUM)
        hipLaunchKernelGGL((seg_reduce_kernel<T, U, POLICY, BLOCK, MODE_SUM>), grid, dim3(BLOCK), 0, s, t);
    else
        hipLaunchKernelGGL((seg_reduce_kernel<T, U, POLICY, BLOCK, MODE_ANY_OP>), grid, dim3(BLOCK), 0, s, t);
}

template <typename T, int U, int BLOCK>
la_status_t launch_policy(const StepTable& t, int policy, dim3 grid, hipStream_t s)
{
    switch (policy) {
    case 0: launch_op<T, U, 0, BLOCK>(t, grid, s); break;
    case 1: launch_op<T, U, 1, BLOCK>(t, grid, s); break;
    case 2: launch_op<T, U, 2, BLOCK>(t, grid, s); break;
    case 3: launch_op<T, U, 3, BLOCK>(t, grid, s); break;
    case 4: launch_op<T, U, 4, BLOCK>(t, grid, s); break;
    case 5: launch_op<T, U, 5, BLOCK>(t, grid, s); break;
    case 6: launch_op<T, U, 6, BLOCK>(t, grid, s); break;
    case 7: launch_op<T, U, 7, BLOCK>(t, grid, s); break;
    default: return fail(LA_ERR_INVALID_ARG, "unsupported cache policy %d", policy);
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(LA_ERR_DEVICE, "kernel launch failed: %s", hipGetErrorString(e));
    return LA_OK;
}

// This file is compiled once per element type and launch-shape family
// (-DLA_KERNEL_DTYPE=<la_dtype_t value> -DLA_KERNEL_SHAPE=<0..2>), so that the instances build in
// parallel; launch_step in dispatch.cpp picks the family.  Families: 0 = workgroups of 256 lanes
// (1, 2, 4 vectors per lane), 1 = 1024 lanes with 1 or 2 vectors, 2 = 1024 lanes with 4 or 8.
#if !defined(LA_KERNEL_DTYPE) || !defined(LA_KERNEL_SHAPE)
#error "compile kernels.hip with -DLA_KERNEL_DTYPE=0..4 -DLA_KERNEL_SHAPE=0..2"
#endif

la_status_t launch_family(const StepTable& t, const Tuning& tune, dim3 grid, hipStream_t s)
{
    using T = ElemTraits;
#if LA_KERNEL_SHAPE == 0
    if (tune.block == 256) {
        switch (tune.unroll) {
        case 1: return launch_policy<T, 1, 256>(t, tune.cache_policy, grid, s);
        case 2: return launch_policy<T, 2, 256>(t, tune.cache_policy, grid, s);
        case 4: return launch_policy<T, 4, 256>(t, tune.cache_policy, grid, s);
        }
    }
#elif LA_KERNEL_SHAPE == 1
    if (tune.block == 1024) {
        switch (tune.unroll) {
        case 1: return launch_policy<T, 1, 1024>(t, tune.cache_policy, grid, s);
        case 2: return launch_policy<T, 2, 1024>(t, tune.cache_policy, grid, s);
        }
    }
#elif LA_KERNEL_SHAPE == 2
    if (tune.block == 1024) {
        switch (tune.unroll) {
        case 4: return launch_policy<T, 4, 1024>(t, tune.cache_policy, grid, s);
        case 8: return launch_policy<T, 8, 1024>(t, tune.cache_policy, grid, s); // 128 KiB tiles
        }
    }
#else
#error "LA_KERNEL_SHAPE must be 0..2"
#endif
    return fail(LA_ERR_INVALID_ARG, "internal: %d lanes x %d vectors is not in kernel family %d", tune.block,
                tune.unroll, (int)LA_KERNEL_SHAPE);
}

} // namespace

#define LA_CONCAT3(a, b, c) a##b##_##c
#define LA_FAMILY_NAME(d, f) LA_CONCAT3(launch_family_, d, f)
la_status_t LA_FAMILY_NAME(LA_KERNEL_DTYPE, LA_KERNEL_SHAPE)(const StepTable& t, const Tuning& tune, uint32_t blocks,
                                                             void* stream)
{
    return launch_family(t, tune, dim3(blocks), static_cast<hipStream_t>(stream));
}

} // namespace la
