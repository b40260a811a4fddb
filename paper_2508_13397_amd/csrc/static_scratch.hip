// la_reduce_segments_static: la_reduce_segments for callers that cannot allocate (code under HIP
// graph capture, tight serving loops, harnesses that forbid hipMalloc).  The per-call device
// tables of la_reduce_segments -- the segment records and the resolved source and destination
// addresses that the kernel reads -- live in a file-scope device array instead of a
// stream-ordered allocation, and are written there by a small kernel that receives the call's
// pointers and offsets as kernel arguments (no pinned host chunk, no copy engine).  The reduce
// itself is the same kernel, planned by the same host code.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <mutex>

#include "la_internal.hpp"

namespace la {
namespace {

// Each GPU the library runs on holds this array until the process ends.
constexpr uint32_t SCRATCH_BYTES = 1u << 20;
static __device__ __align__(256) unsigned char scratch[SCRATCH_BYTES];

constexpr int MAX_SOURCES = 64;         // k of one call
constexpr uint32_t MAX_SEGMENTS = 8192; // host-side planning arrays
constexpr uint32_t OFFSETS_PER_FILL = 384;

// The name `scratch` is a host-side stand-in in host code; the array's device address is looked
// up once per device, with that device current, and only that address is ever handed to a kernel.
constexpr int MAX_DEVICES = 64;
std::mutex g_mu;
unsigned char* g_scratch_ptr[MAX_DEVICES] = {};

la_status_t scratch_of_current_device(unsigned char** out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES)
        return fail(LA_ERR_DEVICE, "la_reduce_segments_static: no current device (or device index beyond %d)", MAX_DEVICES - 1);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return fail(LA_ERR_DEVICE, "la_reduce_segments_static: hipGetSymbolAddress failed: %s", hipGetErrorString(e));
        g_scratch_ptr[dev] = static_cast<unsigned char*>(p);
    }
    *out = g_scratch_ptr[dev];
    return LA_OK;
}

// What one fill launch needs, by value (under the 4 KiB limit of kernel arguments).
struct FillArgs {
    uint64_t dst;              // byte address of the owned buffer
    uint64_t src[MAX_SOURCES]; // byte addresses of the k incoming buffers
    uint64_t seg_len;          // elements
    uint64_t seg_at, src_at, dst_at; // byte offsets of the three tables in the scratch array
    uint32_t k, esize;
    uint32_t congruent, align; // all operands agree modulo 16 bytes; modulo 128 (else 16)
    uint32_t first, count;     // segments [first, first + count) are written by this launch
    uint64_t off[OFFSETS_PER_FILL]; // their element offsets
};
static_assert(sizeof(FillArgs) <= 4000, "kernel arguments are limited to 4 KiB");

// One lane per segment: the segment's record, its k + 1 source addresses (the owned range first:
// dst = ((dst + src0) + src1) + ...) and its destination address.  `tables` is the device address
// of the scratch array.
__global__ __launch_bounds__(128) void fill_tables_kernel(FillArgs a, unsigned char* tables)
{
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= a.count) return;
    const uint32_t s = a.first + i;
    const uint64_t byte_off = a.off[i] * a.esize;
    const uint32_t K = a.k + 1;
    uint64_t* sp = reinterpret_cast<uint64_t*>(tables + a.src_at) + (uint64_t)s * K;
    sp[0] = a.dst + byte_off;
    for (uint32_t t = 0; t < a.k; ++t) sp[1 + t] = a.src[t] + byte_off;
    reinterpret_cast<uint64_t*>(tables + a.dst_at)[s] = a.dst + byte_off;
    SegInfo si;
    si.alias_mask = 1; // source 0 is the destination; no other source may alias it
    (void)finish_segment(si, a.seg_len, a.dst + byte_off, a.esize, a.congruent != 0, a.align);
    reinterpret_cast<SegInfo*>(tables + a.seg_at)[s] = si;
}

// host-side planning arrays (guarded by g_mu): the same records the device writes, and the
// destination addresses, as plan_tiles and plan_edges read them
SegInfo h_seg[MAX_SEGMENTS];
uint64_t h_dp[MAX_SEGMENTS];
size_t h_sorted[MAX_SEGMENTS];
FillArgs h_args;

} // namespace
} // namespace la

using namespace la;

extern "C" la_status_t la_reduce_segments_static(void* dst, const void* const* srcs, int k, const size_t* seg_offsets,
                                                 size_t num_segments, size_t seg_len, la_dtype_t dtype, la_op_t op,
                                                 void* hip_stream)
{
    const char* who = "la_reduce_segments_static";
    bool nothing = false;
    la_status_t st = check_reduce_segments_args(who, dst, srcs, k, seg_offsets, num_segments, seg_len, dtype, op, &nothing);
    if (st != LA_OK || nothing) return st;
    if (k > MAX_SOURCES) return fail(LA_ERR_INVALID_ARG, "%s: k = %d exceeds the limit of %d sources", who, k, MAX_SOURCES);
    if (num_segments > MAX_SEGMENTS)
        return fail(LA_ERR_INVALID_ARG, "%s: %zu segments exceed the limit of %u", who, num_segments, MAX_SEGMENTS);
    const size_t e = dtype_size(dtype);
    const size_t K = (size_t)k + 1;
    const uint64_t seg_bytes = align_up(num_segments * sizeof(SegInfo), 256);
    const uint64_t src_bytes = align_up(num_segments * K * sizeof(uint64_t), 256);
    const uint64_t dst_bytes = align_up(num_segments * sizeof(uint64_t), 256);
    const uint64_t total_bytes = seg_bytes + src_bytes + dst_bytes;
    if (total_bytes > SCRATCH_BYTES)
        return fail(LA_ERR_INVALID_ARG, "%s: the tables of %zu segments with %d sources take %llu bytes; the static scratch holds %u",
                    who, num_segments, k, (unsigned long long)total_bytes, SCRATCH_BYTES);

    std::lock_guard<std::mutex> lock(g_mu);
    std::copy(seg_offsets, seg_offsets + num_segments, h_sorted);
    std::sort(h_sorted, h_sorted + num_segments);
    for (size_t s = 1; s < num_segments; ++s)
        if (h_sorted[s] < h_sorted[s - 1] + seg_len) return fail(LA_ERR_INVALID_ARG, "%s: segments overlap", who);

    const uint64_t d = reinterpret_cast<uint64_t>(dst);
    bool congruent = true;
    uint32_t align = 128;
    for (int t = 0; t < k; ++t) {
        const uint64_t x = reinterpret_cast<uint64_t>(srcs[t]) ^ d; // the same offset is added to all operands
        if (x & 15u) congruent = false;
        if (x & 127u) align = 16;
    }
    uint64_t longest = 0;
    for (size_t s = 0; s < num_segments; ++s) {
        h_dp[s] = d + (uint64_t)seg_offsets[s] * e;
        h_seg[s].alias_mask = 1;
        longest = std::max(longest, finish_segment(h_seg[s], seg_len, h_dp[s], (uint32_t)e, congruent, align));
    }
    StepTable t;
    t.k = (uint32_t)K;
    t.m = 1;
    t.op = (uint32_t)op;
    t.num_segments = (uint32_t)num_segments;
    const Tuning tune = resolve_tuning(current_tuning(), t.k, t.m, longest, (uint64_t)num_segments * seg_len * e, false, e,
                                       (uint64_t)(K + 1) * num_segments * seg_len * e);
    t.tiles_per_seg = plan_tiles(h_seg, h_dp, num_segments, 1, e, tune, longest, &t.tiling);
    t.edge_blocks = plan_edges(h_seg, num_segments, e, tune);
    st = check_launch(t, dtype, tune);
    if (st != LA_OK) return st;

    unsigned char* tables = nullptr;
    st = scratch_of_current_device(&tables);
    if (st != LA_OK) return st;
    t.seg = reinterpret_cast<const SegInfo*>(tables);
    t.src_ptr = reinterpret_cast<const uint64_t*>(tables + seg_bytes);
    t.dst_ptr = reinterpret_cast<const uint64_t*>(tables + seg_bytes + src_bytes);

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    FillArgs& a = h_args;
    a.dst = d;
    for (int i = 0; i < MAX_SOURCES; ++i) a.src[i] = i < k ? reinterpret_cast<uint64_t>(srcs[i]) : 0;
    a.seg_len = seg_len;
    a.seg_at = 0;
    a.src_at = seg_bytes;
    a.dst_at = seg_bytes + src_bytes;
    a.k = (uint32_t)k;
    a.esize = (uint32_t)e;
    a.congruent = congruent ? 1u : 0u;
    a.align = align;
    for (size_t first = 0; first < num_segments; first += OFFSETS_PER_FILL) {
        a.first = (uint32_t)first;
        a.count = (uint32_t)std::min<size_t>(OFFSETS_PER_FILL, num_segments - first);
        for (uint32_t i = 0; i < OFFSETS_PER_FILL; ++i) a.off[i] = i < a.count ? (uint64_t)seg_offsets[first + i] : 0;
        hipLaunchKernelGGL(fill_tables_kernel, dim3((a.count + 127) / 128), dim3(128), 0, stream, a, tables);
        const hipError_t he = hipGetLastError();
        if (he != hipSuccess) return fail(LA_ERR_DEVICE, "%s: table launch failed: %s", who, hipGetErrorString(he));
    }
    return launch_step(t, dtype, tune, hip_stream);
}
