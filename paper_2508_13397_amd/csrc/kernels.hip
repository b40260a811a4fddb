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
// round-robin) stream disjoint, adjacent 4-16 KiB pieces of the same operand rows at once.
#include <hip/hip_runtime.h>

#include "la_internal.hpp"

namespace la {

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int KBATCH = 4; // operands whose loads are issued together

// ---- element types ---------------------------------------------------------------------------

struct I32 {
    using elem = uint32_t;
    static constexpr int VEC = 4; // elements per 16 bytes
    struct Acc {
        uint32_t v[4];
    };
    __device__ static Acc widen(u32x4 x) { return Acc{{x.x, x.y, x.z, x.w}}; }
    __device__ static void add(Acc& a, u32x4 x)
    {
        a.v[0] += x.x; // wraps (two's complement)
        a.v[1] += x.y;
        a.v[2] += x.z;
        a.v[3] += x.w;
    }
    __device__ static u32x4 narrow(const Acc& a) { return u32x4{a.v[0], a.v[1], a.v[2], a.v[3]}; }
    using sacc = uint32_t;
    __device__ static sacc swiden(elem x) { return x; }
    __device__ static sacc sadd(sacc a, elem x) { return a + x; }
    __device__ static elem snarrow(sacc a) { return a; }
};

struct F32 {
    using elem = float;
    static constexpr int VEC = 4;
    struct Acc {
        float v[4];
    };
    __device__ static Acc widen(u32x4 x)
    {
        return Acc{{__uint_as_float(x.x), __uint_as_float(x.y), __uint_as_float(x.z), __uint_as_float(x.w)}};
    }
    __device__ static void add(Acc& a, u32x4 x)
    {
        a.v[0] = a.v[0] + __uint_as_float(x.x);
        a.v[1] = a.v[1] + __uint_as_float(x.y);
        a.v[2] = a.v[2] + __uint_as_float(x.z);
        a.v[3] = a.v[3] + __uint_as_float(x.w);
    }
    __device__ static u32x4 narrow(const Acc& a)
    {
        return u32x4{__float_as_uint(a.v[0]), __float_as_uint(a.v[1]), __float_as_uint(a.v[2]),
                     __float_as_uint(a.v[3])};
    }
    using sacc = float;
    __device__ static sacc swiden(elem x) { return x; }
    __device__ static sacc sadd(sacc a, elem x) { return a + x; }
    __device__ static elem snarrow(sacc a) { return a; }
};

// bf16 is the upper half of a binary32.  Operands are widened exactly, summed in fp32 and
// rounded to nearest, ties to even, once when the step stores its result.
__device__ inline uint32_t f32_to_bf16_bits(float f)
{
    const uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x0040u; // NaN: keep it quiet
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

struct BF16 {
    using elem = uint16_t;
    static constexpr int VEC = 8;
    struct Acc {
        float v[8];
    };
    __device__ static float lo(uint32_t w) { return __uint_as_float(w << 16); }
    __device__ static float hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
    __device__ static Acc widen(u32x4 x)
    {
        return Acc{{lo(x.x), hi(x.x), lo(x.y), hi(x.y), lo(x.z), hi(x.z), lo(x.w), hi(x.w)}};
    }
    __device__ static void add(Acc& a, u32x4 x)
    {
        a.v[0] = a.v[0] + lo(x.x);
        a.v[1] = a.v[1] + hi(x.x);
        a.v[2] = a.v[2] + lo(x.y);
        a.v[3] = a.v[3] + hi(x.y);
        a.v[4] = a.v[4] + lo(x.z);
        a.v[5] = a.v[5] + hi(x.z);
        a.v[6] = a.v[6] + lo(x.w);
        a.v[7] = a.v[7] + hi(x.w);
    }
    __device__ static uint32_t pack(float l, float h)
    {
        return f32_to_bf16_bits(l) | (f32_to_bf16_bits(h) << 16);
    }
    __device__ static u32x4 narrow(const Acc& a)
    {
        return u32x4{pack(a.v[0], a.v[1]), pack(a.v[2], a.v[3]), pack(a.v[4], a.v[5]), pack(a.v[6], a.v[7])};
    }
    using sacc = float;
    __device__ static sacc swiden(elem x) { return __uint_as_float((uint32_t)x << 16); }
    __device__ static sacc sadd(sacc a, elem x) { return a + __uint_as_float((uint32_t)x << 16); }
    __device__ static elem snarrow(sacc a) { return (elem)f32_to_bf16_bits(a); }
};

// ---- memory access -----------------------------------------------------------------------------
//
// 16-byte accesses go through raw buffer instructions: the descriptor of an operand is rebased
// to the workgroup's tile and sized to the bytes that remain in the segment, so the hardware
// range check drops what lies beyond a ragged tail (loads return 0, stores are discarded) and the
// lanes need no bounds test.  The aux operand carries the cache policy bits of the instruction.

constexpr int AUX_PLAIN = 0;
constexpr int AUX_NT = 2;   // non-temporal: the line is not kept
constexpr int AUX_SC1 = 16; // scope bit 1 (write-through towards memory at agent scope)

// Cache policy of a launch: {loads of pure sources, loads of sources that the segment also
// overwrites, stores}.
template <int POLICY>
struct Policy;
template <> struct Policy<0> { static constexpr int LD = AUX_PLAIN, LDA = AUX_PLAIN, ST = AUX_PLAIN; };
template <> struct Policy<1> { static constexpr int LD = AUX_NT, LDA = AUX_PLAIN, ST = AUX_PLAIN; };
template <> struct Policy<2> { static constexpr int LD = AUX_NT, LDA = AUX_PLAIN, ST = AUX_SC1; };
template <> struct Policy<3> { static constexpr int LD = AUX_NT, LDA = AUX_NT, ST = AUX_NT; };
template <> struct Policy<4> { static constexpr int LD = AUX_PLAIN, LDA = AUX_PLAIN, ST = AUX_NT; };
template <> struct Policy<5> { static constexpr int LD = AUX_NT, LDA = AUX_NT, ST = AUX_PLAIN; };
template <> struct Policy<6> { static constexpr int LD = AUX_NT, LDA = AUX_NT, ST = AUX_SC1; };
template <> struct Policy<7> { static constexpr int LD = AUX_PLAIN, LDA = AUX_PLAIN, ST = AUX_SC1; };

__device__ inline __amdgpu_buffer_rsrc_t tile_rsrc(uint64_t base, uint64_t tile_off, uint32_t tile_bytes)
{
    // raw buffer (stride 0), 32-bit data format word as used for untyped accesses on gfx9
    return __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<void*>(base + tile_off), 0, (int)tile_bytes, 0x00020000);
}

template <int AUX>
__device__ inline u32x4 load16(__amdgpu_buffer_rsrc_t r, uint32_t byte_off)
{
    return __builtin_amdgcn_raw_buffer_load_b128(r, byte_off, 0, AUX);
}

template <int AUX>
__device__ inline void store16(__amdgpu_buffer_rsrc_t r, uint32_t byte_off, u32x4 v)
{
    __builtin_amdgcn_raw_buffer_store_b128(v, r, byte_off, 0, AUX);
}

// source t of a segment: plain-source policy unless the segment also writes that range
template <typename P>
__device__ inline u32x4 load_src(__amdgpu_buffer_rsrc_t r, uint32_t byte_off, bool in_place)
{
    if constexpr (P::LD == P::LDA) {
        return load16<P::LD>(r, byte_off);
    } else {
        if (in_place) return load16<P::LDA>(r, byte_off); // uniform across the workgroup
        return load16<P::LD>(r, byte_off);
    }
}

// One element of one segment, all k operands in order: the slow lanes (segment heads and
// tails that do not fill a 16-byte vector, and segments whose operands are not congruent
// modulo 16 bytes).
template <typename T>
__device__ inline void reduce_one(const uint64_t* sp, const uint64_t* dp, uint32_t k, uint32_t m, uint64_t e)
{
    using elem = typename T::elem;
    typename T::sacc a = T::swiden(reinterpret_cast<const elem*>(sp[0])[e]);
    for (uint32_t t = 1; t < k; ++t) a = T::sadd(a, reinterpret_cast<const elem*>(sp[t])[e]);
    const elem r = T::snarrow(a);
    for (uint32_t d = 0; d < m; ++d) reinterpret_cast<elem*>(dp[d])[e] = r;
}

// ---- the kernel -------------------------------------------------------------------------------

template <typename T, int U, int POLICY, int BLOCK>
__global__ __launch_bounds__(BLOCK) void seg_reduce_kernel(StepTable tab)
{
    using P = Policy<POLICY>;
    const uint32_t seg = blockIdx.x / tab.tiles_per_seg;
    const uint32_t tile = blockIdx.x - seg * tab.tiles_per_seg;
    const uint32_t k = tab.k, m = tab.m;
    const SegInfo si = tab.seg[seg];
    const uint64_t* sp = tab.src_ptr + (uint64_t)seg * k;
    const uint64_t* dp = tab.dst_ptr + (uint64_t)seg * m;
    const uint32_t tid = threadIdx.x;
    constexpr uint64_t TILE = (uint64_t)BLOCK * U; // vectors per tile

    if (!si.vec_ok) {
        // operands disagree on their 16-byte phase: element-wise, still coalesced
        const uint64_t lo = (uint64_t)tile * TILE * T::VEC;
        uint64_t hi = lo + TILE * T::VEC;
        if (hi > si.len) hi = si.len;
        for (uint64_t e = lo + tid; e < hi; e += BLOCK) reduce_one<T>(sp, dp, k, m, e);
        return;
    }

    const uint64_t body = si.len - si.head;    // elements from the first 16-byte boundary on
    const uint64_t nvec = body / T::VEC;       // whole vectors
    const uint32_t tail = (uint32_t)(body % T::VEC);

    if (tile == 0 && tid < si.head + tail) {
        // the few elements before the first and after the last whole vector
        const uint64_t e = tid < si.head ? tid : si.head + nvec * T::VEC + (tid - si.head);
        reduce_one<T>(sp, dp, k, m, e);
    }

    const uint64_t tile_v0 = (uint64_t)tile * TILE;
    if (tile_v0 >= nvec) return; // uniform: nothing left for this workgroup
    const uint64_t left = nvec - tile_v0;
    const uint32_t tile_bytes = (uint32_t)(left < TILE ? left : TILE) * 16u;
    const uint64_t tile_off = (uint64_t)si.head * sizeof(typename T::elem) + tile_v0 * 16u;
    const uint64_t in_place = si.alias_mask;

    uint32_t off[U];
#pragma unroll
    for (int u = 0; u < U; ++u) off[u] = (tid + (uint32_t)u * BLOCK) * 16u;

    typename T::Acc acc[U];
    {
        const __amdgpu_buffer_rsrc_t r = tile_rsrc(sp[0], tile_off, tile_bytes);
        const bool ip = in_place & 1u;
#pragma unroll
        for (int u = 0; u < U; ++u) acc[u] = T::widen(load_src<P>(r, off[u], ip));
    }
    uint32_t t = 1;
    // full batches: KBATCH*U independent 16-byte loads per lane are issued before the adds
    for (; t + KBATCH <= k; t += KBATCH) {
        u32x4 x[KBATCH][U];
#pragma unroll
        for (int b = 0; b < KBATCH; ++b) {
            const __amdgpu_buffer_rsrc_t r = tile_rsrc(sp[t + b], tile_off, tile_bytes);
            const bool ip = (in_place >> ((t + b) & 63u)) & 1u;
#pragma unroll
            for (int u = 0; u < U; ++u) x[b][u] = load_src<P>(r, off[u], ip);
        }
#pragma unroll
        for (int b = 0; b < KBATCH; ++b)
#pragma unroll
            for (int u = 0; u < U; ++u) T::add(acc[u], x[b][u]);
    }
    // remaining 0..KBATCH-1 operands
    if (t < k) {
        const uint32_t rem = k - t;
        u32x4 x[KBATCH - 1][U];
#pragma unroll
        for (int b = 0; b < KBATCH - 1; ++b) {
            if ((uint32_t)b < rem) {
                const __amdgpu_buffer_rsrc_t r = tile_rsrc(sp[t + b], tile_off, tile_bytes);
                const bool ip = (in_place >> ((t + b) & 63u)) & 1u;
#pragma unroll
                for (int u = 0; u < U; ++u) x[b][u] = load_src<P>(r, off[u], ip);
            }
        }
#pragma unroll
        for (int b = 0; b < KBATCH - 1; ++b) {
            if ((uint32_t)b < rem) {
#pragma unroll
                for (int u = 0; u < U; ++u) T::add(acc[u], x[b][u]);
            }
        }
    }

    u32x4 out[U];
#pragma unroll
    for (int u = 0; u < U; ++u) out[u] = T::narrow(acc[u]);
    for (uint32_t d = 0; d < m; ++d) {
        const __amdgpu_buffer_rsrc_t r = tile_rsrc(dp[d], tile_off, tile_bytes);
#pragma unroll
        for (int u = 0; u < U; ++u) store16<P::ST>(r, off[u], out[u]);
    }
}

template <typename T, int U, int BLOCK>
la_status_t launch_policy(const StepTable& t, int policy, dim3 grid, hipStream_t s)
{
    switch (policy) {
    case 0: hipLaunchKernelGGL((seg_reduce_kernel<T, U, 0, BLOCK>), grid, dim3(BLOCK), 0, s, t); break;
    case 1: hipLaunchKernelGGL((seg_reduce_kernel<T, U, 1, BLOCK>), grid, dim3(BLOCK), 0, s, t); break;
    case 2: hipLaunchKernelGGL((seg_reduce_kernel<T, U, 2, BLOCK>), grid, dim3(BLOCK), 0, s, t); break;
    case 3: hipLaunchKernelGGL((seg_reduce_kernel<T, U, 3, BLOCK>), grid, dim3(BLOCK), 0, s, t); break;
    case 4: hipLaunchKernelGGL((seg_reduce_kernel<T, U, 4, BLOCK>), grid, dim3(BLOCK), 0, s, t); break;
    case 5: hipLaunchKernelGGL((seg_reduce_kernel<T, U, 5, BLOCK>), grid, dim3(BLOCK), 0, s, t); break;
    case 6: hipLaunchKernelGGL((seg_reduce_kernel<T, U, 6, BLOCK>), grid, dim3(BLOCK), 0, s, t); break;
    case 7: hipLaunchKernelGGL((seg_reduce_kernel<T, U, 7, BLOCK>), grid, dim3(BLOCK), 0, s, t); break;
    default: return fail(LA_ERR_INVALID_ARG, "unsupported cache policy %d", policy);
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(LA_ERR_DEVICE, "kernel launch failed: %s", hipGetErrorString(e));
    return LA_OK;
}

template <typename T, int BLOCK>
la_status_t launch_unroll(const StepTable& t, const Tuning& tune, dim3 grid, hipStream_t s)
{
    switch (tune.unroll) {
    case 1: return launch_policy<T, 1, BLOCK>(t, tune.cache_policy, grid, s);
    case 2: return launch_policy<T, 2, BLOCK>(t, tune.cache_policy, grid, s);
    case 4: return launch_policy<T, 4, BLOCK>(t, tune.cache_policy, grid, s);
    case 8: return launch_policy<T, 8, BLOCK>(t, tune.cache_policy, grid, s);
    }
    return fail(LA_ERR_INVALID_ARG, "unsupported unroll %d", tune.unroll);
}

template <typename T>
la_status_t launch_block(const StepTable& t, const Tuning& tune, dim3 grid, hipStream_t s)
{
    switch (tune.block) {
    case 256: return launch_unroll<T, 256>(t, tune, grid, s);
    case 512: return launch_unroll<T, 512>(t, tune, grid, s);
    case 1024: return launch_unroll<T, 1024>(t, tune, grid, s);
    }
    return fail(LA_ERR_INVALID_ARG, "unsupported block size %d", tune.block);
}

} // namespace

uint32_t tiles_for(uint64_t max_units, const Tuning& tune)
{
    const uint64_t tile = (uint64_t)tune.block * (uint64_t)tune.unroll;
    const uint64_t tiles = (max_units + tile - 1) / tile;
    return (uint32_t)(tiles ? tiles : 1);
}

// The caller guarantees: tables are device-resident and hold num_segments * k (resp. m)
// pointers; every pointer range [ptr, ptr + len*esize) is valid device memory;
// tiles_per_seg == tiles_for(longest segment in vectors, tune).
la_status_t launch_step(const StepTable& t, la_dtype_t dtype, const Tuning& tune, void* hip_stream)
{
    if (t.num_segments == 0) return LA_OK;
    if (t.k < 1 || t.m < 1) return fail(LA_ERR_INVALID_ARG, "internal: step with k=%u m=%u", t.k, t.m);
    const uint64_t blocks = (uint64_t)t.num_segments * t.tiles_per_seg;
    if (blocks > 0x7fffffffull) return fail(LA_ERR_INVALID_ARG, "step needs %llu workgroups", (unsigned long long)blocks);
    const dim3 grid((uint32_t)blocks);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    switch (dtype) {
    case LA_I32: return launch_block<I32>(t, tune, grid, s);
    case LA_F32: return launch_block<F32>(t, tune, grid, s);
    case LA_BF16: return launch_block<BF16>(t, tune, grid, s);
    }
    return fail(LA_ERR_UNSUPPORTED, "unknown dtype %d", (int)dtype);
}

} // namespace la
