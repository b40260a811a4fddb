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

template <bool NT>
__device__ inline u32x4 load16(uint64_t base, uint64_t vec)
{
    const u32x4* p = reinterpret_cast<const u32x4*>(base) + vec;
    if constexpr (NT)
        return __builtin_nontemporal_load(p);
    else
        return *p;
}

template <bool NT>
__device__ inline void store16(uint64_t base, uint64_t vec, u32x4 v)
{
    u32x4* p = reinterpret_cast<u32x4*>(base) + vec;
    if constexpr (NT)
        __builtin_nontemporal_store(v, p);
    else
        *p = v;
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

template <typename T, int U, bool NTL, bool NTS, int BLOCK>
__global__ __launch_bounds__(BLOCK) void seg_reduce_kernel(StepTable tab)
{
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
    const uint64_t shift = (uint64_t)si.head * sizeof(typename T::elem); // bytes to the boundary

    if (tile == 0 && tid < si.head + tail) {
        // the few elements before the first and after the last whole vector
        const uint64_t e = tid < si.head ? tid : si.head + nvec * T::VEC + (tid - si.head);
        reduce_one<T>(sp, dp, k, m, e);
    }

    const uint64_t v0 = (uint64_t)tile * TILE + tid;
    if (v0 >= nvec) return;
    const bool full = (uint64_t)(tile + 1) * TILE <= nvec; // uniform across the workgroup

    typename T::Acc acc[U];
    {
        const uint64_t base = sp[0] + shift;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint64_t v = v0 + (uint64_t)u * BLOCK;
            u32x4 x = u32x4{0, 0, 0, 0};
            if (full || v < nvec) x = load16<NTL>(base, v);
            acc[u] = T::widen(x);
        }
    }
    uint32_t t = 1;
    // full batches: KBATCH*U independent 16-byte loads per lane are issued before the adds
    for (; t + KBATCH <= k; t += KBATCH) {
        u32x4 x[KBATCH][U];
#pragma unroll
        for (int b = 0; b < KBATCH; ++b) {
            const uint64_t base = sp[t + b] + shift;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint64_t v = v0 + (uint64_t)u * BLOCK;
                x[b][u] = u32x4{0, 0, 0, 0};
                if (full || v < nvec) x[b][u] = load16<NTL>(base, v);
            }
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
                const uint64_t base = sp[t + b] + shift;
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const uint64_t v = v0 + (uint64_t)u * BLOCK;
                    x[b][u] = u32x4{0, 0, 0, 0};
                    if (full || v < nvec) x[b][u] = load16<NTL>(base, v);
                }
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
        const uint64_t base = dp[d] + shift;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint64_t v = v0 + (uint64_t)u * BLOCK;
            if (full || v < nvec) store16<NTS>(base, v, out[u]);
        }
    }
}

template <typename T, int U, int BLOCK>
la_status_t launch_nt(const StepTable& t, int nt, dim3 grid, hipStream_t s)
{
    switch (nt & 3) {
    case 0: hipLaunchKernelGGL((seg_reduce_kernel<T, U, false, false, BLOCK>), grid, dim3(BLOCK), 0, s, t); break;
    case 1: hipLaunchKernelGGL((seg_reduce_kernel<T, U, true, false, BLOCK>), grid, dim3(BLOCK), 0, s, t); break;
    case 2: hipLaunchKernelGGL((seg_reduce_kernel<T, U, false, true, BLOCK>), grid, dim3(BLOCK), 0, s, t); break;
    default: hipLaunchKernelGGL((seg_reduce_kernel<T, U, true, true, BLOCK>), grid, dim3(BLOCK), 0, s, t); break;
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(LA_ERR_DEVICE, "kernel launch failed: %s", hipGetErrorString(e));
    return LA_OK;
}

template <typename T, int BLOCK>
la_status_t launch_unroll(const StepTable& t, const Tuning& tune, dim3 grid, hipStream_t s)
{
    switch (tune.unroll) {
    case 1: return launch_nt<T, 1, BLOCK>(t, tune.nontemporal, grid, s);
    case 2: return launch_nt<T, 2, BLOCK>(t, tune.nontemporal, grid, s);
    case 4: return launch_nt<T, 4, BLOCK>(t, tune.nontemporal, grid, s);
    case 8: return launch_nt<T, 8, BLOCK>(t, tune.nontemporal, grid, s);
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
