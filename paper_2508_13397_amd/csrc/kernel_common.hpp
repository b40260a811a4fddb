// Device code shared by the kernels of liblaneallreduce: element types, binary operations, 16-byte
// buffer accesses with a cache policy per access class, the constant-address-space view of the step
// tables, and the k-way reduce of one tile (reduce_run) and of one element (reduce_one).
// Included by the .hip sources only; everything lives in an anonymous namespace of its includer.
#pragma once

#include <hip/hip_runtime.h>

#include "la_internal.hpp"

namespace la {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// operands whose loads are issued together: about 8 independent 16-byte loads per lane
constexpr int batch_for(int unroll) { return unroll >= 8 ? 1 : unroll >= 4 ? 2 : 4; }

// ---- binary operations -----------------------------------------------------------------------
// The paper reduces with MPI_SUM; product, maximum and minimum run on the same schedules.  The
// operation is a launch argument (uniform across the grid) in the instances that serve them; the
// sum has instances of its own with the operation compiled in (the run-time choice cost the
// 16-bit types 9 % on the widest reduce).

// Maximum / minimum of two floating-point numbers: a NaN loses against a number, two NaNs give
// the running value, and +0 is larger than -0.  a is the running value, b the next operand.
template <typename F>
__device__ inline bool sign_of(F x)
{
    if constexpr (sizeof(F) == 4)
        return (__float_as_uint((float)x) >> 31) != 0;
    else
        return (__double_as_longlong((double)x) < 0);
}

template <typename F>
__device__ inline F fmax_ordered(F a, F b)
{
    if (b != b) return a;
    if (a != a) return b;
    if (a < b) return b;
    if (a == b && a == F(0)) return sign_of(a) ? b : a;
    return a;
}

template <typename F>
__device__ inline F fmin_ordered(F a, F b)
{
    if (b != b) return a;
    if (a != a) return b;
    if (b < a) return b;
    if (a == b && a == F(0)) return sign_of(a) ? a : b;
    return a;
}

template <typename F>
__device__ inline F combine_fp(uint32_t op, F a, F b)
{
    switch (op) {
    case LA_SUM: return a + b;
    case LA_PROD: return a * b;
    case LA_MAX: return fmax_ordered(a, b);
    default: return fmin_ordered(a, b);
    }
}

// int32: sum and product wrap (two's complement), maximum and minimum compare as signed
__device__ inline uint32_t combine_u32(uint32_t op, uint32_t a, uint32_t b)
{
    switch (op) {
    case LA_SUM: return a + b;
    case LA_PROD: return a * b;
    case LA_MAX: return (int32_t)b > (int32_t)a ? b : a;
    default: return (int32_t)b < (int32_t)a ? b : a;
    }
}

// ---- element types ---------------------------------------------------------------------------
// Each type says how a 16-byte vector is widened into accumulators, combined with the next
// operand's vector, and narrowed for the store; and the same for a single element (heads, tails
// and operands that are not congruent modulo 16 bytes).

struct I32 {
    using elem = uint32_t;
    static constexpr int VEC = 4; // elements per 16 bytes
    struct Acc {
        uint32_t v[4];
    };
    __device__ static Acc widen(u32x4 x) { return Acc{{x.x, x.y, x.z, x.w}}; }
    __device__ static void add(Acc& a, u32x4 x, uint32_t op)
    {
        a.v[0] = combine_u32(op, a.v[0], x.x);
        a.v[1] = combine_u32(op, a.v[1], x.y);
        a.v[2] = combine_u32(op, a.v[2], x.z);
        a.v[3] = combine_u32(op, a.v[3], x.w);
    }
    __device__ static u32x4 narrow(const Acc& a) { return u32x4{a.v[0], a.v[1], a.v[2], a.v[3]}; }
    using sacc = uint32_t;
    __device__ static sacc swiden(elem x) { return x; }
    __device__ static sacc sadd(sacc a, elem x, uint32_t op) { return combine_u32(op, a, x); }
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
    __device__ static void add(Acc& a, u32x4 x, uint32_t op)
    {
        a.v[0] = combine_fp(op, a.v[0], __uint_as_float(x.x));
        a.v[1] = combine_fp(op, a.v[1], __uint_as_float(x.y));
        a.v[2] = combine_fp(op, a.v[2], __uint_as_float(x.z));
        a.v[3] = combine_fp(op, a.v[3], __uint_as_float(x.w));
    }
    __device__ static u32x4 narrow(const Acc& a)
    {
        return u32x4{__float_as_uint(a.v[0]), __float_as_uint(a.v[1]), __float_as_uint(a.v[2]),
                     __float_as_uint(a.v[3])};
    }
    using sacc = float;
    __device__ static sacc swiden(elem x) { return x; }
    __device__ static sacc sadd(sacc a, elem x, uint32_t op) { return combine_fp(op, a, x); }
    __device__ static elem snarrow(sacc a) { return a; }
};

struct F64 {
    using elem = double;
    static constexpr int VEC = 2;
    struct Acc {
        double v[2];
    };
    __device__ static double join(uint32_t lo, uint32_t hi)
    {
        return __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));
    }
    __device__ static Acc widen(u32x4 x) { return Acc{{join(x.x, x.y), join(x.z, x.w)}}; }
    __device__ static void add(Acc& a, u32x4 x, uint32_t op)
    {
        a.v[0] = combine_fp(op, a.v[0], join(x.x, x.y));
        a.v[1] = combine_fp(op, a.v[1], join(x.z, x.w));
    }
    __device__ static u32x4 narrow(const Acc& a)
    {
        const uint64_t p = (uint64_t)__double_as_longlong(a.v[0]), q = (uint64_t)__double_as_longlong(a.v[1]);
        return u32x4{(uint32_t)p, (uint32_t)(p >> 32), (uint32_t)q, (uint32_t)(q >> 32)};
    }
    using sacc = double;
    __device__ static sacc swiden(elem x) { return x; }
    __device__ static sacc sadd(sacc a, elem x, uint32_t op) { return combine_fp(op, a, x); }
    __device__ static elem snarrow(sacc a) { return a; }
};

// 16-bit floating types: operands are widened exactly to fp32, combined in fp32 and rounded to
// nearest, ties to even, once when the step stores its result.
template <typename H>
struct Half16 {
    using elem = uint16_t;
    static constexpr int VEC = 8;
    struct Acc {
        float v[8];
    };
    __device__ static float lo(uint32_t w) { return H::widen((uint16_t)(w & 0xffffu)); }
    __device__ static float hi(uint32_t w) { return H::widen((uint16_t)(w >> 16)); }
    __device__ static Acc widen(u32x4 x)
    {
        return Acc{{lo(x.x), hi(x.x), lo(x.y), hi(x.y), lo(x.z), hi(x.z), lo(x.w), hi(x.w)}};
    }
    __device__ static void add(Acc& a, u32x4 x, uint32_t op)
    {
        a.v[0] = combine_fp(op, a.v[0], lo(x.x));
        a.v[1] = combine_fp(op, a.v[1], hi(x.x));
        a.v[2] = combine_fp(op, a.v[2], lo(x.y));
        a.v[3] = combine_fp(op, a.v[3], hi(x.y));
        a.v[4] = combine_fp(op, a.v[4], lo(x.z));
        a.v[5] = combine_fp(op, a.v[5], hi(x.z));
        a.v[6] = combine_fp(op, a.v[6], lo(x.w));
        a.v[7] = combine_fp(op, a.v[7], hi(x.w));
    }
    __device__ static uint32_t pack(float l, float h) { return (uint32_t)H::narrow(l) | ((uint32_t)H::narrow(h) << 16); }
    __device__ static u32x4 narrow(const Acc& a)
    {
        return u32x4{pack(a.v[0], a.v[1]), pack(a.v[2], a.v[3]), pack(a.v[4], a.v[5]), pack(a.v[6], a.v[7])};
    }
    using sacc = float;
    __device__ static sacc swiden(elem x) { return H::widen(x); }
    __device__ static sacc sadd(sacc a, elem x, uint32_t op) { return combine_fp(op, a, H::widen(x)); }
    __device__ static elem snarrow(sacc a) { return H::narrow(a); }
};

// bf16 is the upper half of a binary32
struct Bf16Conv {
    __device__ static float widen(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }
    __device__ static uint16_t narrow(float f)
    {
        const uint32_t u = __float_as_uint(f);
        if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u); // NaN: keep it quiet
        return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
    }
};

// IEEE binary16 through the hardware conversions (v_cvt_f32_f16 is exact, v_cvt_f16_f32 rounds
// to nearest even in the default rounding mode, subnormals included)
struct F16Conv {
    __device__ static float widen(uint16_t h) { return (float)__builtin_bit_cast(_Float16, h); }
    __device__ static uint16_t narrow(float f) { return __builtin_bit_cast(uint16_t, (_Float16)f); }
};

using BF16 = Half16<Bf16Conv>;
using F16 = Half16<F16Conv>;

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

// The step tables are written by the host before the launch and never by a kernel.  Reading
// them through the constant address space tells the compiler so: an address that is uniform
// across the wave is then fetched with scalar loads into SGPRs even after the kernel has issued
// stores.  Through a generic pointer the destination addresses of the store loop came back as
// vector loads, each followed by a wait for every outstanding store and a per-lane uniformity
// loop around every store instruction.
#define LA_CONSTANT __attribute__((address_space(4)))
using table_u64 = const LA_CONSTANT uint64_t*;
using table_seg = const LA_CONSTANT SegInfo*;

template <typename X>
__device__ inline const LA_CONSTANT X* as_table(const X* p)
{
    return (const LA_CONSTANT X*)p;
}

// One element of one segment, all k operands in order: the lanes of segment heads and tails that
// do not fill a 16-byte vector.  The loads of up to ONE_BATCH sources are issued before the first
// of them is added (still in table order): one source at a time, a fan-in of 16 is 16 memory
// latencies in a row in the segment's first workgroup, which at small sizes is the whole launch
// (measured: 10 us of 23) and at medium sizes idles a third of the workgroups.
constexpr uint32_t ONE_BATCH = 8;

template <typename T>
__device__ inline void reduce_one(table_u64 sp, table_u64 dp, uint32_t k, uint32_t m, uint32_t group, uint64_t e,
                                  uint32_t op)
{
    using elem = typename T::elem;
    if (k == 1) { // a copy moves the bits as they are (a signalling NaN stays one)
        const elem x = reinterpret_cast<const elem*>(sp[0])[e];
        for (uint32_t d = 0; d < m; ++d) reinterpret_cast<elem*>(dp[d])[e] = x;
        return;
    }
    typename T::sacc total = T::swiden(elem());
    for (uint32_t t0 = 0; t0 < k; t0 += group) { // one run when group == k
        const uint32_t t1 = t0 + group < k ? t0 + group : k;
        typename T::sacc a = T::swiden(elem());
        for (uint32_t t = t0; t < t1; t += ONE_BATCH) {
            elem x[ONE_BATCH];
#pragma unroll
            for (uint32_t j = 0; j < ONE_BATCH; ++j)
                if (t + j < t1) x[j] = reinterpret_cast<const elem*>(sp[t + j])[e];
#pragma unroll
            for (uint32_t j = 0; j < ONE_BATCH; ++j)
                if (t + j < t1) a = (t + j == t0) ? T::swiden(x[j]) : T::sadd(a, x[j], op);
        }
        const elem run = T::snarrow(a);
        total = t0 == 0 ? T::swiden(run) : T::sadd(total, run, op);
    }
    const elem r = T::snarrow(total);
    for (uint32_t d = 0; d < m; ++d) reinterpret_cast<elem*>(dp[d])[e] = r;
}

// 16 bytes at an address that is only aligned to the element size: the segments whose operands
// disagree modulo 16 bytes (views at different odd offsets).  The packed type tells the compiler
// the true alignment; it emits one global 128-bit access, which the memory system splits where it
// straddles a line.
template <int ALIGN>
struct __attribute__((packed, aligned(ALIGN))) Unaligned16 {
    u32x4 v;
};

#define LA_GLOBAL __attribute__((address_space(1)))

template <int ALIGN>
__device__ inline u32x4 load16_unaligned(uint64_t addr)
{
    return ((const LA_GLOBAL Unaligned16<ALIGN>*)addr)->v;
}

template <int ALIGN>
__device__ inline void store16_unaligned(uint64_t addr, u32x4 v)
{
    ((LA_GLOBAL Unaligned16<ALIGN>*)addr)->v = v;
}

// One 16-byte vector of one segment from operands of any alignment, all k operands in order.
template <typename T>
__device__ inline void reduce_vector_unaligned(table_u64 sp, table_u64 dp, uint32_t k, uint32_t m, uint32_t group,
                                               uint64_t byte_off, uint32_t op)
{
    constexpr int A = (int)sizeof(typename T::elem);
    if (k == 1) { // a copy moves the bits as they are
        const u32x4 x = load16_unaligned<A>(sp[0] + byte_off);
        for (uint32_t d = 0; d < m; ++d) store16_unaligned<A>(dp[d] + byte_off, x);
        return;
    }
    typename T::Acc total;
    for (uint32_t t0 = 0; t0 < k; t0 += group) { // one run when group == k
        const uint32_t t1 = t0 + group < k ? t0 + group : k;
        typename T::Acc a = T::widen(load16_unaligned<A>(sp[t0] + byte_off));
#pragma unroll 4
        for (uint32_t t = t0 + 1; t < t1; ++t) T::add(a, load16_unaligned<A>(sp[t] + byte_off), op);
        if (t0 == 0)
            total = T::widen(T::narrow(a));
        else
            T::add(total, T::narrow(a), op);
    }
    const u32x4 r = T::narrow(total);
    for (uint32_t d = 0; d < m; ++d) store16_unaligned<A>(dp[d] + byte_off, r);
}

// ---- the kernel -------------------------------------------------------------------------------

// Kernel modes.  The sum has instances of its own with the paper's operation compiled in; the
// others take the operation from the launch.  A grouped step adds its sources in runs of
// `group`: every run is reduced and rounded to the buffer's element type as if it had been stored,
// and the run results are then combined in order (one launch that yields, bit for bit, what a
// reduce launch per level would).
enum { MODE_SUM = 0, MODE_ANY_OP = 1, MODE_GROUPED = 2 };

// acc[u] = sources t0 .. t1-1 of the segment, combined in table order (t0 < t1)
template <typename T, int U, typename P>
__device__ __forceinline__ void reduce_run(typename T::Acc (&acc)[U], table_u64 sp, uint32_t t0, uint32_t t1,
                                           uint64_t in_place, uint64_t tile_off, uint32_t tile_bytes,
                                           const uint32_t (&off)[U], uint32_t op)
{
    constexpr int KBATCH = batch_for(U);
    {
        const __amdgpu_buffer_rsrc_t r = tile_rsrc(sp[t0], tile_off, tile_bytes);
        const bool ip = t0 < 64u && ((in_place >> t0) & 1u); // the mask covers 64 sources
#pragma unroll
        for (int u = 0; u < U; ++u) acc[u] = T::widen(load_src<P>(r, off[u], ip));
    }
    uint32_t t = t0 + 1;
    // full batches: KBATCH*U independent 16-byte loads per lane are issued before the adds
    for (; t + KBATCH <= t1; t += KBATCH) {
        u32x4 x[KBATCH][U];
#pragma unroll
        for (int b = 0; b < KBATCH; ++b) {
            const __amdgpu_buffer_rsrc_t r = tile_rsrc(sp[t + b], tile_off, tile_bytes);
            const bool ip = t + b < 64u && ((in_place >> (t + b)) & 1u);
#pragma unroll
            for (int u = 0; u < U; ++u) x[b][u] = load_src<P>(r, off[u], ip);
        }
#pragma unroll
        for (int b = 0; b < KBATCH; ++b)
#pragma unroll
            for (int u = 0; u < U; ++u) T::add(acc[u], x[b][u], op);
    }
    // remaining 0..KBATCH-1 operands
    if constexpr (KBATCH > 1) {
        if (t < t1) {
            const uint32_t rem = t1 - t;
            u32x4 x[KBATCH > 1 ? KBATCH - 1 : 1][U];
#pragma unroll
            for (int b = 0; b < KBATCH - 1; ++b) {
                if ((uint32_t)b < rem) {
                    const __amdgpu_buffer_rsrc_t r = tile_rsrc(sp[t + b], tile_off, tile_bytes);
                    const bool ip = t + b < 64u && ((in_place >> (t + b)) & 1u);
#pragma unroll
                    for (int u = 0; u < U; ++u) x[b][u] = load_src<P>(r, off[u], ip);
                }
            }
#pragma unroll
            for (int b = 0; b < KBATCH - 1; ++b) {
                if ((uint32_t)b < rem) {
#pragma unroll
                    for (int u = 0; u < U; ++u) T::add(acc[u], x[b][u], op);
                }
            }
        }
    }
}

// The .hip sources are compiled once per element type (-DLA_KERNEL_DTYPE=<la_dtype_t value>), so
// that the instances build in parallel.
#if defined(LA_KERNEL_DTYPE)
#if LA_KERNEL_DTYPE == 0
using ElemTraits = I32;
#elif LA_KERNEL_DTYPE == 1
using ElemTraits = F32;
#elif LA_KERNEL_DTYPE == 2
using ElemTraits = BF16;
#elif LA_KERNEL_DTYPE == 3
using ElemTraits = F16;
#elif LA_KERNEL_DTYPE == 4
using ElemTraits = F64;
#else
#error "LA_KERNEL_DTYPE must be 0..4"
#endif
#endif

} // namespace
} // namespace la
