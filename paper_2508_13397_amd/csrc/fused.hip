// gfx950 kernel that runs a whole run of steps in one launch, chain by chain.
//
// Algorithm 1 needs 2(P - 1) dependent steps, and the ring form of Algorithm 2's inter-node stage
// 2(N - 1); one launch per step costs about 4 us of launch gap whatever the step carries, which at
// P = 1024 is most of the time.  But the steps are column-wise: a chunk at elements [a, b) only ever
// meets elements [a, b) of other buffers (fusion.cpp), so the element axis falls into chains that
// never exchange data.  Here one wave owns up to 64 * U 16-byte vectors of one chain and executes
// the chain's operations in step order: it combines the (at most two) sources in table order and
// stores to the (at most two) destinations, the arithmetic and the stores of the per-step launches.
// A lane works on the same elements in every operation, so what an operation reads from an earlier
// one was stored by the same lane: program order is all the ordering there is.  No barrier, no flag,
// no wait on another wave: every workgroup ends after its chain's last operation.
//
// Three things keep memory latency out of the chain of dependent operations:
//  * a source that no earlier operation of the chain has written is an original input of the run; its
//    address is known from the start, so its load is issued PREFETCH_DEPTH operations ahead
//    (non-temporal: it is read once);
//  * a source that is exactly what the previous operation stored (the chunk a rank has just received
//    from its predecessor) is taken from the registers of the lane that stored it;
//  * the operation records themselves are requested RECORD_DEPTH operations ahead.
#include <hip/hip_runtime.h>

#include "kernel_common.hpp"
#include "la_internal.hpp"

namespace la {

namespace {

constexpr int PREFETCH_DEPTH = 4; // original inputs are requested this many operations ahead
constexpr int RECORD_DEPTH = 8;   // operation records this many ahead; chains are padded to a multiple of it

// What every operation of a workgroup's chain needs.
template <int U>
struct ChainContext {
    uint64_t ops;        // address of the chain's first record
    uint64_t tile_off;   // bytes from the chain's first element to this workgroup's first vector
    uint32_t tile_bytes;
    uint32_t num_ops, op;
    uint32_t off[U];
    uint32_t record_lane; // byte offset of the dword of a record that this lane fetches
};

// The 64-byte record of operation j, one dword per lane (lanes 16 and up repeat lanes 0 to 15).
// The records of a chain are read once, in order, from tables of tens of megabytes, so every one is
// a trip to memory.  Fetched with scalar loads that trip stalls the wave at its next scalar use
// (scalar loads complete out of order and can only be waited for all together): 1.6 us per operation
// on Algorithm 1 over 1024 ranks.  A vector load is counted in order, so the record can be requested
// RECORD_DEPTH operations ahead and picked up, lane by lane, when its operation comes.  Beyond the
// chain's end the last record is fetched again (and never used).
template <int U>
__device__ __forceinline__ uint32_t load_record(const ChainContext<U>& c, uint32_t j)
{
    const uint32_t at = j < c.num_ops ? j : c.num_ops - 1;
    return *reinterpret_cast<const LA_GLOBAL uint32_t*>(c.ops + (uint64_t)at * sizeof(FusedOp) + c.record_lane);
}

__device__ __forceinline__ uint32_t record_dword(uint32_t rec, int i)
{
    return (uint32_t)__builtin_amdgcn_readlane((int)rec, i);
}

__device__ __forceinline__ uint64_t record_address(uint32_t rec, int i) // addr[i] of the record
{
    return (uint64_t)record_dword(rec, 4 + 2 * i) | ((uint64_t)record_dword(rec, 5 + 2 * i) << 32);
}

// Operation with record `rec` of the chain; `ahead` is the record of the operation PREFETCH_DEPTH
// later; `slot` holds the operation's prefetched source (if it has one) and is refilled with that
// of the later operation; `last` is what this lane stored in the previous operation.
template <typename T, int U>
__device__ __forceinline__ void chain_op(const ChainContext<U>& c, uint32_t rec, uint32_t ahead, u32x4 (&slot)[U],
                                         u32x4 (&last)[U])
{
    using P = Policy<1>; // original inputs non-temporal; sources an earlier operation wrote, and all stores, plain
    if ((record_dword(rec, 1) & 1u) != 0) { // not padding behind the chain's last operation
        const uint32_t km = record_dword(rec, 2), pf = record_dword(rec, 3);
        const uint32_t k = km & 0xffffu, m = km >> 16;
        const int32_t ps = (int16_t)(pf & 0xffffu), fw = (int16_t)(pf >> 16);
        const uint64_t s0 = record_address(rec, 0), a1 = record_address(rec, 1);
        u32x4 x0[U], out[U];
        // A source that is exactly what this lane stored in the previous operation of the chain (the
        // chunk a rank has just received) is taken from the registers, one that was requested ahead
        // of time from its slot; only a source that is neither is loaded now (plain: an earlier
        // operation of the chain may have written it).
        if (fw == 0) {
#pragma unroll
            for (int u = 0; u < U; ++u) x0[u] = last[u];
        } else if (ps == 0) {
#pragma unroll
            for (int u = 0; u < U; ++u) x0[u] = slot[u];
        } else {
            const __amdgpu_buffer_rsrc_t r = tile_rsrc(s0, c.tile_off, c.tile_bytes);
#pragma unroll
            for (int u = 0; u < U; ++u) x0[u] = load16<P::LDA>(r, c.off[u]);
        }
        if (k == 2) {
            u32x4 x1[U];
            if (fw == 1) {
#pragma unroll
                for (int u = 0; u < U; ++u) x1[u] = last[u];
            } else if (ps == 1) {
#pragma unroll
                for (int u = 0; u < U; ++u) x1[u] = slot[u];
            } else {
                const __amdgpu_buffer_rsrc_t r = tile_rsrc(a1, c.tile_off, c.tile_bytes);
#pragma unroll
                for (int u = 0; u < U; ++u) x1[u] = load16<P::LDA>(r, c.off[u]);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                typename T::Acc a = T::widen(x0[u]);
                T::add(a, x1[u], c.op);
                out[u] = T::narrow(a);
            }
        } else { // a copy moves the bits as they are
#pragma unroll
            for (int u = 0; u < U; ++u) out[u] = x0[u];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) last[u] = out[u];
        const uint64_t d0 = k == 2 ? record_address(rec, 2) : a1;
        {
            const __amdgpu_buffer_rsrc_t r = tile_rsrc(d0, c.tile_off, c.tile_bytes);
#pragma unroll
            for (int u = 0; u < U; ++u) store16<P::ST>(r, c.off[u], out[u]);
        }
        if (m == 2) {
            const uint64_t d1 = k == 2 ? record_address(rec, 3) : record_address(rec, 2);
            const __amdgpu_buffer_rsrc_t r = tile_rsrc(d1, c.tile_off, c.tile_bytes);
#pragma unroll
            for (int u = 0; u < U; ++u) store16<P::ST>(r, c.off[u], out[u]);
        }
    }
    // the slot is free: request the original input of the operation PREFETCH_DEPTH ahead, if it has one
    const int32_t pn = (int16_t)(record_dword(ahead, 3) & 0xffffu);
    if (pn >= 0 && (record_dword(ahead, 1) & 1u) != 0) {
        const uint64_t next = pn == 1 ? record_address(ahead, 1) : record_address(ahead, 0);
        const __amdgpu_buffer_rsrc_t r = tile_rsrc(next, c.tile_off, c.tile_bytes);
#pragma unroll
        for (int u = 0; u < U; ++u) slot[u] = load16<P::LD>(r, c.off[u]);
    }
}

// The elements before the first and after the last whole 16-byte vector of a chain (at most 14):
// one lane each, operation after operation, in a workgroup of their own.  Every source is loaded
// from memory; a lane reads what it stored itself.
template <typename T>
__device__ void edge_chain(const LA_CONSTANT FusedOp* ops, uint32_t num_ops, uint64_t elem, uint32_t op)
{
    using elem_t = typename T::elem;
    for (uint32_t j = 0; j < num_ops; ++j) {
        if ((ops[j].live & 1u) == 0) continue;
        const uint32_t k = ops[j].k, m = ops[j].m;
        const elem_t e0 = reinterpret_cast<const elem_t*>(ops[j].addr[0])[elem];
        elem_t r = e0;
        if (k == 2) r = T::snarrow(T::sadd(T::swiden(e0), reinterpret_cast<const elem_t*>(ops[j].addr[1])[elem], op));
        reinterpret_cast<elem_t*>(ops[j].addr[k])[elem] = r;
        if (m == 2) reinterpret_cast<elem_t*>(ops[j].addr[k + 1])[elem] = r;
    }
}

// Eight consecutive operations of one of the two shapes that make up a ring, as straight-line code.
//   FUSED_BLOCK_ADD   every operation adds what the lane stored in the previous operation (source 1)
//                     to an original input that was requested ahead of time (source 0) and stores to
//                     one destination: a rank receives a partial sum and adds its own copy;
//   FUSED_BLOCK_COPY  every operation stores what the lane stored in the previous operation to one
//                     destination: a rank receives a finished chunk.
// The host marks a block (in its first record) only if, in addition, the four operations behind it
// want a prefetch (ADD) or none of them does (COPY), so that no access in the block is conditional.
// Without branches the compiler can count which of the loads in flight an operation has to wait
// for; the general path below, with its branches, waits for all of them in every operation, which
// made every operation as long as a trip to memory (1.4 us on Algorithm 1 over 1024 ranks).
template <typename T, int U, int KIND>
__device__ __forceinline__ void ring_block(const ChainContext<U>& c, uint32_t j, uint32_t (&r)[RECORD_DEPTH],
                                           u32x4 (&slot)[PREFETCH_DEPTH][U], u32x4 (&last)[U])
{
    using P = Policy<1>;
#pragma unroll
    for (int i = 0; i < RECORD_DEPTH; ++i) {
        // The record is "produced" here as far as the compiler can tell, so its lane reads (cheap,
        // free of side effects) are not gathered at the top of the block, where the wait for the
        // youngest record would be a wait for a load issued one operation ago.
        asm volatile("" : "+v"(r[i]));
        const uint32_t rec = r[i];
        if constexpr (KIND == FUSED_BLOCK_ADD) {
            const uint64_t d0 = record_address(rec, 2);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                typename T::Acc a = T::widen(slot[i % PREFETCH_DEPTH][u]);
                T::add(a, last[u], c.op);
                last[u] = T::narrow(a);
            }
            const __amdgpu_buffer_rsrc_t rd = tile_rsrc(d0, c.tile_off, c.tile_bytes);
#pragma unroll
            for (int u = 0; u < U; ++u) store16<P::ST>(rd, c.off[u], last[u]);
            const __amdgpu_buffer_rsrc_t rn =
                tile_rsrc(record_address(r[(i + PREFETCH_DEPTH) % RECORD_DEPTH], 0), c.tile_off, c.tile_bytes);
#pragma unroll
            for (int u = 0; u < U; ++u) slot[i % PREFETCH_DEPTH][u] = load16<P::LD>(rn, c.off[u]);
        } else {
            const __amdgpu_buffer_rsrc_t rd = tile_rsrc(record_address(rec, 1), c.tile_off, c.tile_bytes);
#pragma unroll
            for (int u = 0; u < U; ++u) store16<P::ST>(rd, c.off[u], last[u]);
        }
        r[i] = load_record<U>(c, j + RECORD_DEPTH + (uint32_t)i);
        __builtin_amdgcn_sched_barrier(0); // and the scheduler keeps every operation's instructions together
    }
}

template <typename T, int U, int MODE>
__global__ __launch_bounds__(FUSED_LANES) __attribute__((amdgpu_waves_per_eu(8, 8))) void fused_chain_kernel(FusedTable tab)
{
    using elem = typename T::elem;
    static_assert(PREFETCH_DEPTH == 4 && RECORD_DEPTH == 8 && RECORD_DEPTH == (int)FUSED_CHAIN_PAD, "slots and padding");
    const uint32_t tid = threadIdx.x;
    const uint32_t chain = ((const LA_CONSTANT uint32_t*)tab.wg_chain)[blockIdx.x];
    const uint32_t tile = ((const LA_CONSTANT uint32_t*)tab.wg_tile)[blockIdx.x];
    const LA_CONSTANT ChainInfo* ci = as_table(tab.chain) + chain;
    const uint64_t nvec = ci->nvec;
    const uint32_t head = ci->head, tail = ci->tail;
    const uint32_t op = MODE == MODE_SUM ? (uint32_t)LA_SUM : tab.op_code;
    if (tile == FUSED_EDGE_TILE) {
        if (tid < head + tail)
            edge_chain<T>(as_table(tab.op) + ci->first_op, ci->num_ops,
                          tid < head ? tid : (uint64_t)head + nvec * T::VEC + (tid - head), op);
        return;
    }

    constexpr uint64_t TILE = (uint64_t)FUSED_LANES * U; // vectors per workgroup
    const uint64_t v0 = (uint64_t)tile * TILE;
    const uint64_t left = nvec - v0; // the host makes tiles only where there are vectors
    ChainContext<U> c;
    c.ops = reinterpret_cast<uint64_t>(tab.op + ci->first_op);
    c.num_ops = ci->num_ops; // a multiple of RECORD_DEPTH
    c.op = op;
    c.tile_bytes = (uint32_t)(left < TILE ? left : TILE) * 16u;
    c.tile_off = (uint64_t)head * sizeof(elem) + v0 * 16u;
#pragma unroll
    for (int u = 0; u < U; ++u) c.off[u] = (tid + (uint32_t)u * FUSED_LANES) * 16u;
    c.record_lane = (tid & 15u) * 4u;

    uint32_t r[RECORD_DEPTH];
#pragma unroll
    for (int i = 0; i < RECORD_DEPTH; ++i) r[i] = load_record<U>(c, (uint32_t)i);
    u32x4 slot[PREFETCH_DEPTH][U], last[U], none[U];
#pragma unroll
    for (int u = 0; u < U; ++u) last[u] = none[u] = u32x4{0, 0, 0, 0};
    // the first PREFETCH_DEPTH operations' original inputs: requested through the same code as later
    // ones, by four operations that do nothing (a record of zeros is padding) but prefetch
#pragma unroll
    for (int i = 0; i < PREFETCH_DEPTH; ++i) chain_op<T, U>(c, 0u, r[i], slot[i], none);
    // Consecutive blocks of one ring shape run in a loop of their own: with a single path round the
    // loop the values it carries (records, prefetched inputs, the vector in hand) stay in their
    // registers, whereas at a join of the three paths they were moved, and a move waits for every
    // load that is still in flight.
    uint32_t j = 0;
    while (j < c.num_ops) {
        const uint32_t kind = record_dword(r[0], 1) >> 8; // of the eight operations that start here
        if (MODE == MODE_SUM && kind == FUSED_BLOCK_ADD) {
            do {
                ring_block<T, U, FUSED_BLOCK_ADD>(c, j, r, slot, last);
                j += RECORD_DEPTH;
            } while (j < c.num_ops && (record_dword(r[0], 1) >> 8) == FUSED_BLOCK_ADD);
        } else if (kind == FUSED_BLOCK_COPY) {
            do {
                ring_block<T, U, FUSED_BLOCK_COPY>(c, j, r, slot, last);
                j += RECORD_DEPTH;
            } while (j < c.num_ops && (record_dword(r[0], 1) >> 8) == FUSED_BLOCK_COPY);
        } else {
#pragma unroll
            for (int i = 0; i < RECORD_DEPTH; ++i) {
                chain_op<T, U>(c, r[i], r[(i + PREFETCH_DEPTH) % RECORD_DEPTH], slot[i % PREFETCH_DEPTH], last);
                r[i] = load_record<U>(c, j + RECORD_DEPTH + (uint32_t)i);
            }
            j += RECORD_DEPTH;
        }
    }
}

template <typename T, int U>
la_status_t launch_unroll(const FusedTable& t, hipStream_t s)
{
    if (t.op_code == (uint32_t)LA_SUM)
        hipLaunchKernelGGL((fused_chain_kernel<T, U, MODE_SUM>), dim3(t.workgroups), dim3(FUSED_LANES), 0, s, t);
    else
        hipLaunchKernelGGL((fused_chain_kernel<T, U, MODE_ANY_OP>), dim3(t.workgroups), dim3(FUSED_LANES), 0, s, t);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(LA_ERR_DEVICE, "kernel launch failed: %s", hipGetErrorString(e));
    return LA_OK;
}

} // namespace

#if !defined(LA_KERNEL_DTYPE)
#error "compile fused.hip with -DLA_KERNEL_DTYPE=0..4"
#endif

#define LA_CONCAT2(a, b) a##b
#define LA_FUSED_NAME(d) LA_CONCAT2(launch_fused_, d)
// The caller guarantees: the tables are device-resident and consistent (every workgroup's chain and
// tile exist, every op has one or two sources and destinations whose addresses are valid for the
// chain's whole column range), all operand addresses agree modulo 16 bytes, unroll is 1 and wg_tile
// counts tiles of 64 vectors.
la_status_t LA_FUSED_NAME(LA_KERNEL_DTYPE)(const FusedTable& t, int unroll, void* stream)
{
    // one vector per lane: more, smaller pieces of chains in flight did better at every size measured
    // (16 ranks x 64 MiB: 467 / 489 / 517 us with 1 / 2 / 4 vectors; 1024 ranks x 4 MiB: 2927 / 2957 / 3331)
    if (unroll != 1) return fail(LA_ERR_INVALID_ARG, "internal: fused launch with %d vectors per lane", unroll);
    return launch_unroll<ElemTraits, 1>(t, static_cast<hipStream_t>(stream));
}

} // namespace la
