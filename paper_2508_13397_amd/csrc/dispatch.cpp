// Picks the kernel family of an element type and launch shape; the families are built from
// kernels.hip, one translation unit each.
#include "la_internal.hpp"

namespace la {

// launch_family_<dtype>_<family>: one per translation unit built from kernels.hip
#define LA_DECLARE_FAMILIES(d)                                                                          \
    la_status_t launch_family_##d##_0(const StepTable&, const Tuning&, uint32_t blocks, void* stream); \
    la_status_t launch_family_##d##_1(const StepTable&, const Tuning&, uint32_t blocks, void* stream); \
    la_status_t launch_family_##d##_2(const StepTable&, const Tuning&, uint32_t blocks, void* stream);
LA_DECLARE_FAMILIES(0)
LA_DECLARE_FAMILIES(1)
LA_DECLARE_FAMILIES(2)
LA_DECLARE_FAMILIES(3)
LA_DECLARE_FAMILIES(4)
#undef LA_DECLARE_FAMILIES

la_status_t launch_fused_0(const FusedTable&, int unroll, void* stream);
la_status_t launch_fused_1(const FusedTable&, int unroll, void* stream);
la_status_t launch_fused_2(const FusedTable&, int unroll, void* stream);
la_status_t launch_fused_3(const FusedTable&, int unroll, void* stream);
la_status_t launch_fused_4(const FusedTable&, int unroll, void* stream);

namespace {
using FamilyFn = la_status_t (*)(const StepTable&, const Tuning&, uint32_t, void*);
#define LA_FAMILY_ROW(d) {launch_family_##d##_0, launch_family_##d##_1, launch_family_##d##_2}
const FamilyFn kFamilies[5][3] = {LA_FAMILY_ROW(0), LA_FAMILY_ROW(1), LA_FAMILY_ROW(2), LA_FAMILY_ROW(3), LA_FAMILY_ROW(4)};
#undef LA_FAMILY_ROW

// 0: 256 lanes x {1, 2, 4} vectors; 1: 1024 x {1, 2}; 2: 1024 x {4, 8}; -1: no such kernel
int family_of(const Tuning& tune)
{
    const int u = tune.unroll;
    if (tune.block == 256) return (u == 1 || u == 2 || u == 4) ? 0 : -1;
    if (tune.block == 1024) return (u == 1 || u == 2) ? 1 : (u == 4 || u == 8) ? 2 : -1;
    return -1;
}
} // namespace

uint32_t tiles_for(uint64_t max_units, const Tuning& tune)
{
    const uint64_t tile = (uint64_t)tune.block * (uint64_t)tune.unroll;
    const uint64_t tiles = (max_units + tile - 1) / tile;
    return (uint32_t)(tiles ? tiles : 1);
}

// Everything that can refuse a launch, without launching: callers that enqueue other work for the
// launch first (a table upload) ask this before they enqueue anything.
la_status_t check_launch(const StepTable& t, la_dtype_t dtype, const Tuning& tune)
{
    if (t.num_segments == 0) return LA_OK;
    if (t.k < 1 || t.m < 1) return fail(LA_ERR_INVALID_ARG, "internal: step with k=%u m=%u", t.k, t.m);
    if (!known_op((int)t.op)) return fail(LA_ERR_UNSUPPORTED, "unknown operation %u", t.op);
    const uint64_t blocks = (uint64_t)t.edge_blocks + (uint64_t)t.num_segments * t.tiles_per_seg;
    if (blocks > 0x7fffffffull) return fail(LA_ERR_INVALID_ARG, "step needs %llu workgroups", (unsigned long long)blocks);
    if (family_of(tune) < 0)
        return fail(LA_ERR_INVALID_ARG, "unsupported launch shape: %d lanes x %d vectors", tune.block, tune.unroll);
    if (tune.cache_policy < 0 || tune.cache_policy > 7)
        return fail(LA_ERR_INVALID_ARG, "unsupported cache policy %d", tune.cache_policy);
    if (!known_dtype((int)dtype)) return fail(LA_ERR_UNSUPPORTED, "unknown dtype %d", (int)dtype);
    return LA_OK;
}

// The caller guarantees: tables are device-resident and hold num_segments * k (resp. m)
// pointers; every pointer range [ptr, ptr + len*esize) is valid device memory;
// tiles_per_seg covers the longest segment in tiles of tune.block * tune.unroll vectors (counted
// from the tile boundary before its start when t.tiling is TILING_ALIGNED); edge_blocks is 0 or
// covers every segment with EDGE_LANES lanes each.
la_status_t launch_step(const StepTable& t, la_dtype_t dtype, const Tuning& tune, void* hip_stream)
{
    if (t.num_segments == 0) return LA_OK;
    const la_status_t st = check_launch(t, dtype, tune);
    if (st != LA_OK) return st;
    const uint64_t blocks = (uint64_t)t.edge_blocks + (uint64_t)t.num_segments * t.tiles_per_seg;
    return kFamilies[(int)dtype][family_of(tune)](t, tune, (uint32_t)blocks, hip_stream);
}

// One launch for the whole schedule (fused.hip, one translation unit per element type).
la_status_t launch_fused(const FusedTable& t, la_dtype_t dtype, int unroll, void* hip_stream)
{
    if (t.workgroups == 0) return LA_OK;
    if (!known_op((int)t.op_code)) return fail(LA_ERR_UNSUPPORTED, "unknown operation %u", t.op_code);
    if (t.workgroups > 0x7fffffffu) return fail(LA_ERR_INVALID_ARG, "fused launch needs %u workgroups", t.workgroups);
    switch (dtype) {
    case LA_I32: return launch_fused_0(t, unroll, hip_stream);
    case LA_F32: return launch_fused_1(t, unroll, hip_stream);
    case LA_BF16: return launch_fused_2(t, unroll, hip_stream);
    case LA_F16: return launch_fused_3(t, unroll, hip_stream);
    case LA_F64: return launch_fused_4(t, unroll, hip_stream);
    }
    return fail(LA_ERR_UNSUPPORTED, "unknown dtype %d", (int)dtype);
}

} // namespace la
