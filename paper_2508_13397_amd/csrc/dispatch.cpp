// Picks the kernel family of an element type; the families are built from kernels.hip, one
// translation unit per type.
#include "la_internal.hpp"

namespace la {

la_status_t launch_step_i32(const StepTable& t, const Tuning& tune, uint32_t blocks, void* stream);
la_status_t launch_step_f32(const StepTable& t, const Tuning& tune, uint32_t blocks, void* stream);
la_status_t launch_step_bf16(const StepTable& t, const Tuning& tune, uint32_t blocks, void* stream);
la_status_t launch_step_f16(const StepTable& t, const Tuning& tune, uint32_t blocks, void* stream);
la_status_t launch_step_f64(const StepTable& t, const Tuning& tune, uint32_t blocks, void* stream);

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
    if (!known_op((int)t.op)) return fail(LA_ERR_UNSUPPORTED, "unknown operation %u", t.op);
    const uint64_t blocks = (uint64_t)t.num_segments * t.tiles_per_seg;
    if (blocks > 0x7fffffffull) return fail(LA_ERR_INVALID_ARG, "step needs %llu workgroups", (unsigned long long)blocks);
    switch (dtype) {
    case LA_I32: return launch_step_i32(t, tune, (uint32_t)blocks, hip_stream);
    case LA_F32: return launch_step_f32(t, tune, (uint32_t)blocks, hip_stream);
    case LA_BF16: return launch_step_bf16(t, tune, (uint32_t)blocks, hip_stream);
    case LA_F16: return launch_step_f16(t, tune, (uint32_t)blocks, hip_stream);
    case LA_F64: return launch_step_f64(t, tune, (uint32_t)blocks, hip_stream);
    }
    return fail(LA_ERR_UNSUPPORTED, "unknown dtype %d", (int)dtype);
}

} // namespace la
