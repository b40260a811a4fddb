// Host-only exerciser of the schedule generator, the table accessors, the launch planner and the
// column analysis: builds schedules for many topologies, algorithms, flags, lengths and element
// types and reads everything back through the C header.  tests/test_host_sanitizers.py compiles it
// together with the library's host sources under AddressSanitizer and UBSan (host side only) and
// runs it; no GPU call is made, the kernel launchers are the stubs below.
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "la_internal.hpp"
#include "lane_allreduce.h"

namespace la {
#define LA_STUB(d)                                                                                                   \
    la_status_t launch_family_##d##_0(const StepTable&, const Tuning&, uint32_t, void*) { return LA_ERR_DEVICE; }   \
    la_status_t launch_family_##d##_1(const StepTable&, const Tuning&, uint32_t, void*) { return LA_ERR_DEVICE; }   \
    la_status_t launch_family_##d##_2(const StepTable&, const Tuning&, uint32_t, void*) { return LA_ERR_DEVICE; }   \
    la_status_t launch_fused_##d(const FusedTable&, int, void*) { return LA_ERR_DEVICE; }
LA_STUB(0) LA_STUB(1) LA_STUB(2) LA_STUB(3) LA_STUB(4)
#undef LA_STUB
} // namespace la

static unsigned long long rng = 88172645463325252ull;
static unsigned rnd() { rng ^= rng << 13; rng ^= rng >> 7; rng ^= rng << 17; return (unsigned)(rng >> 11); }

int main()
{
    const int topos[][3] = {{1, 1, 1}, {1, 1, 2}, {2, 1, 1}, {2, 2, 2}, {3, 2, 2}, {4, 4, 1}, {5, 1, 3}, {16, 1, 1}, {2, 4, 2}, {3, 3, 3}, {8, 4, 4}};
    const unsigned flagsets[] = {0,1,2,3,4,5,6,8,10,12,16,17,20,32,64,33,65,36,68,128,129,132,256,24,40,72,136,264,48,80};
    const size_t ns[] = {1, 7, 100, 4097, 70001};
    long built = 0, refused = 0;
    for (auto& t : topos) {
        la_topology_t* topo = nullptr;
        if (la_topology_create(t[0], t[1], t[2], &topo) != LA_OK) return 1;
        if (la_topology_num_ranks(topo) != t[0] * t[1] * t[2]) return 9;
        for (int algo = 0; algo < 5; ++algo)
            for (unsigned flags : flagsets)
                for (size_t n : ns) {
                    for (int dt = 0; dt < 5; dt += (n % 3 == 0 ? 1 : 2)) {
                        la_schedule_t* s = nullptr;
                        const la_status_t st = la_schedule_build_ex(topo, (la_algo_t)algo, n, (la_dtype_t)dt, flags, &s);
                        if (st != LA_OK) { ++refused; continue; }
                        ++built;
                        const int steps = la_schedule_num_steps(s), nb = la_schedule_num_buffers(s);
                        const size_t e = dt == 4 ? 8 : (dt >= 2 ? 2 : 4);
                        const bool oop = (flags & 16u) != 0;
                        // fake addresses: aligned or shifted by a few elements
                        std::vector<const void*> bufs(nb), send(nb);
                        const size_t shift = (rnd() % 3 == 0) ? (rnd() % 8) * e : 0;
                        for (int b = 0; b < nb; ++b) {
                            bufs[b] = (const void*)((1ull << 40) + (unsigned long long)b * ((n * e + 4095) / 4096 * 4096 + 4096) + shift);
                            send[b] = (const void*)((1ull << 44) + (unsigned long long)b * ((n * e + 4095) / 4096 * 4096 + 4096) + shift);
                        }
                        const void* staging = la_schedule_staging_elems(s) ? (const void*)(1ull << 46) : nullptr;
                        for (int i = 0; i < steps; ++i) {
                            int kind, stage, k, m; size_t S, lmax, br, bw;
                            if (la_schedule_step_info(s, i, &kind, &stage, &S, &lmax, &k, &m, &br, &bw) != LA_OK) return 2;
                            std::vector<uint64_t> len(S), so(S * k), dof(S * m);
                            std::vector<int32_t> sb(S * k), db(S * m);
                            if (la_schedule_step_table(s, i, len.data(), sb.data(), so.data(), db.data(), dof.data()) != LA_OK) return 3;
                            (void)la_schedule_step_group(s, i);
                            la_launch_plan_t plan;
                            const la_status_t ps = la_schedule_launch_plan(s, i, bufs.data(), oop ? send.data() : nullptr, staging, &plan);
                            if (ps != LA_OK) { std::printf("plan failed: %s\n", la_last_error()); return 4; }
                            size_t count = 0;
                            if (la_schedule_launch_segments(s, i, bufs.data(), oop ? send.data() : nullptr, staging, 0, &count, nullptr, nullptr, nullptr) != LA_OK) return 5;
                            std::vector<uint64_t> l2(count), sa(count * k), da(count * m);
                            if (la_schedule_launch_segments(s, i, bufs.data(), oop ? send.data() : nullptr, staging, count, &count, l2.data(), sa.data(), da.data()) != LA_OK) return 6;
                        }
                        for (int b = 0; b < nb; ++b) {
                            uint64_t off[64], ln[64];
                            (void)la_schedule_owned_ranges(s, b, 64, off, ln);
                        }
                        const int runs = la_schedule_fusion_runs(s);
                        for (int r = 0; r < runs; ++r) {
                            int f, c, a; uint64_t C, O; size_t br, bw;
                            if (la_schedule_fusion_info(s, r, &f, &c, &C, &O, &a, &br, &bw) != LA_OK) return 7;
                            std::vector<uint64_t> lo(C), ln(C), fo(C + 1);
                            std::vector<uint32_t> os(O), og(O);
                            std::vector<int32_t> pf(O), fw(O);
                            if (la_schedule_fusion_table(s, r, lo.data(), ln.data(), fo.data(), os.data(), og.data(), pf.data(), fw.data()) != LA_OK) return 8;
                        }
                        la_schedule_destroy(s);
                    }
                }
        la_topology_destroy(topo);
    }
    std::printf("built %ld schedules, %ld refused: ok\n", built, refused);
    return 0;
}
