// A consumer of the C ABI with no Python and no torch in the process: allocates the rank buffers
// with HIP, runs the emulated all-reduce of every algorithm on int32 data and compares every
// element of every rank with the definition (the wrapping sum over the ranks).
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <vector>

#include "lane_allreduce.h"

#define HIP_OK(x)                                                                      \
    do {                                                                               \
        hipError_t e_ = (x);                                                           \
        if (e_ != hipSuccess) {                                                        \
            std::printf("%s failed: %s\n", #x, hipGetErrorString(e_));                 \
            return 10;                                                                 \
        }                                                                              \
    } while (0)

static int run(int nodes, int gpus, int procs, la_algo_t algo, unsigned flags, size_t n)
{
    la_topology_t* topo = nullptr;
    la_schedule_t* sched = nullptr;
    if (la_topology_create(nodes, gpus, procs, &topo) != LA_OK) return 1;
    if (la_schedule_build_ex(topo, algo, n, LA_I32, flags, &sched) != LA_OK) {
        std::printf("build: %s\n", la_last_error());
        return 2;
    }
    const int B = la_schedule_num_buffers(sched);
    std::vector<std::vector<int32_t>> host(B, std::vector<int32_t>(n));
    std::vector<uint32_t> want(n, 0u);
    for (int b = 0; b < B; ++b)
        for (size_t i = 0; i < n; ++i) {
            const uint32_t v = (uint32_t)(i * 2654435761u) ^ (uint32_t)(b * 40503u + 0x9e3779b9u);
            host[b][i] = (int32_t)v;
            want[i] += v;
        }
    std::vector<void*> dev(B, nullptr);
    for (int b = 0; b < B; ++b) {
        HIP_OK(hipMalloc(&dev[b], n * sizeof(int32_t)));
        HIP_OK(hipMemcpy(dev[b], host[b].data(), n * sizeof(int32_t), hipMemcpyHostToDevice));
    }
    hipStream_t stream = nullptr;
    HIP_OK(hipStreamCreate(&stream));
    const la_status_t st = la_allreduce_emulated(sched, dev.data(), n, LA_I32, LA_SUM, stream);
    if (st != LA_OK) {
        std::printf("run: %s: %s\n", la_status_string(st), la_last_error());
        return 3;
    }
    HIP_OK(hipStreamSynchronize(stream));
    int bad = 0;
    for (int b = 0; b < B && !bad; ++b) {
        HIP_OK(hipMemcpy(host[b].data(), dev[b], n * sizeof(int32_t), hipMemcpyDeviceToHost));
        for (size_t i = 0; i < n; ++i)
            if ((uint32_t)host[b][i] != want[i]) {
                std::printf("mismatch: buffer %d element %zu\n", b, i);
                bad = 1;
                break;
            }
    }
    for (int b = 0; b < B; ++b) HIP_OK(hipFree(dev[b]));
    HIP_OK(hipStreamDestroy(stream));
    la_schedule_destroy(sched);
    la_topology_destroy(topo);
    return bad ? 4 : 0;
}

int main()
{
    struct Case {
        int nodes, gpus, procs;
        la_algo_t algo;
        unsigned flags;
        size_t n;
    };
    const Case cases[] = {
        {2, 4, 1, LA_ALGO_LANE, LA_SCHED_DEFAULT, 65536},
        {2, 2, 2, LA_ALGO_LANE_MULTIPROC, LA_SCHED_DEFAULT, 100003},
        {3, 2, 1, LA_ALGO_RING, LA_SCHED_DEFAULT, 40961},
        {2, 2, 2, LA_ALGO_LANE_MULTIPROC, LA_SCHED_STAGED, 12289},
        {2, 2, 2, LA_ALGO_LANE_MULTIPROC, LA_SCHED_SHARED_BUFFERS, 70001},
        {4, 2, 1, LA_ALGO_LANE, LA_SCHED_SINGLE_LAUNCH, 262147},
        {2, 2, 2, LA_ALGO_RABENSEIFNER, LA_SCHED_DEFAULT, 5000},
    };
    for (const Case& c : cases) {
        const int rc = run(c.nodes, c.gpus, c.procs, c.algo, c.flags, c.n);
        std::printf("case %dx%dx%d algo %d flags %u n %zu: %s\n", c.nodes, c.gpus, c.procs, (int)c.algo, c.flags, c.n,
                    rc == 0 ? "ok" : "FAILED");
        std::fflush(stdout);
        if (rc) return rc;
    }
    std::printf("all ok\n");
    return 0;
}
