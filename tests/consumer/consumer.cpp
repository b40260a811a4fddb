// A consumer of the C ABI with no Python and no torch in the process: allocates the rank buffers
// with HIP, runs the emulated all-reduce of every algorithm on int32 data and compares every
// element of every rank with the definition (the wrapping sum over the ranks); executes the step
// tables it reads through la_schedule_step_info / la_schedule_step_table on the host and compares
// with what the library left after every step; calls la_reduce_segments (and its allocation-free
// variant) and the out-of-place entry point; and checks that bad arguments are refused with
// LA_ERR_INVALID_ARG and a message.
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

static uint32_t value(int b, size_t i)
{
    return (uint32_t)(i * 2654435761u) ^ (uint32_t)(b * 40503u + 0x9e3779b9u);
}

// The tables as data: every step run on the GPU by itself (la_schedule_run_steps, with a given
// operation) and, from the tables read through the C ABI, on the host; the states must agree after
// every step.  int32: sum wraps, maximum compares as signed.
static int steps_from_tables(int nodes, int gpus, int procs, la_algo_t algo, unsigned flags, size_t n, la_op_t op)
{
    la_topology_t* topo = nullptr;
    la_schedule_t* sched = nullptr;
    if (la_topology_create(nodes, gpus, procs, &topo) != LA_OK) return 1;
    if (la_schedule_build_ex(topo, algo, n, LA_I32, flags, &sched) != LA_OK) return 2;
    const int B = la_schedule_num_buffers(sched), S = la_schedule_num_steps(sched);
    if (B != la_topology_num_ranks(topo) || S < 1) return 3;
    std::vector<std::vector<uint32_t>> host(B, std::vector<uint32_t>(n)), got(B, std::vector<uint32_t>(n));
    std::vector<void*> dev(B, nullptr);
    for (int b = 0; b < B; ++b) {
        for (size_t i = 0; i < n; ++i) host[b][i] = value(b, i);
        HIP_OK(hipMalloc(&dev[b], n * sizeof(uint32_t)));
        HIP_OK(hipMemcpy(dev[b], host[b].data(), n * sizeof(uint32_t), hipMemcpyHostToDevice));
    }
    size_t total_read = 0, total_written = 0;
    for (int step = 0; step < S; ++step) {
        int kind = -1, stage = -1, k = 0, m = 0;
        size_t segs = 0, longest = 0, rd = 0, wr = 0;
        if (la_schedule_step_info(sched, step, &kind, &stage, &segs, &longest, &k, &m, &rd, &wr) != LA_OK) return 4;
        if (k < 1 || m < 1 || segs < 1 || (kind != LA_STEP_REDUCE && kind != LA_STEP_COPY) || longest > n) return 5;
        std::vector<uint64_t> len(segs), soff(segs * k), doff(segs * m);
        std::vector<int32_t> sbuf(segs * k), dbuf(segs * m);
        if (la_schedule_step_table(sched, step, len.data(), sbuf.data(), soff.data(), dbuf.data(), doff.data()) != LA_OK) return 6;
        size_t elems = 0;
        std::vector<std::vector<uint32_t>> before = host; // every segment of a step reads the state before the step
        for (size_t g = 0; g < segs; ++g) {
            elems += len[g];
            for (uint64_t i = 0; i < len[g]; ++i) {
                uint32_t acc = before[sbuf[g * k]][soff[g * k] + i];
                for (int t = 1; t < k; ++t) {
                    const uint32_t x = before[sbuf[g * k + t]][soff[g * k + t] + i];
                    acc = op == LA_SUM ? acc + x : ((int32_t)x > (int32_t)acc ? x : acc);
                }
                for (int d = 0; d < m; ++d) host[dbuf[g * m + d]][doff[g * m + d] + i] = acc;
            }
        }
        if (rd != elems * (size_t)k * 4 || wr != elems * (size_t)m * 4) return 7; // bytes of the step as documented
        total_read += rd;
        total_written += wr;
        if (la_schedule_run_steps(sched, step, 1, dev.data(), op, nullptr) != LA_OK) {
            std::printf("run_steps: %s\n", la_last_error());
            return 8;
        }
        HIP_OK(hipDeviceSynchronize());
        for (int b = 0; b < B; ++b) {
            HIP_OK(hipMemcpy(got[b].data(), dev[b], n * sizeof(uint32_t), hipMemcpyDeviceToHost));
            if (got[b] != host[b]) {
                std::printf("step %d (stage %d): buffer %d differs from the tables executed on the host\n", step, stage, b);
                return 9;
            }
        }
    }
    // the end state is the definition on every rank
    for (size_t i = 0; i < n; ++i) {
        uint32_t want = value(0, i);
        for (int b = 1; b < B; ++b) {
            const uint32_t x = value(b, i);
            want = op == LA_SUM ? want + x : ((int32_t)x > (int32_t)want ? x : want);
        }
        for (int b = 0; b < B; ++b)
            if (host[b][i] != want) return 11;
    }
    // the column analysis through the C ABI: the operations of every run cover its steps' segments exactly
    const int runs = la_schedule_fusion_runs(sched);
    if (runs < 0) return 12;
    for (int r = 0; r < runs; ++r) {
        int first = -1, count = 0, automatic = -1;
        uint64_t chains = 0, ops = 0;
        size_t frd = 0, fwr = 0;
        if (la_schedule_fusion_info(sched, r, &first, &count, &chains, &ops, &automatic, &frd, &fwr) != LA_OK) return 13;
        if (first < 0 || count < 2 || first + count > S || chains < 1 || ops < chains || frd > total_read || fwr > total_written) return 14;
    }
    for (int b = 0; b < B; ++b) HIP_OK(hipFree(dev[b]));
    la_schedule_destroy(sched);
    la_topology_destroy(topo);
    return 0;
}

// la_reduce_segments and la_reduce_segments_static: dst = ((dst + src0) + src1) + ... on the segments, untouched elsewhere.
static int reduce_segments()
{
    const size_t n = 200003, seg_len = 7001;
    const size_t offs[4] = {5, 20000, 90001, 193000};
    const int k = 3;
    for (int variant = 0; variant < 2; ++variant) {
        std::vector<uint32_t> host_dst(n), want(n), back(n);
        std::vector<std::vector<uint32_t>> host_src(k, std::vector<uint32_t>(n));
        for (size_t i = 0; i < n; ++i) {
            host_dst[i] = want[i] = value(100, i);
            for (int t = 0; t < k; ++t) host_src[t][i] = value(t, i);
        }
        for (size_t s : offs)
            for (size_t i = s; i < s + seg_len; ++i)
                for (int t = 0; t < k; ++t) want[i] += host_src[t][i];
        void* dst = nullptr;
        void* src[k];
        HIP_OK(hipMalloc(&dst, n * 4));
        HIP_OK(hipMemcpy(dst, host_dst.data(), n * 4, hipMemcpyHostToDevice));
        for (int t = 0; t < k; ++t) {
            HIP_OK(hipMalloc(&src[t], n * 4));
            HIP_OK(hipMemcpy(src[t], host_src[t].data(), n * 4, hipMemcpyHostToDevice));
        }
        const la_status_t st = variant == 0 ? la_reduce_segments(dst, src, k, offs, 4, seg_len, LA_I32, LA_SUM, nullptr)
                                            : la_reduce_segments_static(dst, src, k, offs, 4, seg_len, LA_I32, LA_SUM, nullptr);
        if (st != LA_OK) {
            std::printf("reduce_segments variant %d: %s\n", variant, la_last_error());
            return 1;
        }
        HIP_OK(hipDeviceSynchronize());
        HIP_OK(hipMemcpy(back.data(), dst, n * 4, hipMemcpyDeviceToHost));
        if (back != want) return 2;
        // refused calls: a source that is the destination, overlapping segments, a NULL source
        const size_t overlap[2] = {0, seg_len - 1};
        void* alias[1] = {dst};
        void* null_src[1] = {nullptr};
        if (la_reduce_segments(dst, alias, 1, offs, 4, seg_len, LA_I32, LA_SUM, nullptr) != LA_ERR_INVALID_ARG) return 3;
        if (la_reduce_segments(dst, src, k, overlap, 2, seg_len, LA_I32, LA_SUM, nullptr) != LA_ERR_INVALID_ARG) return 4;
        if (la_reduce_segments(dst, null_src, 1, offs, 4, seg_len, LA_I32, LA_SUM, nullptr) != LA_ERR_INVALID_ARG) return 5;
        if (la_last_error()[0] == 0) return 6;
        HIP_OK(hipDeviceSynchronize());
        HIP_OK(hipMemcpy(back.data(), dst, n * 4, hipMemcpyDeviceToHost));
        if (back != want) return 7; // a refused call enqueues nothing
        HIP_OK(hipFree(dst));
        for (int t = 0; t < k; ++t) HIP_OK(hipFree(src[t]));
    }
    return 0;
}

// Separate send and receive buffers, and the argument errors of the run calls.
static int out_of_place_and_errors()
{
    const size_t n = 30011;
    la_topology_t* topo = nullptr;
    la_schedule_t *oop = nullptr, *in_place = nullptr;
    if (la_topology_create(2, 2, 2, &topo) != LA_OK) return 1;
    if (la_schedule_build_ex(topo, LA_ALGO_LANE_MULTIPROC, n, LA_I32, LA_SCHED_OUT_OF_PLACE, &oop) != LA_OK) return 2;
    if (la_schedule_build(topo, LA_ALGO_LANE_MULTIPROC, n, LA_I32, &in_place) != LA_OK) return 3;
    const int B = 8;
    std::vector<void*> send(B), recv(B);
    std::vector<uint32_t> want(n, 0u), tmp(n);
    for (int b = 0; b < B; ++b) {
        for (size_t i = 0; i < n; ++i) {
            tmp[i] = value(b, i);
            want[i] += tmp[i];
        }
        HIP_OK(hipMalloc(&send[b], n * 4));
        HIP_OK(hipMalloc(&recv[b], n * 4));
        HIP_OK(hipMemcpy(send[b], tmp.data(), n * 4, hipMemcpyHostToDevice));
        HIP_OK(hipMemset(recv[b], 0x5a, n * 4));
    }
    if (la_allreduce_emulated_out_of_place(oop, send.data(), recv.data(), n, LA_I32, LA_SUM, nullptr) != LA_OK) {
        std::printf("out of place: %s\n", la_last_error());
        return 4;
    }
    HIP_OK(hipDeviceSynchronize());
    for (int b = 0; b < B; ++b) {
        HIP_OK(hipMemcpy(tmp.data(), recv[b], n * 4, hipMemcpyDeviceToHost));
        if (tmp != want) return 5;
        HIP_OK(hipMemcpy(tmp.data(), send[b], n * 4, hipMemcpyDeviceToHost));
        for (size_t i = 0; i < n; ++i)
            if (tmp[i] != value(b, i)) return 6; // the send buffers are never written
    }
    // refused: the wrong entry point for the schedule, a NULL buffer, one pointer twice, n that differs from the schedule's
    if (la_allreduce_emulated(oop, recv.data(), n, LA_I32, LA_SUM, nullptr) != LA_ERR_INVALID_ARG) return 7;
    std::vector<void*> bad = recv;
    bad[3] = nullptr;
    if (la_allreduce_emulated(in_place, bad.data(), n, LA_I32, LA_SUM, nullptr) != LA_ERR_INVALID_ARG) return 8;
    bad = recv;
    bad[5] = bad[2];
    if (la_allreduce_emulated(in_place, bad.data(), n, LA_I32, LA_SUM, nullptr) != LA_ERR_INVALID_ARG) return 9;
    if (la_allreduce_emulated(in_place, recv.data(), n + 1, LA_I32, LA_SUM, nullptr) != LA_ERR_INVALID_ARG) return 10;
    if (la_allreduce_emulated(in_place, recv.data(), n, LA_F32, LA_SUM, nullptr) != LA_ERR_INVALID_ARG) return 11;
    if (la_allreduce_emulated(in_place, recv.data(), n, LA_I32, (la_op_t)9, nullptr) != LA_ERR_UNSUPPORTED) return 12;
    if (la_last_error()[0] == 0) return 13;
    HIP_OK(hipDeviceSynchronize());
    for (int b = 0; b < B; ++b) { // the refused calls enqueued nothing
        HIP_OK(hipMemcpy(tmp.data(), recv[b], n * 4, hipMemcpyDeviceToHost));
        if (tmp != want) return 14;
        HIP_OK(hipFree(send[b]));
        HIP_OK(hipFree(recv[b]));
    }
    la_schedule_destroy(oop);
    la_schedule_destroy(in_place);
    la_topology_destroy(topo);
    return 0;
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
    struct TableCase {
        int nodes, gpus, procs;
        la_algo_t algo;
        unsigned flags;
        size_t n;
        la_op_t op;
    };
    const TableCase table_cases[] = {
        {2, 2, 2, LA_ALGO_LANE_MULTIPROC, LA_SCHED_DEFAULT, 10007, LA_SUM},
        {3, 2, 1, LA_ALGO_RING, LA_SCHED_DEFAULT, 5003, LA_MAX},
        {3, 2, 2, LA_ALGO_LANE, LA_SCHED_INNER_RING | LA_SCHED_P2P_GATHER, 7001, LA_SUM},
    };
    for (const TableCase& c : table_cases) {
        const int rc = steps_from_tables(c.nodes, c.gpus, c.procs, c.algo, c.flags, c.n, c.op);
        std::printf("tables %dx%dx%d algo %d flags %u n %zu op %d: %s\n", c.nodes, c.gpus, c.procs, (int)c.algo, c.flags, c.n,
                    (int)c.op, rc == 0 ? "ok" : "FAILED");
        std::fflush(stdout);
        if (rc) return 100 + rc;
    }
    int rc = reduce_segments();
    std::printf("reduce_segments and reduce_segments_static: %s\n", rc == 0 ? "ok" : "FAILED");
    if (rc) return 200 + rc;
    rc = out_of_place_and_errors();
    std::printf("out-of-place entry point and refused arguments: %s\n", rc == 0 ? "ok" : "FAILED");
    if (rc) return 300 + rc;
    std::printf("all ok\n");
    return 0;
}
