// Column analysis of a schedule: which element ranges never exchange data, and the ordered list of
// (step, segment) pairs that work on each of them.  Host code only.
//
// Algorithms 1 and 2 (and recursive halving / doubling) move and add chunks that sit at the same
// element offset in every rank's buffer: a message carries elements [a, b) of the sender to
// elements [a, b) of the receiver.  So the whole all-reduce is a column-wise computation, and the
// dependencies between its steps run along columns only.  Cutting the element axis at every offset
// where a segment of any step of a run starts or ends gives ranges ("chains") on which every step
// either acts as a whole or not at all; a chain's operations, taken in step order, depend on
// nothing outside the chain.  For Algorithm 1 over P ranks the chains are its P chunks, each with
// 2(P - 1) operations: chunk c travelling round the ring.
#include <algorithm>
#include <new>

#include "la_internal.hpp"

namespace la {

namespace {

constexpr uint64_t MAX_FUSED_OPS = 16ull << 20; // 64 bytes each on the device

// A step that can be part of a run: every operand of a segment at the segment's one offset, none in
// the staging area (staged exchanges pack to other offsets), at most two sources and destinations.
bool narrow_step(const la_schedule& s, const Step& p)
{
    if (p.k > FUSED_MAX_FAN || p.m > FUSED_MAX_FAN || p.k < 1 || p.m < 1) return false;
    if (p.group > 0 && p.group < p.k) return false;
    const size_t S = p.num_segments();
    if (S == 0) return false;
    for (size_t g = 0; g < S; ++g) {
        const uint64_t off = p.dst[g * p.m].off;
        for (int t = 0; t < p.k; ++t)
            if (p.src[g * p.k + t].off != off || p.src[g * p.k + t].buf == s.nbuf) return false;
        for (int d = 0; d < p.m; ++d)
            if (p.dst[g * p.m + d].off != off || p.dst[g * p.m + d].buf == s.nbuf) return false;
    }
    return true;
}

// Chains and operations of steps [first, first + count); false if there are too many operations.
bool analyse_run(const la_schedule& s, int first, int count, FusionRun& f)
{
    f.first_step = first;
    f.num_steps = count;
    std::vector<uint64_t> cut;
    for (int i = first; i < first + count; ++i) {
        const Step& p = s.steps[i];
        for (size_t g = 0; g < p.num_segments(); ++g) {
            cut.push_back(p.dst[g * p.m].off);
            cut.push_back(p.dst[g * p.m].off + p.len[g]);
        }
    }
    std::sort(cut.begin(), cut.end());
    cut.erase(std::unique(cut.begin(), cut.end()), cut.end());
    if (cut.size() < 2) return false;
    const size_t R = cut.size() - 1; // candidate ranges [cut[r], cut[r + 1])
    std::vector<uint64_t> count_of(R + 1, 0);
    uint64_t total = 0;
    for (int i = first; i < first + count; ++i) {
        const Step& p = s.steps[i];
        for (size_t g = 0; g < p.num_segments(); ++g) {
            const uint64_t lo = p.dst[g * p.m].off, hi = lo + p.len[g];
            size_t r = std::lower_bound(cut.begin(), cut.end(), lo) - cut.begin();
            for (; r < R && cut[r] < hi; ++r) {
                ++count_of[r];
                if (++total > MAX_FUSED_OPS) return false;
            }
        }
    }
    std::vector<uint64_t> fill(R + 1, 0);
    for (size_t r = 0; r < R; ++r) fill[r + 1] = fill[r] + count_of[r];
    f.op_step.assign(total, 0);
    f.op_seg.assign(total, 0);
    for (int i = first; i < first + count; ++i) {
        const Step& p = s.steps[i];
        for (size_t g = 0; g < p.num_segments(); ++g) {
            const uint64_t lo = p.dst[g * p.m].off, hi = lo + p.len[g];
            size_t r = std::lower_bound(cut.begin(), cut.end(), lo) - cut.begin();
            for (; r < R && cut[r] < hi; ++r) {
                f.op_step[fill[r]] = (uint32_t)i;
                f.op_seg[fill[r]] = (uint32_t)g;
                ++fill[r];
            }
        }
    }
    // chains: the ranges some segment covers (an empty range holds no op, so the ops stay contiguous)
    f.chain_first.assign(1, 0);
    for (size_t r = 0; r < R; ++r) {
        if (count_of[r] == 0) continue;
        f.chain_lo.push_back(cut[r]);
        f.chain_len.push_back(cut[r + 1] - cut[r]);
        f.chain_first.push_back(f.chain_first.back() + count_of[r]);
    }
    // per op: which sources are original inputs of the chain (never written by an earlier op of it),
    // which one is what the previous op stored
    f.op_prefetch.assign(total, -1);
    f.op_forward.assign(total, -1);
    f.max_chain_ops = 0;
    const size_t bufs = 2 * (size_t)s.nbuf + 2;
    std::vector<uint64_t> written_by(bufs, 0); // chain number + 1 of the last chain that wrote the buffer's range
    const size_t C = f.chain_lo.size();
    for (size_t c = 0; c < C; ++c) {
        f.max_chain_ops = std::max(f.max_chain_ops, f.chain_first[c + 1] - f.chain_first[c]);
        for (uint64_t o = f.chain_first[c]; o < f.chain_first[c + 1]; ++o) {
            const Step& p = s.steps[f.op_step[o]];
            const size_t g = f.op_seg[o];
            int pf = -1;
            for (int t = 0; t < p.k && pf < 0; ++t)
                if (written_by[p.src[g * p.k + t].buf] != c + 1) pf = t;
            f.op_prefetch[o] = pf;
            if (o > f.chain_first[c]) {
                const Step& q = s.steps[f.op_step[o - 1]];
                const size_t h = f.op_seg[o - 1];
                for (int t = 0; t < p.k && f.op_forward[o] < 0; ++t)
                    for (int d = 0; d < q.m; ++d)
                        if (q.dst[h * q.m + d].buf == p.src[g * p.k + t].buf) f.op_forward[o] = t;
            }
            for (int d = 0; d < p.m; ++d) written_by[p.dst[g * p.m + d].buf] = c + 1;
        }
    }
    return C > 0;
}

} // namespace

void analyse_fusion(const la_schedule& s)
{
    FusionPlan& f = s.fusion;
    if (f.analysed) return;
    f.runs.clear();
    const int n = (int)s.steps.size();
    for (int i = 0; i < n;) {
        if (!narrow_step(s, s.steps[i])) {
            ++i;
            continue;
        }
        int j = i;
        while (j < n && narrow_step(s, s.steps[j])) ++j;
        if (j - i >= 2) {
            FusionRun run;
            if (analyse_run(s, i, j - i, run)) f.runs.push_back(std::move(run));
        }
        i = j;
    }
    f.analysed = true;
}

} // namespace la

using namespace la;

extern "C" {

int la_schedule_fusion_runs(const la_schedule_t* sched)
{
    if (!sched) return -1;
    try {
        std::lock_guard<std::mutex> lock(sched->mu);
        analyse_fusion(*sched);
    } catch (const std::bad_alloc&) {
        sched->fusion = FusionPlan();
        (void)fail(LA_ERR_OUT_OF_MEMORY, "la_schedule_fusion_runs: out of host memory");
        return -1;
    }
    return (int)sched->fusion.runs.size();
}

la_status_t la_schedule_fusion_info(const la_schedule_t* sched, int run, int* first_step, int* num_steps,
                                    uint64_t* num_chains, uint64_t* num_ops, int* automatic, size_t* bytes_read,
                                    size_t* bytes_written)
{
    if (!sched) return fail(LA_ERR_INVALID_ARG, "la_schedule_fusion_info: schedule is NULL");
    const int runs = la_schedule_fusion_runs(sched);
    if (runs < 0) return LA_ERR_OUT_OF_MEMORY;
    if (run < 0 || run >= runs) return fail(LA_ERR_INVALID_ARG, "la_schedule_fusion_info: run %d out of range (%d runs)", run, runs);
    const FusionRun& f = sched->fusion.runs[run];
    if (first_step) *first_step = f.first_step;
    if (num_steps) *num_steps = f.num_steps;
    if (num_chains) *num_chains = f.chain_lo.size();
    if (num_ops) *num_ops = f.op_step.size();
    if (automatic) *automatic = f.automatic() ? 1 : 0;
    if (bytes_read || bytes_written) {
        // what the fused launch moves: every destination is stored; a source is loaded unless it is
        // taken from the registers of the lane that has just stored it
        const bool forward = current_tuning().forward != 0;
        const uint64_t e = dtype_size(sched->dtype);
        uint64_t rd = 0, wr = 0;
        for (size_t c = 0; c < f.chain_lo.size(); ++c)
            for (uint64_t o = f.chain_first[c]; o < f.chain_first[c + 1]; ++o) {
                const Step& p = sched->steps[f.op_step[o]];
                rd += f.chain_len[c] * e * (uint64_t)(p.k - (forward && f.op_forward[o] >= 0 ? 1 : 0));
                wr += f.chain_len[c] * e * (uint64_t)p.m;
            }
        if (bytes_read) *bytes_read = (size_t)rd;
        if (bytes_written) *bytes_written = (size_t)wr;
    }
    return LA_OK;
}

la_status_t la_schedule_fusion_table(const la_schedule_t* sched, int run, uint64_t* chain_lo, uint64_t* chain_len,
                                     uint64_t* chain_first_op, uint32_t* op_step, uint32_t* op_segment,
                                     int32_t* op_prefetch_source, int32_t* op_forward_source)
{
    const la_status_t st = la_schedule_fusion_info(sched, run, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr);
    if (st != LA_OK) return st;
    const FusionRun& f = sched->fusion.runs[run];
    if (chain_lo) std::copy(f.chain_lo.begin(), f.chain_lo.end(), chain_lo);
    if (chain_len) std::copy(f.chain_len.begin(), f.chain_len.end(), chain_len);
    if (chain_first_op) std::copy(f.chain_first.begin(), f.chain_first.end(), chain_first_op);
    if (op_step) std::copy(f.op_step.begin(), f.op_step.end(), op_step);
    if (op_segment) std::copy(f.op_seg.begin(), f.op_seg.end(), op_segment);
    if (op_prefetch_source) std::copy(f.op_prefetch.begin(), f.op_prefetch.end(), op_prefetch_source);
    if (op_forward_source) std::copy(f.op_forward.begin(), f.op_forward.end(), op_forward_source);
    return LA_OK;
}

} // extern "C"
