// Topology and schedule generator: turns (nodes, GPUs per node, processes per GPU) into the
// per-step segment tables of Algorithm 1 (ring_allreduce) and Algorithm 2 (lane_allreduce, also
// in its multiple-processes-per-GPU form), of the shared-buffer model's standard and multi-lane
// approaches, and of recursive doubling and Rabenseifner's algorithm (Background section); plus
// the passes that derive the staged, out-of-place, stand-alone-half and fused forms.  Host code only.
#include <algorithm>
#include <cstdio>
#include <cstring>
#include <new>

#include "la_internal.hpp"

namespace la {

static thread_local char g_err[512] = "";

la_status_t fail(la_status_t st, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return st;
}

namespace {

inline int imod(int a, int m)
{
    const int r = a % m;
    return r < 0 ? r + m : r;
}

// Sequential allocator of staging slots (elements).
struct Staging {
    uint64_t next = 0, peak = 0;
    uint64_t take(uint64_t cnt)
    {
        const uint64_t at = next;
        next += (cnt + 63) & ~uint64_t(63); // keep slots 16-byte aligned for every dtype
        peak = std::max(peak, next);
        return at;
    }
    void reset() { next = 0; }
};

// A reduce whose operands are `ops` (in summation order) into `dst`; with LA_SCHED_STAGED the
// operands that are not already in the destination's own buffer are first copied to staging.
struct ReduceBuilder {
    const la_schedule& s;
    Step pack, red;
    Staging& st;
    bool staged;
    int P;
    ReduceBuilder(const la_schedule& sc, Staging& stg, int stage, int k, int m) : s(sc), st(stg)
    {
        staged = (sc.flags & LA_SCHED_STAGED) != 0;
        P = sc.nbuf;
        pack.kind = LA_STEP_COPY;
        pack.stage = LA_STAGE_PACK;
        pack.k = 1;
        pack.m = 1;
        red.kind = LA_STEP_REDUCE;
        red.stage = stage;
        red.k = k;
        red.m = m;
    }
    // ops.size() == k, dsts.size() == m; `home` is the rank that performs the reduction
    void add(uint64_t len, const std::vector<Operand>& ops, const std::vector<Operand>& dsts, int home)
    {
        if (len == 0) return;
        red.len.push_back(len);
        for (const Operand& o : ops) {
            if (staged && o.buf != home) {
                const uint64_t slot = st.take(len);
                pack.len.push_back(len);
                pack.src.push_back(o);
                pack.dst.push_back(Operand{P, slot});
                red.src.push_back(Operand{P, slot});
            } else {
                red.src.push_back(o);
            }
        }
        for (const Operand& d : dsts) red.dst.push_back(d);
    }
    void emit(std::vector<Step>& out)
    {
        if (red.len.empty()) return;
        if (staged && !pack.len.empty()) out.push_back(std::move(pack));
        out.push_back(std::move(red));
        st.reset(); // the next reduce step may reuse the staging area
    }
};

void push_copy(Step& c, uint64_t len, Operand from, Operand to)
{
    if (len == 0) return;
    c.len.push_back(len);
    c.src.push_back(from);
    c.dst.push_back(to);
}

// ---- Algorithm 1 ---------------------------------------------------------------------------
// Chunk c starts at rank c and travels to c+1, c+2, ...  In reduce iteration i rank r receives
// chunk rp = r-1-i from its predecessor and adds it to its own copy; in gather iteration i it
// receives the finished chunk r-i.  One launch holds the P segments of an iteration.
void gen_ring(la_schedule& s, Staging& st)
{
    const int P = s.topo.ranks();
    std::vector<Part> chunk(P);
    for (int c = 0; c < P; ++c) chunk[c] = split_part(s.n, P, c);
    for (int r = 0; r < P; ++r) s.owned[r].push_back(chunk[(r + 1) % P]); // after the first loop
    for (int i = 0; i < P - 1; ++i) {
        ReduceBuilder rb(s, st, LA_STAGE_RING_RS, 2, 1);
        for (int r = 0; r < P; ++r) {
            const Part c = chunk[imod(r - 1 - i, P)];
            const int prev = imod(r - 1, P);
            rb.add(c.cnt, {Operand{r, c.off}, Operand{prev, c.off}}, {Operand{r, c.off}}, r);
        }
        rb.emit(s.steps);
    }
    for (int i = 0; i < P - 1; ++i) {
        Step cp;
        cp.kind = LA_STEP_COPY;
        cp.stage = LA_STAGE_RING_AG;
        cp.k = cp.m = 1;
        for (int r = 0; r < P; ++r) {
            const Part c = chunk[imod(r - i, P)];
            push_copy(cp, c.cnt, Operand{imod(r - 1, P), c.off}, Operand{r, c.off});
        }
        if (!cp.len.empty()) s.steps.push_back(std::move(cp));
    }
}

// ---- Background section: recursive doubling and Rabenseifner's algorithm ------------------------
// Both are flat over the P ranks and need P to be a power of two.

int log2_exact(int P)
{
    int L = 0;
    while ((1 << L) < P) ++L;
    return (1 << L) == P ? L : -1;
}

// Recursive doubling: in round s the ranks that differ in bit s exchange their whole buffers and
// each adds the other's to its own.  The two sums of a pair are the same value (the operations
// are commutative), so one segment computes it once and stores it to both buffers.
void gen_recursive_doubling(la_schedule& s, Staging& st, int L)
{
    const int P = s.topo.ranks();
    for (int b = 0; b < L; ++b) {
        ReduceBuilder rb(s, st, LA_STAGE_RECURSIVE_DOUBLING, 2, 2);
        for (int r = 0; r < P; ++r) {
            if (r & (1 << b)) continue;
            const int partner = r | (1 << b);
            rb.add(s.n, {Operand{r, 0}, Operand{partner, 0}}, {Operand{r, 0}, Operand{partner, 0}}, r);
        }
        rb.emit(s.steps);
    }
}

// Rabenseifner: reduce-scatter by recursive halving (partners at distance P/2, P/4, ..., 1; the
// lower rank of a pair keeps the first half of the pair's current range, the upper rank the
// second, and each adds the partner's copy of the half it keeps), then an all-gather by recursive
// doubling over the same ranges in reverse.
void gen_rabenseifner(la_schedule& s, Staging& st, int L)
{
    const int P = s.topo.ranks();
    // range[r][lvl]: what rank r works on before halving round lvl; range[r][L] is what it owns
    std::vector<std::vector<Part>> range(P, std::vector<Part>(L + 1));
    for (int r = 0; r < P; ++r) {
        range[r][0] = Part{0, s.n};
        for (int lvl = 0; lvl < L; ++lvl) {
            const int d = P >> (lvl + 1);
            const Part half = split_part(range[r][lvl].cnt, 2, (r & d) ? 1 : 0);
            range[r][lvl + 1] = Part{range[r][lvl].off + half.off, half.cnt};
        }
    }
    for (int r = 0; r < P; ++r) s.owned[r].push_back(range[r][L]);
    for (int lvl = 0; lvl < L; ++lvl) {
        const int d = P >> (lvl + 1);
        ReduceBuilder rb(s, st, LA_STAGE_RABENSEIFNER_RS, 2, 1);
        for (int r = 0; r < P; ++r) {
            const Part keep = range[r][lvl + 1];
            rb.add(keep.cnt, {Operand{r, keep.off}, Operand{r ^ d, keep.off}}, {Operand{r, keep.off}}, r);
        }
        rb.emit(s.steps);
    }
    for (int lvl = L - 1; lvl >= 0; --lvl) {
        const int d = P >> (lvl + 1);
        Step cp;
        cp.kind = LA_STEP_COPY;
        cp.stage = LA_STAGE_RABENSEIFNER_AG;
        cp.k = cp.m = 1;
        for (int r = 0; r < P; ++r) {
            const Part have = range[r ^ d][lvl + 1]; // what the partner holds complete
            push_copy(cp, have.cnt, Operand{r ^ d, have.off}, Operand{r, have.off});
        }
        if (!cp.len.empty()) s.steps.push_back(std::move(cp));
    }
}

// ---- Algorithm 2 ---------------------------------------------------------------------------
// The buffer is cut into J parts: one lane per GPU, and with the per-process split one
// sub-chunk per process inside each lane.  Part j is owned, on every node, by the process with
// node-local index owner(j).
void gen_lane(la_schedule& s, Staging& st, bool split_procs)
{
    const la_topology& t = s.topo;
    const int N = t.nodes, G = t.gpus, Q = t.procs, R = G * Q;
    const int J = split_procs ? R : G;
    const bool p2p = (s.flags & LA_SCHED_P2P_GATHER) != 0;
    // a stand-alone half needs the inter-node all-reduce as two launches (reduce-scatter, all-gather)
    const bool split = p2p || (s.flags & (LA_SCHED_ONLY_REDUCE_SCATTER | LA_SCHED_ONLY_ALLGATHER)) != 0;
    auto owner = [&](int j) { return split_procs ? j : j * Q; };
    std::vector<Part> part(J);
    for (int j = 0; j < J; ++j) {
        if (!split_procs) {
            part[j] = split_part(s.n, G, j);
        } else {
            const Part lane = split_part(s.n, G, j / Q);
            const Part sub = split_part(lane.cnt, Q, j % Q);
            part[j] = Part{lane.off + sub.off, sub.cnt};
        }
    }

    const bool inner_ring = (s.flags & LA_SCHED_INNER_RING) != 0;
    // what a rank holds fully reduced between the two halves: piece `node` of the part it owns
    for (int node = 0; node < N; ++node)
        for (int j = 0; j < J; ++j) {
            // (the ring form of stage 2 leaves member v with piece v+1, as Algorithm 1 does)
            const Part piece = split_part(part[j].cnt, N, inner_ring ? (node + 1) % N : node);
            s.owned[t.rank_of(node, owner(j))].push_back(Part{part[j].off + piece.off, piece.cnt});
        }

    // S1: reduce-scatter on the node group; the owner adds the R node-local copies of its part
    // in ascending node-local index (its own copy taking its place in that order).
    // LA_SCHED_SINGLE_LAUNCH: S1, S2 and S3 as one two-level reduce.  Piece v of part j is the sum
    // over the nodes, in ascending order, of each node's sum over its R ranks in ascending
    // node-local index, the node sums rounded to the element type as S1 stores them; it is stored
    // to every rank.  Every input is read once and every output written once.
    if (s.flags & LA_SCHED_SINGLE_LAUNCH) {
        Step all;
        all.kind = LA_STEP_REDUCE;
        all.stage = LA_STAGE_S1_S2_S3;
        all.k = all.m = N * R;
        all.group = (N > 1 && R > 1) ? R : 0;
        if (N * R == 1) return;
        for (int j = 0; j < J; ++j)
            for (int v = 0; v < N; ++v) {
                const Part piece = split_part(part[j].cnt, N, v);
                if (piece.cnt == 0) continue;
                const uint64_t off = part[j].off + piece.off;
                all.len.push_back(piece.cnt);
                for (int w = 0; w < N; ++w)
                    for (int l = 0; l < R; ++l) all.src.push_back(Operand{t.rank_of(w, l), off});
                const int me = t.rank_of(v, owner(j));
                all.dst.push_back(Operand{me, off}); // the rank that reduces the piece in Algorithm 2 first
                for (int w = 0; w < N; ++w)
                    for (int l = 0; l < R; ++l)
                        if (t.rank_of(w, l) != me) all.dst.push_back(Operand{t.rank_of(w, l), off});
            }
        if (!all.len.empty()) s.steps.push_back(std::move(all));
        return;
    }

    // LA_SCHED_FUSED_GATHER: the last reduce of a part stores to every rank that the all-gathers
    // would have copied it to, and the all-gather launches disappear.
    const bool fused = (s.flags & LA_SCHED_FUSED_GATHER) != 0;
    const bool s1_is_last = fused && N == 1;
    if (R > 1) {
        ReduceBuilder rb(s, st, s1_is_last ? LA_STAGE_S1_S3 : LA_STAGE_S1, R, s1_is_last ? R : 1);
        for (int node = 0; node < N; ++node)
            for (int j = 0; j < J; ++j) {
                std::vector<Operand> ops(R), dsts;
                for (int l = 0; l < R; ++l) ops[l] = Operand{t.rank_of(node, l), part[j].off};
                const int me = t.rank_of(node, owner(j));
                dsts.push_back(Operand{me, part[j].off});
                if (s1_is_last)
                    for (int l = 0; l < R; ++l)
                        if (l != owner(j)) dsts.push_back(Operand{t.rank_of(node, l), part[j].off});
                rb.add(part[j].cnt, ops, dsts, me);
            }
        rb.emit(s.steps);
    }

    // S2, ring form (LA_SCHED_INNER_RING): Algorithm 1 on every lane communicator at once.  The
    // part is cut into N pieces and member v plays rank v of a ring of N; one launch holds one
    // ring iteration of all J lane communicators.
    if (N > 1 && inner_ring) {
        for (int i = 0; i < N - 1; ++i) {
            ReduceBuilder rb(s, st, LA_STAGE_S2_RING_RS, 2, 1);
            for (int j = 0; j < J; ++j)
                for (int v = 0; v < N; ++v) {
                    const Part piece = split_part(part[j].cnt, N, imod(v - 1 - i, N));
                    const uint64_t off = part[j].off + piece.off;
                    const int me = t.rank_of(v, owner(j)), prev = t.rank_of(imod(v - 1, N), owner(j));
                    rb.add(piece.cnt, {Operand{me, off}, Operand{prev, off}}, {Operand{me, off}}, me);
                }
            rb.emit(s.steps);
        }
        for (int i = 0; i < N - 1; ++i) {
            Step cp;
            cp.kind = LA_STEP_COPY;
            cp.stage = LA_STAGE_S2_RING_AG;
            cp.k = cp.m = 1;
            for (int j = 0; j < J; ++j)
                for (int v = 0; v < N; ++v) {
                    const Part piece = split_part(part[j].cnt, N, imod(v - i, N));
                    const uint64_t off = part[j].off + piece.off;
                    push_copy(cp, piece.cnt, Operand{t.rank_of(imod(v - 1, N), owner(j)), off},
                              Operand{t.rank_of(v, owner(j)), off});
                }
            if (!cp.len.empty()) s.steps.push_back(std::move(cp));
        }
    }

    // S2: all-reduce of part j among its N owners (the lane communicator): member v reduces
    // piece v of the part over the N members in ascending node order, then every member gets
    // every piece.
    if (N > 1 && !inner_ring) {
        ReduceBuilder rb(s, st, fused ? LA_STAGE_S2_S3 : split ? LA_STAGE_S2A : LA_STAGE_S2, N,
                         fused ? N * R : split ? 1 : N);
        Step ag;
        ag.kind = LA_STEP_COPY;
        ag.stage = LA_STAGE_S2B;
        ag.k = 1;
        ag.m = p2p ? 1 : N - 1;
        for (int j = 0; j < J; ++j)
            for (int v = 0; v < N; ++v) {
                const Part piece = split_part(part[j].cnt, N, v);
                const uint64_t off = part[j].off + piece.off;
                std::vector<Operand> ops(N), dsts;
                for (int w = 0; w < N; ++w) ops[w] = Operand{t.rank_of(w, owner(j)), off};
                const int me = t.rank_of(v, owner(j));
                dsts.push_back(Operand{me, off});
                if (fused) { // every rank of every node, the reducing member first
                    for (int w = 0; w < N; ++w)
                        for (int l = 0; l < R; ++l)
                            if (t.rank_of(w, l) != me) dsts.push_back(Operand{t.rank_of(w, l), off});
                    rb.add(piece.cnt, ops, dsts, me);
                    continue;
                }
                if (split && !p2p && piece.cnt > 0) {
                    ag.len.push_back(piece.cnt);
                    ag.src.push_back(Operand{me, off});
                }
                for (int w = 0; w < N; ++w) {
                    if (w == v) continue;
                    const Operand to{t.rank_of(w, owner(j)), off};
                    if (p2p)
                        push_copy(ag, piece.cnt, Operand{me, off}, to);
                    else if (split) {
                        if (piece.cnt > 0) ag.dst.push_back(to);
                    } else
                        dsts.push_back(to);
                }
                rb.add(piece.cnt, ops, dsts, me);
            }
        rb.emit(s.steps);
        if (split && !ag.len.empty()) s.steps.push_back(std::move(ag));
    }

    // S3: all-gather on the node group: every owner's part goes to the other R-1 processes.
    if (R > 1 && !fused) {
        Step ag;
        ag.kind = LA_STEP_COPY;
        ag.stage = LA_STAGE_S3;
        ag.k = 1;
        ag.m = p2p ? 1 : R - 1;
        for (int node = 0; node < N; ++node)
            for (int j = 0; j < J; ++j) {
                if (part[j].cnt == 0) continue;
                const Operand from{t.rank_of(node, owner(j)), part[j].off};
                if (!p2p) {
                    ag.len.push_back(part[j].cnt);
                    ag.src.push_back(from);
                }
                for (int l = 0; l < R; ++l) {
                    if (l == owner(j)) continue;
                    const Operand to{t.rank_of(node, l), part[j].off};
                    if (p2p)
                        push_copy(ag, part[j].cnt, from, to);
                    else
                        ag.dst.push_back(to);
                }
            }
        if (!ag.len.empty()) s.steps.push_back(std::move(ag));
    }
}

// ---- the shared-buffer model -------------------------------------------------------------------
// One buffer per GPU (index node*G + gpu); the Q processes of a GPU work on it, process q on part q
// of a balanced split of n into Q ("Multiple Processes Per GPU": the slice at (s/PPG) * l_r).

// "Standard Approach": Q concurrent all-reduces, one per local rank, each over the N*G processes
// with that local rank (new_comm), each taken to be Algorithm 1.  One launch holds one iteration
// of all Q rings: the message count grows by Q and the message size shrinks by Q.
void gen_shared_standard(la_schedule& s, Staging& st)
{
    const int M = s.topo.nodes * s.topo.gpus, Q = s.topo.procs;
    auto chunk = [&](int q, int c) {
        const Part slice = split_part(s.n, Q, q);
        const Part ch = split_part(slice.cnt, M, c);
        return Part{slice.off + ch.off, ch.cnt};
    };
    for (int u = 0; u < M; ++u)
        for (int q = 0; q < Q; ++q) s.owned[u].push_back(chunk(q, (u + 1) % M));
    for (int i = 0; i < M - 1; ++i) {
        ReduceBuilder rb(s, st, LA_STAGE_RING_RS, 2, 1);
        for (int q = 0; q < Q; ++q)
            for (int u = 0; u < M; ++u) {
                const Part c = chunk(q, imod(u - 1 - i, M));
                rb.add(c.cnt, {Operand{u, c.off}, Operand{imod(u - 1, M), c.off}}, {Operand{u, c.off}}, u);
            }
        rb.emit(s.steps);
    }
    for (int i = 0; i < M - 1; ++i) {
        Step cp;
        cp.kind = LA_STEP_COPY;
        cp.stage = LA_STAGE_RING_AG;
        cp.k = cp.m = 1;
        for (int q = 0; q < Q; ++q)
            for (int u = 0; u < M; ++u) {
                const Part c = chunk(q, imod(u - i, M));
                push_copy(cp, c.cnt, Operand{imod(u - 1, M), c.off}, Operand{u, c.off});
            }
        if (!cp.len.empty()) s.steps.push_back(std::move(cp));
    }
}

// "Multi-lane Approach": every process runs Algorithm 2 on its slice; comm_group = the G
// processes with local rank q on the node, comm_lane = the N processes (node', gpu, q).
void gen_shared_lane(la_schedule& s, Staging& st, int Q)
{
    const la_topology& t = s.topo;
    const int N = t.nodes, G = t.gpus;
    const bool p2p = (s.flags & LA_SCHED_P2P_GATHER) != 0;
    const bool split = p2p || (s.flags & (LA_SCHED_ONLY_REDUCE_SCATTER | LA_SCHED_ONLY_ALLGATHER)) != 0;
    auto buf = [&](int node, int g) { return node * G + g; };
    auto chunk = [&](int q, int g) {
        const Part slice = split_part(s.n, Q, q);
        const Part ch = split_part(slice.cnt, G, g);
        return Part{slice.off + ch.off, ch.cnt};
    };
    for (int q = 0; q < Q; ++q)
        for (int g = 0; g < G; ++g)
            for (int v = 0; v < N; ++v) {
                const Part c = chunk(q, g);
                const Part piece = split_part(c.cnt, N, v);
                s.owned[buf(v, g)].push_back(Part{c.off + piece.off, piece.cnt});
            }
    if (s.flags & LA_SCHED_SINGLE_LAUNCH) { // see gen_lane
        Step all;
        all.kind = LA_STEP_REDUCE;
        all.stage = LA_STAGE_S1_S2_S3;
        all.k = all.m = N * G;
        all.group = (N > 1 && G > 1) ? G : 0;
        if (N * G == 1) return;
        for (int q = 0; q < Q; ++q)
            for (int g = 0; g < G; ++g)
                for (int v = 0; v < N; ++v) {
                    const Part c = chunk(q, g);
                    const Part piece = split_part(c.cnt, N, v);
                    if (piece.cnt == 0) continue;
                    const uint64_t off = c.off + piece.off;
                    all.len.push_back(piece.cnt);
                    for (int w = 0; w < N; ++w)
                        for (int h = 0; h < G; ++h) all.src.push_back(Operand{buf(w, h), off});
                    all.dst.push_back(Operand{buf(v, g), off});
                    for (int w = 0; w < N; ++w)
                        for (int h = 0; h < G; ++h)
                            if (buf(w, h) != buf(v, g)) all.dst.push_back(Operand{buf(w, h), off});
                }
        if (!all.len.empty()) s.steps.push_back(std::move(all));
        return;
    }
    const bool fused = (s.flags & LA_SCHED_FUSED_GATHER) != 0;
    const bool s1_is_last = fused && N == 1;
    if (G > 1) {
        ReduceBuilder rb(s, st, s1_is_last ? LA_STAGE_S1_S3 : LA_STAGE_S1, G, s1_is_last ? G : 1);
        for (int node = 0; node < N; ++node)
            for (int q = 0; q < Q; ++q)
                for (int g = 0; g < G; ++g) {
                    const Part c = chunk(q, g);
                    std::vector<Operand> ops(G), dsts;
                    for (int h = 0; h < G; ++h) ops[h] = Operand{buf(node, h), c.off};
                    dsts.push_back(Operand{buf(node, g), c.off});
                    if (s1_is_last)
                        for (int h = 0; h < G; ++h)
                            if (h != g) dsts.push_back(Operand{buf(node, h), c.off});
                    rb.add(c.cnt, ops, dsts, buf(node, g));
                }
        rb.emit(s.steps);
    }
    if (N > 1) {
        ReduceBuilder rb(s, st, fused ? LA_STAGE_S2_S3 : split ? LA_STAGE_S2A : LA_STAGE_S2, N,
                         fused ? N * G : split ? 1 : N);
        Step ag;
        ag.kind = LA_STEP_COPY;
        ag.stage = LA_STAGE_S2B;
        ag.k = 1;
        ag.m = p2p ? 1 : N - 1;
        for (int q = 0; q < Q; ++q)
            for (int g = 0; g < G; ++g)
                for (int v = 0; v < N; ++v) {
                    const Part c = chunk(q, g);
                    const Part piece = split_part(c.cnt, N, v);
                    const uint64_t off = c.off + piece.off;
                    std::vector<Operand> ops(N), dsts;
                    for (int w = 0; w < N; ++w) ops[w] = Operand{buf(w, g), off};
                    dsts.push_back(Operand{buf(v, g), off});
                    if (fused) {
                        for (int w = 0; w < N; ++w)
                            for (int h = 0; h < G; ++h)
                                if (buf(w, h) != buf(v, g)) dsts.push_back(Operand{buf(w, h), off});
                        rb.add(piece.cnt, ops, dsts, buf(v, g));
                        continue;
                    }
                    if (split && !p2p && piece.cnt > 0) {
                        ag.len.push_back(piece.cnt);
                        ag.src.push_back(Operand{buf(v, g), off});
                    }
                    for (int w = 0; w < N; ++w) {
                        if (w == v) continue;
                        if (p2p)
                            push_copy(ag, piece.cnt, Operand{buf(v, g), off}, Operand{buf(w, g), off});
                        else if (split) {
                            if (piece.cnt > 0) ag.dst.push_back(Operand{buf(w, g), off});
                        } else
                            dsts.push_back(Operand{buf(w, g), off});
                    }
                    rb.add(piece.cnt, ops, dsts, buf(v, g));
                }
        rb.emit(s.steps);
        if (split && !ag.len.empty()) s.steps.push_back(std::move(ag));
    }
    if (G > 1 && !fused) {
        Step ag;
        ag.kind = LA_STEP_COPY;
        ag.stage = LA_STAGE_S3;
        ag.k = 1;
        ag.m = p2p ? 1 : G - 1;
        for (int node = 0; node < N; ++node)
            for (int q = 0; q < Q; ++q)
                for (int g = 0; g < G; ++g) {
                    const Part c = chunk(q, g);
                    if (c.cnt == 0) continue;
                    const Operand from{buf(node, g), c.off};
                    if (!p2p) {
                        ag.len.push_back(c.cnt);
                        ag.src.push_back(from);
                    }
                    for (int h = 0; h < G; ++h) {
                        if (h == g) continue;
                        if (p2p)
                            push_copy(ag, c.cnt, from, Operand{buf(node, h), c.off});
                        else
                            ag.dst.push_back(Operand{buf(node, h), c.off});
                    }
                }
        if (!ag.len.empty()) s.steps.push_back(std::move(ag));
    }
}

// LA_SCHED_STAGED in the shared model: every process first copies its slice of the shared buffer
// into a private staging slot, the all-reduce then runs on those private copies, and the result
// is copied back: the copy to and from a device buffer allocated by the calling process that the
// GPUDirect runs needed because the MPI library refused buffers shared through IPC.
void wrap_copy_in_out(la_schedule& s, Staging& st, int Q)
{
    const int M = s.nbuf;
    std::vector<Part> slice(Q);
    std::vector<uint64_t> slot((size_t)M * Q);
    for (int q = 0; q < Q; ++q) slice[q] = split_part(s.n, Q, q);
    Step in, out;
    in.kind = out.kind = LA_STEP_COPY;
    in.stage = out.stage = LA_STAGE_PACK;
    in.k = in.m = out.k = out.m = 1;
    for (int b = 0; b < M; ++b)
        for (int q = 0; q < Q; ++q) {
            slot[(size_t)b * Q + q] = st.take(slice[q].cnt);
            push_copy(in, slice[q].cnt, Operand{b, slice[q].off}, Operand{M, slot[(size_t)b * Q + q]});
            push_copy(out, slice[q].cnt, Operand{M, slot[(size_t)b * Q + q]}, Operand{b, slice[q].off});
        }
    auto to_private = [&](Operand& o) {
        int q = 0;
        while (q + 1 < Q && o.off >= slice[q].off + slice[q].cnt) ++q;
        o = Operand{M, slot[(size_t)o.buf * Q + q] + (o.off - slice[q].off)};
    };
    for (Step& p : s.steps) {
        for (Operand& o : p.src) to_private(o);
        for (Operand& o : p.dst) to_private(o);
    }
    if (!in.len.empty()) {
        s.steps.insert(s.steps.begin(), std::move(in));
        s.steps.push_back(std::move(out));
    }
}

// ---- out-of-place form ---------------------------------------------------------------------------
// Algorithm 1 is printed with separate send and receive buffers (buf_send, buf_recv, and
// buf_sendfrom switching from one to the other after the first iteration).  With
// LA_SCHED_OUT_OF_PLACE the caller passes both: a source range that no earlier step has written is
// an original input and is read from the send buffer (index nbuf + 1 + b in the tables); all
// stores go to the receive buffers, and the send buffers are never written.

struct Covered { // sorted, disjoint [lo, hi) ranges of one buffer that have been written
    std::vector<std::pair<uint64_t, uint64_t>> iv;
    // 1: fully written, 0: not written at all, -1: partly
    int query(uint64_t lo, uint64_t hi) const
    {
        uint64_t have = 0;
        for (const auto& r : iv) {
            const uint64_t a = std::max(lo, r.first), b = std::min(hi, r.second);
            if (a < b) have += b - a;
        }
        return have == hi - lo ? 1 : have == 0 ? 0 : -1;
    }
    void add(uint64_t lo, uint64_t hi)
    {
        std::vector<std::pair<uint64_t, uint64_t>> out;
        for (const auto& r : iv) {
            if (r.second < lo || r.first > hi) {
                out.push_back(r);
            } else {
                lo = std::min(lo, r.first);
                hi = std::max(hi, r.second);
            }
        }
        out.emplace_back(lo, hi);
        std::sort(out.begin(), out.end());
        iv.swap(out);
    }
};

la_status_t make_out_of_place(la_schedule& s)
{
    const int B = s.nbuf;
    std::vector<Covered> written(B);
    if (s.flags & LA_SCHED_ONLY_ALLGATHER) {
        // the all-gather half takes each rank's owned ranges from its send buffer: one launch
        // moves them into place, after which the half runs on the receive buffers alone
        Step in;
        in.kind = LA_STEP_COPY;
        in.stage = LA_STAGE_COPY_INPUT;
        in.k = in.m = 1;
        for (int b = 0; b < B; ++b)
            for (const Part& w : s.owned[b]) {
                push_copy(in, w.cnt, Operand{B + 1 + b, w.off}, Operand{b, w.off});
                if (w.cnt) written[b].add(w.off, w.off + w.cnt);
            }
        if (!in.len.empty()) s.steps.insert(s.steps.begin(), std::move(in));
    }
    for (Step& p : s.steps) {
        if (p.stage == LA_STAGE_COPY_INPUT) continue;
        const size_t S = p.num_segments();
        for (size_t g = 0; g < S; ++g)
            for (int t = 0; t < p.k; ++t) {
                Operand& o = p.src[g * p.k + t];
                if (o.buf >= B) continue; // staging is always written before it is read
                const int c = written[o.buf].query(o.off, o.off + p.len[g]);
                if (c < 0) return fail(LA_ERR_UNSUPPORTED, "out-of-place: a segment mixes original and reduced data");
                if (c == 0) o.buf = B + 1 + o.buf; // original input: from the send buffer
            }
        for (size_t g = 0; g < S; ++g)
            for (int d = 0; d < p.m; ++d) {
                const Operand& o = p.dst[g * p.m + d];
                if (o.buf < B) written[o.buf].add(o.off, o.off + p.len[g]);
            }
    }
    // whatever no step wrote (a single rank, a node of one rank, ...) is copied across
    Step cp;
    cp.kind = LA_STEP_COPY;
    cp.stage = LA_STAGE_COPY_INPUT;
    cp.k = cp.m = 1;
    const bool half = (s.flags & (LA_SCHED_ONLY_REDUCE_SCATTER | LA_SCHED_ONLY_ALLGATHER)) != 0;
    for (int b = 0; b < B; ++b) {
        // a stand-alone half defines the receive buffer only where the rank owns the result
        // (reduce-scatter) or everywhere (all-gather, whose launches write all but the owned ranges)
        std::vector<Part> want = half ? s.owned[b] : std::vector<Part>{Part{0, s.n}};
        for (const Part& w : want) {
            uint64_t at = w.off;
            const uint64_t end = w.off + w.cnt;
            for (const auto& r : written[b].iv) {
                if (r.second <= at) continue;
                if (r.first >= end) break;
                if (r.first > at) push_copy(cp, r.first - at, Operand{B + 1 + b, at}, Operand{b, at});
                at = r.second;
            }
            if (at < end) push_copy(cp, end - at, Operand{B + 1 + b, at}, Operand{b, at});
        }
    }
    if (!cp.len.empty()) s.steps.push_back(std::move(cp));
    return LA_OK;
}

} // namespace

la_status_t generate_steps(la_schedule& s)
{
    Staging st;
    s.owned.assign(s.nbuf, {});
    if ((s.flags & LA_SCHED_ONLY_REDUCE_SCATTER) && (s.flags & LA_SCHED_ONLY_ALLGATHER))
        return fail(LA_ERR_INVALID_ARG, "LA_SCHED_ONLY_REDUCE_SCATTER and LA_SCHED_ONLY_ALLGATHER exclude each other");
    if (s.flags & LA_SCHED_SINGLE_LAUNCH) {
        if (s.flags & (LA_SCHED_P2P_GATHER | LA_SCHED_INNER_RING | LA_SCHED_ONLY_REDUCE_SCATTER | LA_SCHED_ONLY_ALLGATHER |
                       LA_SCHED_FUSED_GATHER | LA_SCHED_STAGED))
            return fail(LA_ERR_INVALID_ARG, "LA_SCHED_SINGLE_LAUNCH combines only with LA_SCHED_SHARED_BUFFERS and LA_SCHED_OUT_OF_PLACE");
        if (s.algo != LA_ALGO_LANE && s.algo != LA_ALGO_LANE_MULTIPROC)
            return fail(LA_ERR_UNSUPPORTED, "LA_SCHED_SINGLE_LAUNCH applies to the lane schedules only");
    }
    if (s.flags & LA_SCHED_FUSED_GATHER) {
        if (s.flags & (LA_SCHED_P2P_GATHER | LA_SCHED_INNER_RING | LA_SCHED_ONLY_REDUCE_SCATTER | LA_SCHED_ONLY_ALLGATHER))
            return fail(LA_ERR_INVALID_ARG, "LA_SCHED_FUSED_GATHER excludes the point-to-point gather, the inner ring and the stand-alone halves");
        if (s.algo != LA_ALGO_LANE && s.algo != LA_ALGO_LANE_MULTIPROC)
            return fail(LA_ERR_UNSUPPORTED, "LA_SCHED_FUSED_GATHER applies to the lane schedules only");
    }
    if ((s.flags & (LA_SCHED_ONLY_REDUCE_SCATTER | LA_SCHED_ONLY_ALLGATHER)) &&
        (s.algo == LA_ALGO_RECURSIVE_DOUBLING ||
         ((s.flags & LA_SCHED_SHARED_BUFFERS) && (s.flags & LA_SCHED_STAGED))))
        return fail(LA_ERR_UNSUPPORTED, "this schedule has no reduce-scatter / all-gather halves");
    if (s.flags & LA_SCHED_SHARED_BUFFERS) {
        if (s.flags & LA_SCHED_INNER_RING)
            return fail(LA_ERR_UNSUPPORTED, "LA_SCHED_INNER_RING is not available with LA_SCHED_SHARED_BUFFERS");
        const unsigned staged = s.flags & LA_SCHED_STAGED;
        s.flags &= ~(unsigned)LA_SCHED_STAGED; // here staging means copy-in / copy-out, not per-message packs
        const int Q = s.algo == LA_ALGO_LANE ? 1 : s.topo.procs; // "lane": the leader handles the whole buffer
        switch (s.algo) {
        case LA_ALGO_RING: gen_shared_standard(s, st); break;
        case LA_ALGO_LANE:
        case LA_ALGO_LANE_MULTIPROC: gen_shared_lane(s, st, Q); break;
        default: return fail(LA_ERR_UNSUPPORTED, "unknown algorithm %d", (int)s.algo);
        }
        s.flags |= staged;
        if (staged) wrap_copy_in_out(s, st, s.algo == LA_ALGO_RING ? s.topo.procs : Q);
    } else {
        const int L = log2_exact(s.topo.ranks());
        if ((s.algo == LA_ALGO_RECURSIVE_DOUBLING || s.algo == LA_ALGO_RABENSEIFNER) && L < 0)
            return fail(LA_ERR_UNSUPPORTED, "recursive doubling / Rabenseifner need a power-of-two number of ranks (got %d)",
                        s.topo.ranks());
        switch (s.algo) {
        case LA_ALGO_RING: gen_ring(s, st); break;
        case LA_ALGO_LANE: gen_lane(s, st, false); break;
        case LA_ALGO_LANE_MULTIPROC: gen_lane(s, st, true); break;
        case LA_ALGO_RECURSIVE_DOUBLING: gen_recursive_doubling(s, st, L); break;
        case LA_ALGO_RABENSEIFNER: gen_rabenseifner(s, st, L); break;
        default: return fail(LA_ERR_UNSUPPORTED, "unknown algorithm %d", (int)s.algo);
        }
    }
    s.staging_elems = st.peak;
    const unsigned halves = s.flags & (LA_SCHED_ONLY_REDUCE_SCATTER | LA_SCHED_ONLY_ALLGATHER);
    if (halves) {
        // keep the launches of one half; a pack launch belongs to the reduce launch after it
        auto is_gather = [](int stage) {
            return stage == LA_STAGE_S2B || stage == LA_STAGE_S3 || stage == LA_STAGE_RING_AG ||
                   stage == LA_STAGE_S2_RING_AG || stage == LA_STAGE_RABENSEIFNER_AG;
        };
        std::vector<Step> kept;
        for (size_t i = 0; i < s.steps.size(); ++i) {
            int stage = s.steps[i].stage;
            if (stage == LA_STAGE_PACK && i + 1 < s.steps.size()) stage = s.steps[i + 1].stage;
            if (is_gather(stage) == (halves == LA_SCHED_ONLY_ALLGATHER)) kept.push_back(std::move(s.steps[i]));
        }
        s.steps.swap(kept);
    }
    if (s.flags & LA_SCHED_OUT_OF_PLACE) {
        const la_status_t st2 = make_out_of_place(s);
        if (st2 != LA_OK) return st2;
    }
    for (const Step& p : s.steps) {
        const size_t S = p.num_segments();
        if (p.src.size() != S * (size_t)p.k || p.dst.size() != S * (size_t)p.m)
            return fail(LA_ERR_INVALID_ARG, "internal: malformed step table");
    }
    return LA_OK;
}

// No segment of a step may write a range that another segment of the same step reads or
// writes; inside a segment a destination may coincide exactly with a source (in-place
// element-wise update) but not overlap it partially.
la_status_t validate_hazards(const la_schedule& s)
{
    struct Iv {
        int32_t buf;
        uint64_t lo, hi;
        uint32_t seg;
        bool write;
    };
    const uint64_t limit_stage = s.staging_elems;
    const int P = s.nbuf;
    std::vector<Iv> iv;
    for (size_t si = 0; si < s.steps.size(); ++si) {
        const Step& p = s.steps[si];
        iv.clear();
        for (size_t g = 0; g < p.num_segments(); ++g) {
            for (int t = 0; t < p.k; ++t) {
                const Operand& o = p.src[g * p.k + t];
                iv.push_back(Iv{o.buf, o.off, o.off + p.len[g], (uint32_t)g, false});
            }
            for (int d = 0; d < p.m; ++d) {
                const Operand& o = p.dst[g * p.m + d];
                iv.push_back(Iv{o.buf, o.off, o.off + p.len[g], (uint32_t)g, true});
            }
        }
        for (const Iv& x : iv) {
            const uint64_t cap = x.buf == P ? limit_stage : s.n;
            const int top = (s.flags & LA_SCHED_OUT_OF_PLACE) ? 2 * P : P;
            if (x.buf < 0 || x.buf > top || x.hi > cap || (x.write && x.buf > P))
                return fail(LA_ERR_INVALID_ARG, "internal: step %zu has a range outside its buffer", si);
        }
        std::sort(iv.begin(), iv.end(), [](const Iv& a, const Iv& b) {
            if (a.buf != b.buf) return a.buf < b.buf;
            if (a.lo != b.lo) return a.lo < b.lo;
            return a.hi < b.hi;
        });
        // sweep: compare each interval with the ones that start before its end
        for (size_t a = 0; a < iv.size(); ++a) {
            for (size_t b = a + 1; b < iv.size() && iv[b].buf == iv[a].buf && iv[b].lo < iv[a].hi; ++b) {
                if (!iv[a].write && !iv[b].write) continue;
                const bool same_seg = iv[a].seg == iv[b].seg;
                const bool identical = iv[a].lo == iv[b].lo && iv[a].hi == iv[b].hi;
                if (same_seg && identical && !(iv[a].write && iv[b].write)) continue;
                return fail(LA_ERR_INVALID_ARG, "internal: step %zu has a read/write hazard on buffer %d", si,
                            iv[a].buf);
            }
        }
    }
    return LA_OK;
}

} // namespace la

// ---- C ABI: topology and schedule objects ------------------------------------------------------

using namespace la;

extern "C" {

la_status_t la_topology_create(int nodes, int gpus_per_node, int procs_per_gpu, la_topology_t** out)
{
    if (!out) return fail(LA_ERR_INVALID_ARG, "la_topology_create: out is NULL");
    *out = nullptr;
    if (nodes < 1 || gpus_per_node < 1 || procs_per_gpu < 1)
        return fail(LA_ERR_INVALID_ARG, "la_topology_create: counts must be >= 1 (got %d, %d, %d)", nodes,
                    gpus_per_node, procs_per_gpu);
    const uint64_t P = (uint64_t)nodes * (uint64_t)gpus_per_node * (uint64_t)procs_per_gpu;
    if (P > (1u << 20)) return fail(LA_ERR_INVALID_ARG, "la_topology_create: more than 2^20 ranks");
    la_topology* t = new (std::nothrow) la_topology{nodes, gpus_per_node, procs_per_gpu};
    if (!t) return fail(LA_ERR_OUT_OF_MEMORY, "la_topology_create: out of host memory");
    *out = t;
    return LA_OK;
}

la_status_t la_topology_destroy(la_topology_t* topo)
{
    delete topo;
    return LA_OK;
}

int la_topology_num_ranks(const la_topology_t* topo)
{
    return topo ? topo->ranks() : -1;
}

la_status_t la_schedule_build_ex(const la_topology_t* topo, la_algo_t algo, size_t n, la_dtype_t dtype,
                                 unsigned flags, la_schedule_t** out)
{
    if (!out) return fail(LA_ERR_INVALID_ARG, "la_schedule_build: out is NULL");
    *out = nullptr;
    if (!topo) return fail(LA_ERR_INVALID_ARG, "la_schedule_build: topology is NULL");
    if (algo != LA_ALGO_LANE && algo != LA_ALGO_LANE_MULTIPROC)
        flags &= ~(unsigned)LA_SCHED_INNER_RING; // the flat algorithms have no inner stage
    if (n == 0) return fail(LA_ERR_INVALID_ARG, "la_schedule_build: n is 0");
    if (n > (uint64_t(1) << 40)) return fail(LA_ERR_INVALID_ARG, "la_schedule_build: n exceeds 2^40");
    if (!known_dtype((int)dtype)) return fail(LA_ERR_UNSUPPORTED, "la_schedule_build: unknown dtype %d", (int)dtype);
    if (algo != LA_ALGO_RING && algo != LA_ALGO_LANE && algo != LA_ALGO_LANE_MULTIPROC &&
        algo != LA_ALGO_RECURSIVE_DOUBLING && algo != LA_ALGO_RABENSEIFNER)
        return fail(LA_ERR_UNSUPPORTED, "la_schedule_build: unknown algorithm %d", (int)algo);
    if (flags & ~(unsigned)(LA_SCHED_P2P_GATHER | LA_SCHED_STAGED | LA_SCHED_INNER_RING | LA_SCHED_SHARED_BUFFERS |
                               LA_SCHED_OUT_OF_PLACE | LA_SCHED_ONLY_REDUCE_SCATTER | LA_SCHED_ONLY_ALLGATHER |
                               LA_SCHED_FUSED_GATHER | LA_SCHED_SINGLE_LAUNCH))
        return fail(LA_ERR_UNSUPPORTED, "la_schedule_build: unknown flag bits 0x%x", flags);
    la_schedule* s = new (std::nothrow) la_schedule;
    if (!s) return fail(LA_ERR_OUT_OF_MEMORY, "la_schedule_build: out of host memory");
    s->topo = *topo;
    s->algo = algo;
    s->dtype = dtype;
    s->n = n;
    s->flags = flags;
    s->nbuf = (flags & LA_SCHED_SHARED_BUFFERS) ? topo->nodes * topo->gpus : topo->ranks();
    la_status_t st;
    try {
        st = generate_steps(*s);
        if (st == LA_OK) st = validate_hazards(*s);
    } catch (const std::bad_alloc&) {
        st = fail(LA_ERR_OUT_OF_MEMORY, "la_schedule_build: out of host memory");
    }
    if (st != LA_OK) {
        delete s;
        return st;
    }
    *out = s;
    return LA_OK;
}

la_status_t la_schedule_build(const la_topology_t* topo, la_algo_t algo, size_t n, la_dtype_t dtype,
                              la_schedule_t** out)
{
    return la_schedule_build_ex(topo, algo, n, dtype, LA_SCHED_DEFAULT, out);
}

la_status_t la_schedule_destroy(la_schedule_t* sched)
{
    if (!sched) return LA_OK;
    for (la_binding* b : sched->bound) release_binding(b);
    delete sched;
    return LA_OK;
}

int la_schedule_num_steps(const la_schedule_t* sched)
{
    return sched ? (int)sched->steps.size() : -1;
}

int la_schedule_num_buffers(const la_schedule_t* sched)
{
    return sched ? sched->nbuf : -1;
}

int la_schedule_owned_ranges(const la_schedule_t* sched, int buffer, int capacity, uint64_t* offsets, uint64_t* lengths)
{
    if (!sched || buffer < 0 || buffer >= sched->nbuf) return -1;
    int count = 0;
    for (const Part& p : sched->owned[buffer]) {
        if (p.cnt == 0) continue;
        if (count < capacity) {
            if (offsets) offsets[count] = p.off;
            if (lengths) lengths[count] = p.cnt;
        }
        ++count;
    }
    return count;
}

size_t la_schedule_staging_elems(const la_schedule_t* sched)
{
    return sched ? (size_t)sched->staging_elems : 0;
}

la_status_t la_schedule_step_info(const la_schedule_t* sched, int step, int* kind, int* stage,
                                  size_t* num_segments, size_t* seg_len_max, int* fan_in, int* fan_out,
                                  size_t* bytes_read, size_t* bytes_written)
{
    if (!sched) return fail(LA_ERR_INVALID_ARG, "la_schedule_step_info: schedule is NULL");
    if (step < 0 || step >= (int)sched->steps.size())
        return fail(LA_ERR_INVALID_ARG, "la_schedule_step_info: step %d out of range", step);
    const Step& p = sched->steps[step];
    uint64_t total = 0, longest = 0;
    for (uint64_t l : p.len) {
        total += l;
        longest = std::max(longest, l);
    }
    const size_t e = dtype_size(sched->dtype);
    if (kind) *kind = p.kind;
    if (stage) *stage = p.stage;
    if (num_segments) *num_segments = p.num_segments();
    if (seg_len_max) *seg_len_max = (size_t)longest;
    if (fan_in) *fan_in = p.k;
    if (fan_out) *fan_out = p.m;
    if (bytes_read) *bytes_read = (size_t)(total * (uint64_t)p.k * e);
    if (bytes_written) *bytes_written = (size_t)(total * (uint64_t)p.m * e);
    return LA_OK;
}

int la_schedule_step_group(const la_schedule_t* sched, int step)
{
    if (!sched || step < 0 || step >= (int)sched->steps.size()) return -1;
    const Step& p = sched->steps[step];
    return p.group > 0 && p.group < p.k ? p.group : p.k;
}

la_status_t la_schedule_step_table(const la_schedule_t* sched, int step, uint64_t* seg_len, int32_t* src_buf,
                                   uint64_t* src_off, int32_t* dst_buf, uint64_t* dst_off)
{
    if (!sched) return fail(LA_ERR_INVALID_ARG, "la_schedule_step_table: schedule is NULL");
    if (step < 0 || step >= (int)sched->steps.size())
        return fail(LA_ERR_INVALID_ARG, "la_schedule_step_table: step %d out of range", step);
    const Step& p = sched->steps[step];
    if (seg_len) std::copy(p.len.begin(), p.len.end(), seg_len);
    for (size_t i = 0; i < p.src.size(); ++i) {
        if (src_buf) src_buf[i] = p.src[i].buf;
        if (src_off) src_off[i] = p.src[i].off;
    }
    for (size_t i = 0; i < p.dst.size(); ++i) {
        if (dst_buf) dst_buf[i] = p.dst[i].buf;
        if (dst_off) dst_off[i] = p.dst[i].off;
    }
    return LA_OK;
}

const char* la_status_string(la_status_t status)
{
    switch (status) {
    case LA_OK: return "LA_OK";
    case LA_ERR_INVALID_ARG: return "LA_ERR_INVALID_ARG";
    case LA_ERR_UNSUPPORTED: return "LA_ERR_UNSUPPORTED";
    case LA_ERR_OUT_OF_MEMORY: return "LA_ERR_OUT_OF_MEMORY";
    case LA_ERR_DEVICE: return "LA_ERR_DEVICE";
    }
    return "LA_ERR_UNKNOWN";
}

const char* la_last_error(void)
{
    return g_err;
}

} // extern "C"
