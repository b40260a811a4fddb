/*
 * la_oracle.c -- CPU oracle for the emulated lane-aware all-reduce.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
 * GPU library is checked against.  It shares no code, header, table or
 * constant with the HIP path, and the product never calls it: only the tests,
 * the smoke check and the benchmark's CPU-baseline leg load it.
 *
 * Two oracles live here.
 *
 *   oracle_definition_sum   the definition of an all-reduce with SUM: every
 *                           rank ends with the element-wise sum of all P
 *                           input buffers (paper, Introduction: each process
 *                           exchanges and reduces data with all others; the
 *                           MPI_Allreduce(..., MPI_SUM, ...) call of the
 *                           "Standard Approach" subsection).
 *
 *   oracle_allreduce        a rank-centric, message-by-message simulation of
 *                           the schedules: Algorithm 1 (ring_allreduce) and
 *                           Algorithm 2 (lane_allreduce), the latter also in
 *                           its multiple-processes-per-GPU form ("Multi-lane
 *                           Approach" subsection).  P virtual ranks own
 *                           private buffers.  A step has two halves: first
 *                           every rank posts copies of what it sends (so all
 *                           sends see the state at the start of the step),
 *                           then every rank consumes what it received.
 *
 * Readings where the paper is silent (all are this build's, stated once):
 *   - rank r = (node*G + gpu)*Q + proc, following l_r = r mod PPG
 *     ("Multiple Processes Per GPU" subsection);
 *   - every one of the P ranks contributes a private buffer of n elements;
 *   - a length is split into m parts in a balanced way: part i has
 *     floor(len/m) elements plus one if i < len mod m (Algorithms 1 and 2
 *     print an integer division that would drop the remainder);
 *   - the loops of Algorithm 1 run P-1 times (text under Algorithm 1);
 *   - MPI_Reduce_scatter and MPI_Allreduce of Algorithm 2 are vendor black
 *     boxes; here each is a direct exchange: every member sends its copy of a
 *     part to the part's owner, who adds the operands in ascending
 *     communicator rank (its own copy taking its place in that order), and
 *     the all-reduce is that reduce-scatter followed by an all-gather;
 *   - recursive doubling and Rabenseifner's algorithm are only described in
 *     words (Background section): they are taken in their textbook form for a
 *     power-of-two number of ranks (exchange with the rank that differs in one
 *     bit; recursive halving from distance P/2 down, lower rank keeps the
 *     first half; recursive doubling back up);
 *   - the "_ring" variants run Algorithm 1 as that inter-node all-reduce
 *     instead: the owned part is cut into N pieces and member v of the lane
 *     communicator plays rank v of a ring of N;
 *   - lanes first (one per GPU), then sub-chunks (one per process) inside a
 *     lane; "lane" without the multi-process split gives each lane to the
 *     GPU's leader process (local rank 0);
 *   - int32 wraps (two's complement); fp32 is IEEE binary32 add, left to
 *     right; bf16 and fp16 operands are widened exactly to fp32, added in fp32
 *     and rounded once (nearest, ties to even) when a step stores its result;
 *     fp64 is IEEE binary64.  The operations other than the sum (product,
 *     maximum, minimum) are not in the paper; they run on the same schedules
 *     with the binary operations defined under "one binary operation".
 *
 * Parity pins: see tests/test_oracle_*.py (definition, closed forms, the
 * index walk of Algorithm 1, stage boundaries of Algorithm 2, brute force).
 * The paper prints no worked numeric example, so no pin comes from printed
 * values.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_I32 = 0, ORACLE_F32 = 1, ORACLE_BF16 = 2, ORACLE_F16 = 3, ORACLE_F64 = 4 };
/* reduction operations (MPI_SUM is the paper's; the others follow the same schedules) */
enum { OP_SUM = 0, OP_PROD = 1, OP_MAX = 2, OP_MIN = 3 };
enum {
    ORACLE_RING = 0,
    ORACLE_LANE = 1,
    ORACLE_LANE_MULTIPROC = 2,
    /* Algorithm 2 with Algorithm 1 as the all-reduce on the lane communicator (the inter-node ring
     * variant that the Results section measures) */
    ORACLE_LANE_RING = 3,
    ORACLE_LANE_MULTIPROC_RING = 4,
    /* the small- and medium-size algorithms of the Background section, flat over the P ranks
     * (P a power of two) */
    ORACLE_RECURSIVE_DOUBLING = 5,
    ORACLE_RABENSEIFNER = 6
};

/* phases recorded in the message trace */
enum {
    PH_LANE_S1 = 1,  /* intra-node reduce-scatter          */
    PH_LANE_S2A = 2, /* inter-node reduce-scatter of parts */
    PH_LANE_S2B = 3, /* inter-node all-gather of pieces    */
    PH_LANE_S3 = 4,  /* intra-node all-gather              */
    PH_LANE_S2_RING_RS = 5, /* inter-node stage as a ring: reduce loop */
    PH_LANE_S2_RING_AG = 6, /* inter-node stage as a ring: gather loop */
    PH_RING_RS = 10, /* ring reduce-scatter loop           */
    PH_RING_AG = 11, /* ring all-gather loop               */
    PH_RECURSIVE_DOUBLING = 20, /* pairwise exchange of the whole buffer */
    PH_RABENSEIFNER_RS = 21,    /* recursive halving: reduce-scatter      */
    PH_RABENSEIFNER_AG = 22     /* recursive doubling: all-gather         */
};

typedef struct {
    int32_t phase;
    int32_t step; /* round counter, from 0 */
    int32_t src;
    int32_t dst;
    uint64_t off; /* element offset in the rank buffers */
    uint64_t cnt; /* elements */
} oracle_msg_t;

static int g_threads = 1;

void oracle_set_threads(int t)
{
    g_threads = t < 1 ? 1 : t;
}

int oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static size_t elem_size(int dtype)
{
    if (dtype == ORACLE_BF16 || dtype == ORACLE_F16) return 2;
    return dtype == ORACLE_F64 ? 8 : 4;
}

/* ---- bf16 <-> fp32 ------------------------------------------------------ */

/* bf16 is the upper half of a binary32: widening appends 16 zero bits. */
static float bf16_widen(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* Round a binary32 to the nearest bf16, ties to the even mantissa.  Written
 * from the definition: look at the 16 discarded bits, compare with half. */
static uint16_t bf16_round(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    uint32_t exp = (u >> 23) & 0xffu, man = u & 0x7fffffu;
    if (exp == 0xffu && man != 0) /* NaN stays NaN: keep sign, set quiet bit */
        return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t kept = u >> 16, lost = u & 0xffffu;
    if (lost > 0x8000u)
        kept += 1; /* above half: away; a carry into the exponent is right */
    else if (lost == 0x8000u && (kept & 1u))
        kept += 1; /* exactly half: to even */
    return (uint16_t)kept;
}

void oracle_bf16_round(const float* in, uint16_t* out, uint64_t n)
{
    for (uint64_t i = 0; i < n; ++i) out[i] = bf16_round(in[i]);
}

void oracle_bf16_widen(const uint16_t* in, float* out, uint64_t n)
{
    for (uint64_t i = 0; i < n; ++i) out[i] = bf16_widen(in[i]);
}

/* ---- IEEE binary16 <-> fp32 --------------------------------------------- */

/* binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits.  Widening is exact. */
static float f16_widen(uint16_t h)
{
    uint32_t sign = (uint32_t)(h & 0x8000u) << 16, e = (h >> 10) & 0x1fu, m = h & 0x3ffu, u;
    if (e == 0x1fu) {
        u = sign | 0x7f800000u | (m << 13); /* infinity or NaN */
    } else if (e != 0) {
        u = sign | ((e + 112u) << 23) | (m << 13); /* normal: rebias 15 -> 127 */
    } else {
        /* zero or subnormal: m * 2^-24, exactly representable in binary32 */
        float f = (float)m * 5.9604644775390625e-08f; /* 2^-24 */
        memcpy(&u, &f, 4);
        u |= sign;
    }
    float r;
    memcpy(&r, &u, 4);
    return r;
}

/* Round a binary32 to the nearest binary16, ties to even, from the definition. */
static uint16_t f16_round(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    uint32_t a = u & 0x7fffffffu, e = a >> 23, m = a & 0x7fffffu;
    if (a > 0x7f800000u) return (uint16_t)(sign | 0x7e00u); /* NaN */
    if (e == 0xffu) return (uint16_t)(sign | 0x7c00u);      /* infinity */
    if (e >= 113u) {
        /* at least 2^-14: a normal binary16 unless it overflows; drop 13 fraction bits */
        uint32_t kept = ((e - 112u) << 10) | (m >> 13), lost = m & 0x1fffu;
        if (lost > 0x1000u || (lost == 0x1000u && (kept & 1u))) kept += 1; /* a carry moves to the exponent */
        if (kept >= 0x7c00u) kept = 0x7c00u; /* beyond the largest finite value: infinity */
        return (uint16_t)(sign | kept);
    }
    if (e == 0) return sign; /* binary32 subnormals are far below half of 2^-24 */
    /* below 2^-14: the result is a multiple of 2^-24.  value = (2^23 + m) * 2^(e-150), so in
     * units of 2^-24 it is (2^23 + m) >> (126 - e). */
    uint32_t full = 0x800000u | m, shift = 126u - e;
    if (shift > 24u) return sign; /* less than half a unit */
    uint32_t kept = full >> shift, lost = full & ((1u << shift) - 1u), half = 1u << (shift - 1u);
    if (lost > half || (lost == half && (kept & 1u))) kept += 1;
    return (uint16_t)(sign | kept);
}

void oracle_f16_round(const float* in, uint16_t* out, uint64_t n)
{
    for (uint64_t i = 0; i < n; ++i) out[i] = f16_round(in[i]);
}

void oracle_f16_widen(const uint16_t* in, float* out, uint64_t n)
{
    for (uint64_t i = 0; i < n; ++i) out[i] = f16_widen(in[i]);
}

/* ---- balanced split ------------------------------------------------------ */

/* part i of m of a length len: offset (relative) and count */
static void part(uint64_t len, uint64_t m, uint64_t i, uint64_t* off, uint64_t* cnt)
{
    uint64_t q = len / m, rem = len % m;
    *cnt = q + (i < rem ? 1 : 0);
    *off = i * q + (i < rem ? i : rem);
}

void oracle_part(uint64_t len, uint64_t m, uint64_t i, uint64_t* off, uint64_t* cnt)
{
    part(len, m, i, off, cnt);
}

/* ---- the definition ------------------------------------------------------ */

/* ---- one binary operation ------------------------------------------------- */

/* Maximum of two floating-point numbers as the schedules use it: a NaN loses against a number,
 * two NaNs give the first, and +0 is larger than -0.  a is the running value, b the next operand. */
static double max_f64(double a, double b)
{
    if (b != b) return a;
    if (a != a) return b;
    if (a < b) return b;
    if (a == b && a == 0.0) { /* signed zeros: take +0 if either is +0 */
        uint64_t ua, ub;
        memcpy(&ua, &a, 8);
        memcpy(&ub, &b, 8);
        return (ua >> 63) ? b : a;
    }
    return a;
}

static double min_f64(double a, double b)
{
    if (b != b) return a;
    if (a != a) return b;
    if (b < a) return b;
    if (a == b && a == 0.0) { /* take -0 if either is -0 */
        uint64_t ua;
        memcpy(&ua, &a, 8);
        return (ua >> 63) ? a : b;
    }
    return a;
}

/* binary32 operands: max and min are exact, so going through binary64 changes nothing */
static float op_f32(int op, float a, float b)
{
    switch (op) {
    case OP_SUM: return a + b;
    case OP_PROD: return a * b;
    case OP_MAX: return (float)max_f64((double)a, (double)b);
    default: return (float)min_f64((double)a, (double)b);
    }
}

static double op_f64(int op, double a, double b)
{
    switch (op) {
    case OP_SUM: return a + b;
    case OP_PROD: return a * b;
    case OP_MAX: return max_f64(a, b);
    default: return min_f64(a, b);
    }
}

/* int32: sum and product wrap (two's complement), max and min compare as signed */
static uint32_t op_u32(int op, uint32_t a, uint32_t b)
{
    switch (op) {
    case OP_SUM: return a + b;
    case OP_PROD: return a * b;
    case OP_MAX: return (int32_t)b > (int32_t)a ? b : a;
    default: return (int32_t)b < (int32_t)a ? b : a;
    }
}

/* ---- the definition ------------------------------------------------------ */

static double as_double(int dtype, const void* p, uint64_t i)
{
    switch (dtype) {
    case ORACLE_F32: return (double)((const float*)p)[i];
    case ORACLE_BF16: return (double)bf16_widen(((const uint16_t*)p)[i]);
    case ORACLE_F16: return (double)f16_widen(((const uint16_t*)p)[i]);
    default: return ((const double*)p)[i];
    }
}

/* out[i] = in[0][i] op in[1][i] op ... op in[P-1][i].  int32: exact (sum in int64 then wrapped
 * to 32 bits, product modulo 2^32), out is int32[n].  Floating types: computed in fp64 in
 * ascending rank, out is double[n] (the caller applies the tolerance; max and min are exact). */
int oracle_definition_reduce(int dtype, int op, int P, uint64_t n, const void* const* in, void* out)
{
    if (P < 1 || !in || !out || op < OP_SUM || op > OP_MIN) return 1;
    if (dtype == ORACLE_I32) {
        int32_t* o = (int32_t*)out;
        for (uint64_t i = 0; i < n; ++i) {
            if (op == OP_SUM) {
                int64_t s = 0;
                for (int p = 0; p < P; ++p) s += ((const int32_t*)in[p])[i];
                o[i] = (int32_t)(uint32_t)(uint64_t)s;
            } else if (op == OP_PROD) {
                uint64_t s = 1;
                for (int p = 0; p < P; ++p) s = (s * (uint64_t)(uint32_t)((const int32_t*)in[p])[i]) & 0xffffffffull;
                o[i] = (int32_t)(uint32_t)s;
            } else {
                int32_t s = ((const int32_t*)in[0])[i];
                for (int p = 1; p < P; ++p) {
                    int32_t v = ((const int32_t*)in[p])[i];
                    if (op == OP_MAX ? v > s : v < s) s = v;
                }
                o[i] = s;
            }
        }
    } else if (dtype == ORACLE_F32 || dtype == ORACLE_BF16 || dtype == ORACLE_F16 || dtype == ORACLE_F64) {
        double* o = (double*)out;
        for (uint64_t i = 0; i < n; ++i) {
            double s = as_double(dtype, in[0], i);
            for (int p = 1; p < P; ++p) s = op_f64(op, s, as_double(dtype, in[p], i));
            o[i] = s;
        }
    } else {
        return 2;
    }
    return 0;
}

int oracle_definition_sum(int dtype, int P, uint64_t n, const void* const* in, void* out)
{
    return oracle_definition_reduce(dtype, OP_SUM, P, n, in, out);
}

/* ---- element-wise k-operand sum, operands in the order given -------------- */

static void sum_operands(int dtype, int op, void* dst, const void* const* ops, int k, uint64_t cnt)
{
    int64_t m = (int64_t)cnt;
    if (dtype == ORACLE_I32) {
#pragma omp parallel for num_threads(g_threads) schedule(static)
        for (int64_t i = 0; i < m; ++i) {
            uint32_t s = ((const uint32_t*)ops[0])[i];
            for (int t = 1; t < k; ++t) s = op_u32(op, s, ((const uint32_t*)ops[t])[i]);
            ((uint32_t*)dst)[i] = s;
        }
    } else if (dtype == ORACLE_F32) {
#pragma omp parallel for num_threads(g_threads) schedule(static)
        for (int64_t i = 0; i < m; ++i) {
            float s = ((const float*)ops[0])[i];
            for (int t = 1; t < k; ++t) s = op_f32(op, s, ((const float*)ops[t])[i]);
            ((float*)dst)[i] = s;
        }
    } else if (dtype == ORACLE_F64) {
#pragma omp parallel for num_threads(g_threads) schedule(static)
        for (int64_t i = 0; i < m; ++i) {
            double s = ((const double*)ops[0])[i];
            for (int t = 1; t < k; ++t) s = op_f64(op, s, ((const double*)ops[t])[i]);
            ((double*)dst)[i] = s;
        }
    } else if (dtype == ORACLE_F16) {
        /* widened exactly, combined in fp32, rounded once when the step stores */
#pragma omp parallel for num_threads(g_threads) schedule(static)
        for (int64_t i = 0; i < m; ++i) {
            float s = f16_widen(((const uint16_t*)ops[0])[i]);
            for (int t = 1; t < k; ++t) s = op_f32(op, s, f16_widen(((const uint16_t*)ops[t])[i]));
            ((uint16_t*)dst)[i] = f16_round(s);
        }
    } else {
#pragma omp parallel for num_threads(g_threads) schedule(static)
        for (int64_t i = 0; i < m; ++i) {
            float s = bf16_widen(((const uint16_t*)ops[0])[i]);
            for (int t = 1; t < k; ++t) s = op_f32(op, s, bf16_widen(((const uint16_t*)ops[t])[i]));
            ((uint16_t*)dst)[i] = bf16_round(s);
        }
    }
}

/* dst[o] = ((dst[o] + srcs[0][o]) + srcs[1][o]) + ... for o in every segment:
 * "k incoming segments summed into the owned segment". */
int oracle_reduce_segments_op(int dtype, int op, void* dst, const void* const* srcs, int k,
                              const uint64_t* seg_offsets, uint64_t num_segments, uint64_t seg_len);

int oracle_reduce_segments(int dtype, void* dst, const void* const* srcs, int k,
                           const uint64_t* seg_offsets, uint64_t num_segments, uint64_t seg_len)
{
    return oracle_reduce_segments_op(dtype, OP_SUM, dst, srcs, k, seg_offsets, num_segments, seg_len);
}

int oracle_reduce_segments_op(int dtype, int op, void* dst, const void* const* srcs, int k,
                              const uint64_t* seg_offsets, uint64_t num_segments, uint64_t seg_len)
{
    if (k < 0 || k > 4096 || op < OP_SUM || op > OP_MIN) return 1;
    size_t e = elem_size(dtype);
    const void* ops[4097];
    for (uint64_t s = 0; s < num_segments; ++s) {
        uint64_t o = seg_offsets[s];
        ops[0] = (const char*)dst + o * e;
        for (int t = 0; t < k; ++t) ops[t + 1] = (const char*)srcs[t] + o * e;
        sum_operands(dtype, op, (char*)dst + o * e, ops, k + 1, seg_len);
    }
    return 0;
}

/* ---- the virtual machine: P ranks, private buffers, a mailbox ------------ */

typedef struct {
    int src;
    uint64_t off, cnt;
    void* data; /* private copy of the payload */
} letter_t;

typedef struct {
    letter_t* v;
    size_t len, cap;
} inbox_t;

typedef struct {
    int P;
    int dtype;
    int op;         /* the reduction operation of the run */
    size_t esz;
    uint64_t n;
    void** buf;     /* the buffers (caller's memory, updated in place) */
    int share;      /* processes per buffer: 1 = every rank owns buf[r]; Q = the Q processes of a
                       GPU work on the one buffer of their GPU, buf[r / Q] */
    inbox_t* inbox; /* inbox[r]: letters addressed to rank r in this round */
    oracle_msg_t* trace;
    uint64_t trace_cap, trace_len;
    int phase, round;
    int failed;
} world_t;

static char* mem(const world_t* w, int rank)
{
    return (char*)w->buf[rank / w->share];
}

static void post(world_t* w, int src, int dst, uint64_t off, uint64_t cnt)
{
    if (w->trace && w->trace_len < w->trace_cap) {
        oracle_msg_t* t = &w->trace[w->trace_len];
        t->phase = w->phase;
        t->step = w->round;
        t->src = src;
        t->dst = dst;
        t->off = off;
        t->cnt = cnt;
    }
    w->trace_len++;
    inbox_t* b = &w->inbox[dst];
    if (b->len == b->cap) {
        size_t nc = b->cap ? 2 * b->cap : 8;
        letter_t* nv = (letter_t*)realloc(b->v, nc * sizeof(letter_t));
        if (!nv) {
            w->failed = 1;
            return;
        }
        b->v = nv;
        b->cap = nc;
    }
    letter_t* l = &b->v[b->len++];
    l->src = src;
    l->off = off;
    l->cnt = cnt;
    l->data = malloc(cnt * w->esz + 1);
    if (!l->data) {
        w->failed = 1;
        l->cnt = 0;
        return;
    }
    memcpy(l->data, mem(w, src) + off * w->esz, cnt * w->esz);
}

static const letter_t* letter_from(const world_t* w, int at, int src)
{
    const inbox_t* b = &w->inbox[at];
    for (size_t i = 0; i < b->len; ++i)
        if (b->v[i].src == src) return &b->v[i];
    return NULL;
}

static void end_round(world_t* w)
{
    for (int r = 0; r < w->P; ++r) {
        inbox_t* b = &w->inbox[r];
        for (size_t i = 0; i < b->len; ++i) free(b->v[i].data);
        b->len = 0;
    }
    w->round++;
}

static void overwrite(world_t* w, int at, const letter_t* l)
{
    memcpy(mem(w, at) + l->off * w->esz, l->data, l->cnt * w->esz);
}

/* ---- Algorithm 1: ring_allreduce ---------------------------------------- */

static int imod(int a, int m)
{
    int r = a % m;
    return r < 0 ? r + m : r;
}

static int run_ring(world_t* w, int max_rounds)
{
    int P = w->P;
    uint64_t* D = (uint64_t*)malloc(sizeof(uint64_t) * (size_t)P);   /* displacements */
    uint64_t* cnt = (uint64_t*)malloc(sizeof(uint64_t) * (size_t)P); /* counts per chunk */
    if (!D || !cnt) return 3;
    for (int c = 0; c < P; ++c) part(w->n, (uint64_t)P, (uint64_t)c, &D[c], &cnt[c]);

    /* first loop: in round i rank r sends chunk sp = r - i to its successor
     * and adds the chunk rp = r - 1 - i it receives from its predecessor */
    w->phase = PH_RING_RS;
    for (int i = 0; i < P - 1 && w->round < max_rounds; ++i) {
        for (int r = 0; r < P; ++r) {
            int sp = imod(r - i, P);
            post(w, r, (r + 1) % P, D[sp], cnt[sp]);
        }
        for (int r = 0; r < P; ++r) {
            const letter_t* l = letter_from(w, r, imod(r - 1, P));
            if (!l) return 4;
            char* own = mem(w, r) + l->off * w->esz;
            const void* ops[2] = {own, l->data}; /* own = own + incoming */
            sum_operands(w->dtype, w->op, own, ops, 2, l->cnt);
        }
        end_round(w);
    }
    /* second loop: sp starts at r + 1, rp at r; received chunks overwrite */
    w->phase = PH_RING_AG;
    for (int i = 0; i < P - 1 && w->round < max_rounds; ++i) {
        for (int r = 0; r < P; ++r) {
            int sp = imod(r + 1 - i, P);
            post(w, r, (r + 1) % P, D[sp], cnt[sp]);
        }
        for (int r = 0; r < P; ++r) {
            const letter_t* l = letter_from(w, r, imod(r - 1, P));
            if (!l) return 4;
            overwrite(w, r, l);
        }
        end_round(w);
    }
    free(D);
    free(cnt);
    return w->failed ? 3 : 0;
}

/* ---- Background section: recursive doubling and Rabenseifner's algorithm ---- */

static int log2_exact(int P)
{
    int L = 0;
    while ((1 << L) < P) ++L;
    return (1 << L) == P ? L : -1;
}

/* Recursive doubling: log2(P) rounds; in round s rank r exchanges its WHOLE buffer with the
 * rank whose number differs in bit s, and both add what they receive to their own copy. */
static int run_recursive_doubling(world_t* w, int max_rounds)
{
    int P = w->P, L = log2_exact(P);
    if (L < 0) return 2;
    w->phase = PH_RECURSIVE_DOUBLING;
    for (int s = 0; s < L && w->round < max_rounds; ++s) {
        for (int r = 0; r < P; ++r) post(w, r, r ^ (1 << s), 0, w->n);
        for (int r = 0; r < P; ++r) {
            const letter_t* l = letter_from(w, r, r ^ (1 << s));
            if (!l) return 4;
            char* own = mem(w, r);
            const void* two[2] = {own, l->data}; /* own = own + incoming */
            sum_operands(w->dtype, w->op, own, two, 2, l->cnt);
        }
        end_round(w);
    }
    return w->failed ? 3 : 0;
}

/* Rabenseifner: a reduce-scatter by recursive halving (the partner is at distance P/2, P/4, ...;
 * each rank keeps one half of its current range, sends the other half, and adds the partner's
 * copy of the half it keeps), then an all-gather by recursive doubling that walks the same
 * ranges back.  2*log2(P) messages, the data halving at each reduce step. */
static int run_rabenseifner(world_t* w, int max_rounds)
{
    int P = w->P, L = log2_exact(P);
    if (L < 0) return 2;
    /* lo[r][s], cnt[r][s]: the range rank r works on before reduce round s (s = L: what it owns) */
    uint64_t* lo = (uint64_t*)calloc((size_t)P * (size_t)(L + 1), sizeof(uint64_t));
    uint64_t* cnt = (uint64_t*)calloc((size_t)P * (size_t)(L + 1), sizeof(uint64_t));
    if (!lo || !cnt) return 3;
    for (int r = 0; r < P; ++r) {
        lo[r * (L + 1)] = 0;
        cnt[r * (L + 1)] = w->n;
        for (int s = 0; s < L; ++s) {
            int d = P >> (s + 1);
            uint64_t o, c;
            part(cnt[r * (L + 1) + s], 2, (r & d) ? 1 : 0, &o, &c); /* lower ranks keep the first half */
            lo[r * (L + 1) + s + 1] = lo[r * (L + 1) + s] + o;
            cnt[r * (L + 1) + s + 1] = c;
        }
    }
    w->phase = PH_RABENSEIFNER_RS;
    for (int s = 0; s < L && w->round < max_rounds; ++s) {
        int d = P >> (s + 1);
        for (int r = 0; r < P; ++r) {
            int p = r ^ d; /* send the half the partner keeps */
            post(w, r, p, lo[p * (L + 1) + s + 1], cnt[p * (L + 1) + s + 1]);
        }
        for (int r = 0; r < P; ++r) {
            const letter_t* l = letter_from(w, r, r ^ d);
            if (!l || l->off != lo[r * (L + 1) + s + 1]) return 4;
            char* own = mem(w, r) + l->off * w->esz;
            const void* two[2] = {own, l->data};
            sum_operands(w->dtype, w->op, own, two, 2, l->cnt);
        }
        end_round(w);
    }
    w->phase = PH_RABENSEIFNER_AG;
    for (int s = L - 1; s >= 0 && w->round < max_rounds; --s) {
        int d = P >> (s + 1);
        for (int r = 0; r < P; ++r) post(w, r, r ^ d, lo[r * (L + 1) + s + 1], cnt[r * (L + 1) + s + 1]);
        for (int r = 0; r < P; ++r) {
            const letter_t* l = letter_from(w, r, r ^ d);
            if (!l) return 4;
            overwrite(w, r, l);
        }
        end_round(w);
    }
    free(lo);
    free(cnt);
    return w->failed ? 3 : 0;
}

/* ---- Algorithm 2: lane_allreduce, with or without the per-process split -- */

typedef struct {
    int N, G, Q;
    int split_procs; /* 1: every process owns a sub-chunk; 0: the GPU's leader owns the lane */
    int inner_ring;  /* 1: stage 2 is Algorithm 1 run on every lane communicator */
} lane_cfg_t;

static int rank_of(const lane_cfg_t* c, int node, int local)
{
    return node * c->G * c->Q + local; /* local = gpu*Q + proc */
}

static int num_parts(const lane_cfg_t* c)
{
    return c->split_procs ? c->G * c->Q : c->G;
}

/* node-local index of the process that owns part j */
static int owner_local(const lane_cfg_t* c, int j)
{
    return c->split_procs ? j : j * c->Q;
}

/* part j of the buffer: lane g of G, then (if split) sub-chunk q of Q inside it */
static void part_of_buffer(const lane_cfg_t* c, uint64_t n, int j, uint64_t* off, uint64_t* cnt)
{
    if (!c->split_procs) {
        part(n, (uint64_t)c->G, (uint64_t)j, off, cnt);
        return;
    }
    int g = j / c->Q, q = j % c->Q;
    uint64_t lo, lc, so, sc;
    part(n, (uint64_t)c->G, (uint64_t)g, &lo, &lc);
    part(lc, (uint64_t)c->Q, (uint64_t)q, &so, &sc);
    *off = lo + so;
    *cnt = sc;
}

static int run_lane(world_t* w, const lane_cfg_t* c, int max_rounds)
{
    int N = c->N, R = c->G * c->Q, J = num_parts(c);
    const void** ops = (const void**)malloc(sizeof(void*) * (size_t)(R > N ? R : N));
    if (!ops) return 3;

    /* stage 1: reduce-scatter on the node group.  Every process of the node
     * sends its copy of part j to the part's owner; the owner adds the R
     * copies in ascending node-local index. */
    if (w->round < max_rounds) {
        w->phase = PH_LANE_S1;
        for (int node = 0; node < N; ++node)
            for (int j = 0; j < J; ++j) {
                uint64_t off, cnt;
                part_of_buffer(c, w->n, j, &off, &cnt);
                int own = owner_local(c, j);
                for (int l = 0; l < R; ++l)
                    if (l != own) post(w, rank_of(c, node, l), rank_of(c, node, own), off, cnt);
            }
        for (int node = 0; node < N; ++node)
            for (int j = 0; j < J; ++j) {
                uint64_t off, cnt;
                part_of_buffer(c, w->n, j, &off, &cnt);
                int own = owner_local(c, j), me = rank_of(c, node, own);
                char* mine = mem(w, me) + off * w->esz;
                for (int l = 0; l < R; ++l) {
                    if (l == own) {
                        ops[l] = mine;
                    } else {
                        const letter_t* le = letter_from(w, me, rank_of(c, node, l));
                        if (!le || le->off != off) return 4;
                        ops[l] = le->data;
                    }
                }
                sum_operands(w->dtype, w->op, mine, ops, R, cnt);
            }
        end_round(w);
    }

    /* stage 2, ring form: Algorithm 1 on every lane communicator at once.  The
     * part is cut into N pieces; member v plays rank v of a ring of N. */
    if (c->inner_ring) {
        for (int loop = 0; loop < 2; ++loop) {
            w->phase = loop == 0 ? PH_LANE_S2_RING_RS : PH_LANE_S2_RING_AG;
            for (int i = 0; i < N - 1 && w->round < max_rounds; ++i) {
                for (int j = 0; j < J; ++j) {
                    uint64_t off, cnt, po, pc;
                    part_of_buffer(c, w->n, j, &off, &cnt);
                    int own = owner_local(c, j);
                    for (int v = 0; v < N; ++v) {
                        int sp = loop == 0 ? imod(v - i, N) : imod(v + 1 - i, N);
                        part(cnt, (uint64_t)N, (uint64_t)sp, &po, &pc);
                        post(w, rank_of(c, v, own), rank_of(c, (v + 1) % N, own), off + po, pc);
                    }
                }
                for (int j = 0; j < J; ++j) {
                    int own = owner_local(c, j);
                    for (int v = 0; v < N; ++v) {
                        int me = rank_of(c, v, own);
                        const letter_t* le = letter_from(w, me, rank_of(c, imod(v - 1, N), own));
                        if (!le) return 4;
                        if (loop == 0) {
                            char* mine = mem(w, me) + le->off * w->esz;
                            const void* two[2] = {mine, le->data}; /* own = own + incoming */
                            sum_operands(w->dtype, w->op, mine, two, 2, le->cnt);
                        } else {
                            overwrite(w, me, le);
                        }
                    }
                }
                end_round(w);
            }
        }
    }

    /* stage 2: all-reduce of part j on the lane communicator (the owners of
     * part j on the N nodes), as reduce-scatter of N pieces + all-gather. */
    if (!c->inner_ring && w->round < max_rounds) {
        w->phase = PH_LANE_S2A;
        for (int j = 0; j < J; ++j) {
            uint64_t off, cnt;
            part_of_buffer(c, w->n, j, &off, &cnt);
            int own = owner_local(c, j);
            for (int from = 0; from < N; ++from)
                for (int to = 0; to < N; ++to) {
                    uint64_t po, pc;
                    part(cnt, (uint64_t)N, (uint64_t)to, &po, &pc);
                    if (to != from) post(w, rank_of(c, from, own), rank_of(c, to, own), off + po, pc);
                }
        }
        for (int j = 0; j < J; ++j) {
            uint64_t off, cnt;
            part_of_buffer(c, w->n, j, &off, &cnt);
            int own = owner_local(c, j);
            for (int node = 0; node < N; ++node) {
                uint64_t po, pc;
                part(cnt, (uint64_t)N, (uint64_t)node, &po, &pc);
                int me = rank_of(c, node, own);
                char* mine = mem(w, me) + (off + po) * w->esz;
                for (int from = 0; from < N; ++from) {
                    if (from == node) {
                        ops[from] = mine;
                    } else {
                        const letter_t* le = letter_from(w, me, rank_of(c, from, own));
                        if (!le || le->off != off + po) return 4;
                        ops[from] = le->data;
                    }
                }
                sum_operands(w->dtype, w->op, mine, ops, N, pc);
            }
        }
        end_round(w);
    }
    if (!c->inner_ring && w->round < max_rounds) {
        w->phase = PH_LANE_S2B;
        for (int j = 0; j < J; ++j) {
            uint64_t off, cnt;
            part_of_buffer(c, w->n, j, &off, &cnt);
            int own = owner_local(c, j);
            for (int from = 0; from < N; ++from) {
                uint64_t po, pc;
                part(cnt, (uint64_t)N, (uint64_t)from, &po, &pc);
                for (int to = 0; to < N; ++to)
                    if (to != from) post(w, rank_of(c, from, own), rank_of(c, to, own), off + po, pc);
            }
        }
        for (int r = 0; r < w->P; ++r)
            for (size_t i = 0; i < w->inbox[r].len; ++i) overwrite(w, r, &w->inbox[r].v[i]);
        end_round(w);
    }

    /* stage 3: all-gather on the node group: each owner sends its part to
     * the other R-1 processes of its node. */
    if (w->round < max_rounds) {
        w->phase = PH_LANE_S3;
        for (int node = 0; node < N; ++node)
            for (int j = 0; j < J; ++j) {
                uint64_t off, cnt;
                part_of_buffer(c, w->n, j, &off, &cnt);
                int own = owner_local(c, j);
                for (int l = 0; l < R; ++l)
                    if (l != own) post(w, rank_of(c, node, own), rank_of(c, node, l), off, cnt);
            }
        for (int r = 0; r < w->P; ++r)
            for (size_t i = 0; i < w->inbox[r].len; ++i) overwrite(w, r, &w->inbox[r].v[i]);
        end_round(w);
    }
    free(ops);
    return w->failed ? 3 : 0;
}

/* ---- the shared-buffer model ("Multiple Processes Per GPU" subsection) --------
 * One buffer per GPU, N*G in all; the Q processes of a GPU all work on it, process q on the
 * slice that starts at (s / PPG) * l_r: here part q of a balanced split of n into Q.  Processes
 * with equal local rank q on all GPUs form new_comm (N*G members, member u = node*G + gpu). */

static int proc_rank(int G, int Q, int node, int gpu, int q)
{
    return (node * G + gpu) * Q + q;
}

/* "Standard Approach": every process calls the library all-reduce on its slice over new_comm;
 * the Q all-reduces run concurrently.  The library algorithm is a black box; it is taken to be
 * Algorithm 1, the standard choice for large buffers (Background section). */
static int run_shared_standard(world_t* w, int N, int G, int Q, int max_rounds)
{
    const int M = N * G; /* members of new_comm */
    for (int loop = 0; loop < 2; ++loop) {
        w->phase = loop == 0 ? PH_RING_RS : PH_RING_AG;
        for (int i = 0; i < M - 1 && w->round < max_rounds; ++i) {
            for (int q = 0; q < Q; ++q) {
                uint64_t so, sc, co, cc;
                part(w->n, (uint64_t)Q, (uint64_t)q, &so, &sc);
                for (int u = 0; u < M; ++u) {
                    int sp = loop == 0 ? imod(u - i, M) : imod(u + 1 - i, M);
                    part(sc, (uint64_t)M, (uint64_t)sp, &co, &cc);
                    post(w, u * Q + q, ((u + 1) % M) * Q + q, so + co, cc);
                }
            }
            for (int q = 0; q < Q; ++q)
                for (int u = 0; u < M; ++u) {
                    int me = u * Q + q;
                    const letter_t* le = letter_from(w, me, imod(u - 1, M) * Q + q);
                    if (!le) return 4;
                    if (loop == 0) {
                        char* mine = mem(w, me) + le->off * w->esz;
                        const void* two[2] = {mine, le->data};
                        sum_operands(w->dtype, w->op, mine, two, 2, le->cnt);
                    } else {
                        overwrite(w, me, le);
                    }
                }
            end_round(w);
        }
    }
    return w->failed ? 3 : 0;
}

/* "Multi-lane Approach": every process runs Algorithm 2 on its slice.  comm_group = the G
 * processes with local rank q on the node's GPUs, comm_lane = the N processes (node', gpu, q). */
static int run_shared_lane(world_t* w, int N, int G, int Q, int max_rounds)
{
    const void** ops = (const void**)malloc(sizeof(void*) * (size_t)(G > N ? G : N));
    if (!ops) return 3;
    /* stage 1: reduce-scatter of slice q on comm_group: GPU g's process receives chunk g */
    if (w->round < max_rounds) {
        w->phase = PH_LANE_S1;
        for (int node = 0; node < N; ++node)
            for (int q = 0; q < Q; ++q) {
                uint64_t so, sc, co, cc;
                part(w->n, (uint64_t)Q, (uint64_t)q, &so, &sc);
                for (int g = 0; g < G; ++g) {
                    part(sc, (uint64_t)G, (uint64_t)g, &co, &cc);
                    for (int from = 0; from < G; ++from)
                        if (from != g) post(w, proc_rank(G, Q, node, from, q), proc_rank(G, Q, node, g, q), so + co, cc);
                }
            }
        for (int node = 0; node < N; ++node)
            for (int q = 0; q < Q; ++q) {
                uint64_t so, sc, co, cc;
                part(w->n, (uint64_t)Q, (uint64_t)q, &so, &sc);
                for (int g = 0; g < G; ++g) {
                    part(sc, (uint64_t)G, (uint64_t)g, &co, &cc);
                    int me = proc_rank(G, Q, node, g, q);
                    char* mine = mem(w, me) + (so + co) * w->esz;
                    for (int from = 0; from < G; ++from) {
                        if (from == g) {
                            ops[from] = mine;
                        } else {
                            const letter_t* le = letter_from(w, me, proc_rank(G, Q, node, from, q));
                            if (!le) return 4;
                            ops[from] = le->data;
                        }
                    }
                    sum_operands(w->dtype, w->op, mine, ops, G, cc);
                }
            }
        end_round(w);
    }
    /* stage 2: all-reduce of the owned chunk on comm_lane (reduce-scatter of N pieces, then
     * all-gather), operands in ascending node order */
    for (int half = 0; half < 2; ++half) {
        if (w->round >= max_rounds) break;
        w->phase = half == 0 ? PH_LANE_S2A : PH_LANE_S2B;
        for (int q = 0; q < Q; ++q) {
            uint64_t so, sc, co, cc, po, pc;
            part(w->n, (uint64_t)Q, (uint64_t)q, &so, &sc);
            for (int g = 0; g < G; ++g) {
                part(sc, (uint64_t)G, (uint64_t)g, &co, &cc);
                for (int from = 0; from < N; ++from)
                    for (int to = 0; to < N; ++to) {
                        if (to == from) continue;
                        /* first half: piece `to` goes to its reducer; second half: the reduced
                         * piece `from` goes to everybody else */
                        part(cc, (uint64_t)N, (uint64_t)(half == 0 ? to : from), &po, &pc);
                        post(w, proc_rank(G, Q, from, g, q), proc_rank(G, Q, to, g, q), so + co + po, pc);
                    }
            }
        }
        if (half == 0) {
            for (int q = 0; q < Q; ++q) {
                uint64_t so, sc, co, cc, po, pc;
                part(w->n, (uint64_t)Q, (uint64_t)q, &so, &sc);
                for (int g = 0; g < G; ++g) {
                    part(sc, (uint64_t)G, (uint64_t)g, &co, &cc);
                    for (int node = 0; node < N; ++node) {
                        part(cc, (uint64_t)N, (uint64_t)node, &po, &pc);
                        int me = proc_rank(G, Q, node, g, q);
                        char* mine = mem(w, me) + (so + co + po) * w->esz;
                        for (int from = 0; from < N; ++from) {
                            if (from == node) {
                                ops[from] = mine;
                            } else {
                                const letter_t* le = letter_from(w, me, proc_rank(G, Q, from, g, q));
                                if (!le) return 4;
                                ops[from] = le->data;
                            }
                        }
                        sum_operands(w->dtype, w->op, mine, ops, N, pc);
                    }
                }
            }
        } else {
            for (int r = 0; r < w->P; ++r)
                for (size_t i = 0; i < w->inbox[r].len; ++i) overwrite(w, r, &w->inbox[r].v[i]);
        }
        end_round(w);
    }
    /* stage 3: all-gatherv of slice q on comm_group */
    if (w->round < max_rounds) {
        w->phase = PH_LANE_S3;
        for (int node = 0; node < N; ++node)
            for (int q = 0; q < Q; ++q) {
                uint64_t so, sc, co, cc;
                part(w->n, (uint64_t)Q, (uint64_t)q, &so, &sc);
                for (int g = 0; g < G; ++g) {
                    part(sc, (uint64_t)G, (uint64_t)g, &co, &cc);
                    for (int to = 0; to < G; ++to)
                        if (to != g) post(w, proc_rank(G, Q, node, g, q), proc_rank(G, Q, node, to, q), so + co, cc);
                }
            }
        for (int r = 0; r < w->P; ++r)
            for (size_t i = 0; i < w->inbox[r].len; ++i) overwrite(w, r, &w->inbox[r].v[i]);
        end_round(w);
    }
    free(ops);
    return w->failed ? 3 : 0;
}

/*
 * Run a schedule over P = N*G*Q private buffers of n elements, in place.
 *   max_rounds < 0: run to the end; otherwise stop after that many rounds
 *   (ring: one round per loop iteration; lane: S1, S2a, S2b, S3 are one round
 *   each; lane with the ring inside: S1, then one round per ring iteration,
 *   then S3), so that tests can look at intermediate states.
 *   trace / trace_cap: optional log of every message; *trace_len receives the
 *   number of messages sent (which may exceed trace_cap).
 * Returns 0 on success.
 */
static int run_world(int shared, int op, int algo, int N, int G, int Q, uint64_t n, int dtype, void** bufs,
                     int max_rounds, oracle_msg_t* trace, uint64_t trace_cap, uint64_t* trace_len);

/* Same as oracle_allreduce / oracle_allreduce_shared with an operation other than the sum. */
int oracle_allreduce_op(int shared, int op, int algo, int N, int G, int Q, uint64_t n, int dtype, void** bufs,
                        int max_rounds, oracle_msg_t* trace, uint64_t trace_cap, uint64_t* trace_len)
{
    if (op < OP_SUM || op > OP_MIN) return 2;
    return run_world(shared, op, algo, N, G, Q, n, dtype, bufs, max_rounds, trace, trace_cap, trace_len);
}

int oracle_allreduce(int algo, int N, int G, int Q, uint64_t n, int dtype, void** bufs,
                     int max_rounds, oracle_msg_t* trace, uint64_t trace_cap, uint64_t* trace_len)
{
    return run_world(0, OP_SUM, algo, N, G, Q, n, dtype, bufs, max_rounds, trace, trace_cap, trace_len);
}

/* The shared-buffer model: bufs holds N*G buffers (index node*G + gpu) of n elements; P = N*G*Q
 * processes.  algo: ORACLE_RING = the "standard" multi-process all-reduce (Q concurrent rings
 * over new_comm); ORACLE_LANE_MULTIPROC = Algorithm 2 per process on its slice.  Every buffer
 * ends with the sum of the N*G buffers. */
int oracle_allreduce_shared(int algo, int N, int G, int Q, uint64_t n, int dtype, void** bufs,
                            int max_rounds, oracle_msg_t* trace, uint64_t trace_cap, uint64_t* trace_len)
{
    return run_world(1, OP_SUM, algo, N, G, Q, n, dtype, bufs, max_rounds, trace, trace_cap, trace_len);
}

static int run_world(int shared, int op, int algo, int N, int G, int Q, uint64_t n, int dtype, void** bufs,
                     int max_rounds, oracle_msg_t* trace, uint64_t trace_cap, uint64_t* trace_len)
{
    if (N < 1 || G < 1 || Q < 1 || !bufs) return 1;
    if (dtype < ORACLE_I32 || dtype > ORACLE_F64) return 2;
    world_t w;
    memset(&w, 0, sizeof w);
    w.P = N * G * Q;
    w.dtype = dtype;
    w.op = op;
    w.esz = elem_size(dtype);
    w.n = n;
    w.buf = bufs;
    w.share = shared ? Q : 1;
    w.inbox = (inbox_t*)calloc((size_t)w.P, sizeof(inbox_t));
    if (!w.inbox) return 3;
    w.trace = trace;
    w.trace_cap = trace ? trace_cap : 0;
    int limit = max_rounds < 0 ? 0x7fffffff : max_rounds;
    int rc;
    if (shared) {
        if (algo == ORACLE_RING)
            rc = run_shared_standard(&w, N, G, Q, limit);
        else if (algo == ORACLE_LANE_MULTIPROC)
            rc = run_shared_lane(&w, N, G, Q, limit);
        else
            rc = 2;
    } else if (algo == ORACLE_RING) {
        rc = run_ring(&w, limit);
    } else if (algo == ORACLE_RECURSIVE_DOUBLING) {
        rc = run_recursive_doubling(&w, limit);
    } else if (algo == ORACLE_RABENSEIFNER) {
        rc = run_rabenseifner(&w, limit);
    } else if (algo == ORACLE_LANE || algo == ORACLE_LANE_MULTIPROC || algo == ORACLE_LANE_RING ||
               algo == ORACLE_LANE_MULTIPROC_RING) {
        lane_cfg_t c = {N, G, Q, algo == ORACLE_LANE_MULTIPROC || algo == ORACLE_LANE_MULTIPROC_RING,
                        algo == ORACLE_LANE_RING || algo == ORACLE_LANE_MULTIPROC_RING};
        rc = run_lane(&w, &c, limit);
    } else {
        rc = 2;
    }
    for (int r = 0; r < w.P; ++r) {
        for (size_t i = 0; i < w.inbox[r].len; ++i) free(w.inbox[r].v[i].data);
        free(w.inbox[r].v);
    }
    free(w.inbox);
    if (trace_len) *trace_len = w.trace_len;
    return rc;
}
