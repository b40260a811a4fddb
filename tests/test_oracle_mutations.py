"""Are the pins sharp?  Each case plants one plausible mistake in a copy of the oracle's C source
(a wrong index, sign, order, bound or rounding rule), builds it, and requires that at least one
pin of tests/test_oracle_pins.py fails on the broken build.  CPU only."""
import os
import subprocess
import sys

import pytest

import oracle as oracle_pkg
import test_oracle_pins as pins

SRC = os.path.join(os.path.dirname(oracle_pkg.__file__), "la_oracle.c")

# (name, text in la_oracle.c, replacement)
MUTATIONS = [
    ("split_remainder_dropped", "*cnt = q + (i < rem ? 1 : 0);", "*cnt = q;"),
    ("split_offset_wrong", "*off = i * q + (i < rem ? i : rem);", "*off = i * q;"),
    ("ring_rs_walks_forward", "int sp = imod(r - i, P);", "int sp = imod(r + i, P);"),
    ("ring_ag_starts_at_r", "int sp = imod(r + 1 - i, P);", "int sp = imod(r - i, P);"),
    ("ring_one_round_short", "for (int i = 0; i < P - 1 && w->round < max_rounds; ++i) {\n        for (int r = 0; r < P; ++r) {\n            int sp = imod(r + 1",
     "for (int i = 0; i < P - 2 && w->round < max_rounds; ++i) {\n        for (int r = 0; r < P; ++r) {\n            int sp = imod(r + 1"),
    ("ring_sends_to_predecessor", "post(w, r, (r + 1) % P, D[sp], cnt[sp]);\n        }\n        for (int r = 0; r < P; ++r) {\n            const letter_t* l = letter_from(w, r, imod(r - 1, P));\n            if (!l) return 4;\n            char* own",
     "post(w, r, imod(r - 1, P), D[sp], cnt[sp]);\n        }\n        for (int r = 0; r < P; ++r) {\n            const letter_t* l = letter_from(w, r, (r + 1) % P);\n            if (!l) return 4;\n            char* own"),
    ("s1_owner_first", "                for (int l = 0; l < R; ++l) {\n                    if (l == own) {\n                        ops[l] = mine;",
     "                ops[0] = mine;\n                for (int l = 0; l < R; ++l) {\n                    if (l == own) {\n                        if (l) ops[l] = ops[0]; if (l) ops[0] = mine;"),
    ("s1_drops_last_operand", "sum_operands(w->dtype, w->op, mine, ops, R, cnt);", "sum_operands(w->dtype, w->op, mine, ops, R > 1 ? R - 1 : R, cnt);"),
    ("s2a_piece_index_swapped", "part(cnt, (uint64_t)N, (uint64_t)to, &po, &pc);\n                    if (to != from) post",
     "part(cnt, (uint64_t)N, (uint64_t)from, &po, &pc);\n                    if (to != from) post"),
    ("s2a_descending_order", "ops[from] = le->data;", "ops[N - 1 - from] = le->data;"),
    ("s2b_skipped", "w->phase = PH_LANE_S2B;\n        for (int j = 0; j < J; ++j) {", "w->phase = PH_LANE_S2B;\n        for (int j = 0; j < 0; ++j) {"),
    ("s3_misses_last_local", "for (int l = 0; l < R; ++l)\n                    if (l != own) post(w, rank_of(c, node, own), rank_of(c, node, l), off, cnt);",
     "for (int l = 0; l < R - 1; ++l)\n                    if (l != own) post(w, rank_of(c, node, own), rank_of(c, node, l), off, cnt);"),
    ("proc_major_split", "*off = lo + so;", "*off = (uint64_t)q * (n / (uint64_t)c->Q) + so + lo / (uint64_t)c->Q;"),
    ("lane_owner_not_leader", "return c->split_procs ? j : j * c->Q;", "return c->split_procs ? j : j * c->Q + (c->Q - 1);"),
    ("inner_ring_walks_forward", "int sp = loop == 0 ? imod(v - i, N) : imod(v + 1 - i, N);", "int sp = loop == 0 ? imod(v + i, N) : imod(v + 1 - i, N);"),
    ("inner_ring_gather_starts_at_v", "int sp = loop == 0 ? imod(v - i, N) : imod(v + 1 - i, N);", "int sp = loop == 0 ? imod(v - i, N) : imod(v - i, N);"),
    ("inner_ring_pieces_of_whole_buffer", "part(cnt, (uint64_t)N, (uint64_t)sp, &po, &pc);\n                        post(w, rank_of(c, v, own), rank_of(c, (v + 1) % N, own), off + po, pc);",
     "part(w->n, (uint64_t)N, (uint64_t)sp, &po, &pc);\n                        post(w, rank_of(c, v, own), rank_of(c, (v + 1) % N, own), po, pc);"),
    ("inner_ring_one_round_short", "for (int i = 0; i < N - 1 && w->round < max_rounds; ++i) {\n                for (int j = 0; j < J; ++j) {\n                    uint64_t off, cnt, po, pc;",
     "for (int i = 0; i < N - 2 + loop && w->round < max_rounds; ++i) {\n                for (int j = 0; j < J; ++j) {\n                    uint64_t off, cnt, po, pc;"),
    ("shared_standard_gpu_major_slices", "part(sc, (uint64_t)M, (uint64_t)sp, &co, &cc);\n                    post(w, u * Q + q, ((u + 1) % M) * Q + q, so + co, cc);",
     "part(w->n, (uint64_t)M, (uint64_t)sp, &co, &cc); part(cc, (uint64_t)Q, (uint64_t)q, &so, &sc);\n                    post(w, u * Q + q, ((u + 1) % M) * Q + q, so + co, sc);"),
    ("shared_standard_crosses_local_ranks", "post(w, u * Q + q, ((u + 1) % M) * Q + q, so + co, cc);", "post(w, u * Q + q, ((u + 1) % M) * Q + (q + 1) % Q, so + co, cc);"),
    ("shared_lane_s1_descending", "                            ops[from] = le->data;\n                        }\n                    }\n                    sum_operands(w->dtype, w->op, mine, ops, G, cc);",
     "                            ops[from] = le->data;\n                        }\n                    }\n                    if (G > 1) { const void* t0 = ops[0]; ops[0] = ops[G - 1]; ops[G - 1] = t0; }\n                    sum_operands(w->dtype, w->op, mine, ops, G, cc);"),
    ("shared_lane_gather_skips_last_gpu", "for (int to = 0; to < G; ++to)\n                        if (to != g) post(w, proc_rank(G, Q, node, g, q), proc_rank(G, Q, node, to, q), so + co, cc);",
     "for (int to = 0; to < G - 1; ++to)\n                        if (to != g) post(w, proc_rank(G, Q, node, g, q), proc_rank(G, Q, node, to, q), so + co, cc);"),
    ("shared_lane_piece_of_wrong_member", "part(cc, (uint64_t)N, (uint64_t)(half == 0 ? to : from), &po, &pc);", "part(cc, (uint64_t)N, (uint64_t)(half == 0 ? from : to), &po, &pc);"),
    ("f16_ties_away", "if (lost > 0x1000u || (lost == 0x1000u && (kept & 1u))) kept += 1; /* a carry", "if (lost >= 0x1000u) kept += 1; /* a carry"),
    ("f16_overflow_saturates", "if (kept >= 0x7c00u) kept = 0x7c00u;", "if (kept >= 0x7c00u) kept = 0x7bffu;"),
    ("f16_subnormal_shift_off_by_one", "uint32_t full = 0x800000u | m, shift = 126u - e;", "uint32_t full = 0x800000u | m, shift = 125u - e;"),
    ("f16_subnormal_truncates", "if (lost > half || (lost == half && (kept & 1u))) kept += 1;", "if (lost > half + half) kept += 1;"),
    ("f16_widen_wrong_bias", "u = sign | ((e + 112u) << 23) | (m << 13); /* normal", "u = sign | ((e + 111u) << 23) | (m << 13); /* normal"),
    ("f16_rounds_every_add", "for (int t = 1; t < k; ++t) s = op_f32(op, s, f16_widen(((const uint16_t*)ops[t])[i]));",
     "for (int t = 1; t < k; ++t) s = f16_widen(f16_round(op_f32(op, s, f16_widen(((const uint16_t*)ops[t])[i]))));"),
    ("max_nan_wins", "if (b != b) return a;\n    if (a != a) return b;\n    if (a < b) return b;", "if (b != b) return b;\n    if (a != a) return a;\n    if (a < b) return b;"),
    ("max_ignores_signed_zero", "return (ua >> 63) ? b : a;", "return a;"),
    ("min_is_max", "if (b < a) return b;\n    if (a == b && a == 0.0) { /* take -0", "if (a < b) return b;\n    if (a == b && a == 0.0) { /* take -0"),
    ("int_max_compares_unsigned", "case OP_MAX: return (int32_t)b > (int32_t)a ? b : a;", "case OP_MAX: return b > a ? b : a;"),
    ("int_prod_not_wrapping", "case OP_PROD: return a * b;\n    case OP_MAX: return (int32_t)b > (int32_t)a ? b : a;\n    default: return (int32_t)b < (int32_t)a ? b : a;",
     "case OP_PROD: { int64_t z = (int64_t)(int32_t)a * (int32_t)b; return (uint32_t)(z > 2147483647 ? 2147483647 : z < -2147483648LL ? -2147483648LL : z); }\n    case OP_MAX: return (int32_t)b > (int32_t)a ? b : a;\n    default: return (int32_t)b < (int32_t)a ? b : a;"),
    ("f64_in_single", "double s = ((const double*)ops[0])[i];\n            for (int t = 1; t < k; ++t) s = op_f64(op, s, ((const double*)ops[t])[i]);",
     "float s = (float)((const double*)ops[0])[i];\n            for (int t = 1; t < k; ++t) s = op_f32(op, s, (float)((const double*)ops[t])[i]);"),
    ("rd_partner_at_fixed_distance", "for (int r = 0; r < P; ++r) post(w, r, r ^ (1 << s), 0, w->n);", "for (int r = 0; r < P; ++r) post(w, r, r ^ 1, 0, w->n);"),
    ("rd_one_round_short", "for (int s = 0; s < L && w->round < max_rounds; ++s) {\n        for (int r = 0; r < P; ++r) post(w, r, r ^ (1 << s), 0, w->n);",
     "for (int s = 0; s < L - 1 && w->round < max_rounds; ++s) {\n        for (int r = 0; r < P; ++r) post(w, r, r ^ (1 << s), 0, w->n);"),
    ("rab_upper_rank_keeps_first_half", "part(cnt[r * (L + 1) + s], 2, (r & d) ? 1 : 0, &o, &c);", "part(cnt[r * (L + 1) + s], 2, (r & d) ? 0 : 1, &o, &c);"),
    ("rab_starts_at_distance_one", "int d = P >> (s + 1);\n        for (int r = 0; r < P; ++r) {\n            int p = r ^ d; /* send", "int d = 1 << s;\n        for (int r = 0; r < P; ++r) {\n            int p = r ^ d; /* send"),
    ("rab_sends_own_half", "post(w, r, p, lo[p * (L + 1) + s + 1], cnt[p * (L + 1) + s + 1]);", "post(w, r, p, lo[r * (L + 1) + s + 1], cnt[r * (L + 1) + s + 1]);"),
    ("rab_gather_skips_last_round", "for (int s = L - 1; s >= 0 && w->round < max_rounds; --s) {", "for (int s = L - 1; s >= 1 && w->round < max_rounds; --s) {"),
    ("rank_numbering_gpu_minor", "return node * c->G * c->Q + local;", "return local * c->N + node;"),
    ("bf16_truncates", "if (lost > 0x8000u)\n        kept += 1;", "if (lost > 0xffffu)\n        kept += 1;"),
    ("bf16_ties_away", "else if (lost == 0x8000u && (kept & 1u))", "else if (lost == 0x8000u)"),
    ("bf16_rounds_every_add", "for (int t = 1; t < k; ++t) s = op_f32(op, s, bf16_widen(((const uint16_t*)ops[t])[i]));",
     "for (int t = 1; t < k; ++t) s = bf16_widen(bf16_round(op_f32(op, s, bf16_widen(((const uint16_t*)ops[t])[i]))));"),
    ("f32_accumulates_in_double", "float s = ((const float*)ops[0])[i];\n            for (int t = 1; t < k; ++t) s = op_f32(op, s, ((const float*)ops[t])[i]);",
     "double s = ((const float*)ops[0])[i];\n            for (int t = 1; t < k; ++t) s = op_f64(op, s, ((const float*)ops[t])[i]);"),
    ("int_saturates", "case OP_SUM: return a + b;\n    case OP_PROD: return a * b;\n    case OP_MAX: return (int32_t)b > (int32_t)a ? b : a;",
     "case OP_SUM: { int64_t z = (int64_t)(int32_t)a + (int32_t)b; return (uint32_t)(z > 2147483647 ? 2147483647 : z < -2147483648LL ? -2147483648LL : z); }\n    case OP_PROD: return a * b;\n    case OP_MAX: return (int32_t)b > (int32_t)a ? b : a;"),
    ("definition_skips_rank0", "for (int p = 0; p < P; ++p) s += ((const int32_t*)in[p])[i];", "for (int p = 1; p < P; ++p) s += ((const int32_t*)in[p])[i];"),
    ("definition_float_in_single", "double s = as_double(dtype, in[0], i);\n            for (int p = 1; p < P; ++p) s = op_f64(op, s, as_double(dtype, in[p], i));",
     "float s = (float)as_double(dtype, in[0], i);\n            for (int p = 1; p < P; ++p) s = (float)op_f64(op, s, as_double(dtype, in[p], i));"),
    ("reduce_segments_ignores_dst", "sum_operands(dtype, op, (char*)dst + o * e, ops, k + 1, seg_len);", "sum_operands(dtype, op, (char*)dst + o * e, ops + (k > 0), k > 0 ? k : 1, seg_len);"),
    ("overwrite_wrong_offset", "memcpy(mem(w, at) + l->off * w->esz, l->data, l->cnt * w->esz);", "memcpy(mem(w, at) + (l->off ? l->off - 1 : 0) * w->esz, l->data, l->cnt * w->esz);"),
    ("shared_buffer_of_wrong_gpu", "return (char*)w->buf[rank / w->share];", "return (char*)w->buf[w->share > 1 ? rank % (w->P / w->share) : rank];"),
]


def pin_calls(o):
    """every pin, bound to oracle build `o`, cheapest first"""
    calls = [
        lambda: pins.test_part_is_numpy_array_split(o),
        lambda: pins.test_bf16_round_closed_forms(o),
        lambda: pins.test_bf16_round_matches_torch_on_random_bit_patterns(o),
        lambda: pins.test_bf16_widen_all_patterns(o),
        lambda: pins.test_definition_int32_vs_python_integers_with_wrap(o),
        lambda: pins.test_definition_float_vs_fsum(o),
        lambda: pins.test_golden_ring_three_ranks_cancellation(o),
        lambda: pins.test_golden_lane_two_by_two_cancellation(o),
        lambda: pins.test_bf16_rounds_once_per_reduce_step(o),
        lambda: pins.test_ring_order_is_chunk_owner_first_then_successors(o),
        lambda: pins.test_lane_order_is_node_sums_then_across_nodes(o),
        lambda: pins.test_ring_message_pattern(o),
        lambda: pins.test_ring_after_first_loop_rank_owns_next_chunk(o),
        lambda: pins.test_lane_stage_boundaries(o, "lane"),
        lambda: pins.test_lane_stage_boundaries(o, "lane_multiproc"),
        lambda: pins.test_lane_message_shapes(o),
        lambda: pins.test_reduce_segments_vs_numpy(o),
        lambda: pins.test_lane_equals_lane_multiproc_when_one_process_per_gpu(o),
        lambda: pins.test_lane_ring_is_the_flat_ring_when_every_node_has_one_rank(o),
        lambda: pins.test_lane_ring_order_node_sums_walk_the_ring(o),
        lambda: pins.test_lane_ring_messages_and_boundaries(o),
        lambda: pins.test_f16_round_matches_numpy(o),
        lambda: pins.test_f16_widen_all_patterns(o),
        lambda: pins.test_operations_closed_forms(o),
        lambda: pins.test_definition_of_operations_vs_python(o),
        lambda: pins.test_f16_rounds_once_per_reduce_step(o),
        lambda: pins.test_schedules_with_operations_and_wide_types(o, "ring"),
        lambda: pins.test_schedules_with_operations_and_wide_types(o, "lane_multiproc"),
        lambda: pins.test_recursive_doubling_messages_and_order(o),
        lambda: pins.test_rabenseifner_messages_halve_and_order(o),
        lambda: pins.test_small_message_algorithms_bruteforce(o, "recursive_doubling"),
        lambda: pins.test_small_message_algorithms_bruteforce(o, "rabenseifner"),
        lambda: pins.test_shared_model_with_one_process_per_gpu_is_the_private_model(o),
        lambda: pins.test_shared_standard_messages_scale_with_processes_per_gpu(o),
        lambda: pins.test_shared_lane_stages_and_order(o),
        lambda: pins.test_shared_bruteforce_every_small_topology(o, "ring"),
        lambda: pins.test_shared_bruteforce_every_small_topology(o, "lane_multiproc"),
    ]
    for algo in pins.ALGOS:
        for topo in ((2, 1, 1), (1, 2, 1), (1, 1, 2)):
            calls.append(lambda a=algo, t=topo: pins.test_two_ranks_is_one_ieee_add(o, a, t))
        calls.append(lambda a=algo: pins.test_bruteforce_int32_every_small_topology(o, a))
    return calls


@pytest.mark.parametrize("name,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(tmp_path, name, old, new):
    text = open(SRC).read()
    assert text.count(old) >= 1, f"mutation {name}: anchor text not found in la_oracle.c"
    src = tmp_path / "mutant.c"
    src.write_text(text.replace(old, new, 1))
    lib = str(tmp_path / "libmutant.so")
    subprocess.run(["gcc", "-O2", "-std=c99", "-fno-fast-math", "-ffp-contract=off", "-fopenmp", "-fPIC",
                    "-shared", "-w", "-o", lib, str(src)], check=True)
    # a broken build may read or write out of bounds: run its pins in a child process
    code = (
        "import sys; sys.path[:0] = %r\n"
        "import oracle, test_oracle_mutations as m\n"
        "o = oracle.Oracle(%r)\n"
        "for call in m.pin_calls(o):\n"
        "    try:\n"
        "        call()\n"
        "    except (AssertionError, RuntimeError):\n"
        "        sys.exit(3)\n"
        "sys.exit(0)\n"
    ) % ([os.path.dirname(os.path.dirname(SRC)), os.path.dirname(__file__)], lib)
    try:
        rc = subprocess.run([sys.executable, "-c", code], capture_output=True, timeout=300).returncode
    except subprocess.TimeoutExpired:
        rc = 124  # a build that corrupts memory may also hang: the child is killed, the mistake is noticed
    assert rc != 0, f"no pin notices the planted mistake {name!r}"


def test_unmutated_source_passes_the_same_calls(oracle):
    for call in pin_calls(oracle):
        call()
