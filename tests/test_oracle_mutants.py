"""The pins are only worth something if a plausible mistake in the oracle fails one of them.

Each case plants ONE mistake in a copy of the oracle's C source (on the CPU), builds it,
swaps it in for the real library and runs the pin tests: at least one must fail.
"""
import ctypes
import os
import subprocess

import pytest

import oracle
from tests import test_oracle_extras as te
from tests import test_oracle_plan as tp
from tests import test_oracle_score as ts
from tests import test_oracle_select_compact as tc

SRC = os.path.join(os.path.dirname(oracle.__file__), "zp_oracle.c")

MUTANTS = [
    ("mask direction", "j > Tv - w + u) { a[t] = -INFINITY", "j < Tv - w + u) { a[t] = -INFINITY"),
    ("mask off by one", "j > Tv - w + u) { a[t] = -INFINITY", "j >= Tv - w + u) { a[t] = -INFINITY"),
    ("head grouping", "q_row(s, l, bt->q_slot[n], u, h * G + g)", "q_row(s, l, bt->q_slot[n], u, g * s->h_kv + h)"),
    ("sum over group instead of max", "if (p > mx) mx = p;", "mx += p;"),
    ("mean divisor", "S[t] = acc / (double)w;", "S[t] = acc / (double)G;"),
    ("logit scale", "1.0 / sqrt((double)d);", "1.0 / (double)d;"),
    ("no scale", "a[t] = acc * inv_sqrt_d;", "a[t] = acc;"),
    ("slot order inside a block", "size_t ko = kv_row(s, l, tbl[t / b], t % b, h);\n                    double acc = 0.0;\n                    for (int c = 0; c < d; c++) acc += elem(Q",
     "size_t ko = kv_row(s, l, tbl[t / b], b - 1 - t % b, h);\n                    double acc = 0.0;\n                    for (int c = 0; c < d; c++) acc += elem(Q"),
    ("block table ignored", "size_t ko = kv_row(s, l, tbl[t / b], t % b, h);\n                    double acc = 0.0;\n                    for (int c = 0; c < d; c++) acc += elem(Q",
     "size_t ko = kv_row(s, l, t / b, t % b, h);\n                    double acc = 0.0;\n                    for (int c = 0; c < d; c++) acc += elem(Q"),
    ("softmax without max shift and normaliser", "a[t] = exp(a[t] - m) / z;", "a[t] = exp(a[t] - m);"),
    ("stale positions scored", "if (j < 0 || j > Tv - w + u)", "if (j > Tv - w + u)"),
    ("tie break to higher position", "return (a->t > b->t) - (a->t < b->t);", "return (a->t < b->t) - (a->t > b->t);"),
    ("ascending instead of descending", "if (a->s > b->s) return -1;\n    if (a->s < b->s) return 1;", "if (a->s > b->s) return 1;\n    if (a->s < b->s) return -1;"),
    ("window one short", "else if (j >= Tv - w) v = INFINITY;", "else if (j > Tv - w) v = INFINITY;"),
    ("window not filled", "else if (j >= Tv - w) v = INFINITY;", ""),
    ("nan not demoted", "if (v != v) v = -INFINITY;", ""),
    ("stale not demoted", "if (j < 0) v = -INFINITY;            /* stale */\n            else if", "if"),
    ("compaction writes the wrong slot", "kv_row(s, l, dst[r / b], r % b, h)", "kv_row(s, l, dst[r / b], (r + 1) % b, h)"),
    ("compaction reads without snapshot order", "tbl[idx[r] / b], idx[r] % b, h) * esize", "tbl[idx[r] % b], idx[r] / b % b, h) * esize"),
    ("V not moved", "memcpy((char *)V + to, snapV + (size_t)r * rowb, rowb);", ""),
    ("targets ignore dst_table", "bt->dst_table ? bt->dst_table + (size_t)n * (bt->N_max - 1) : tbl;", "tbl;"),
    ("private blocks redirected too", "if (refcnt[tbl[i]] > 1) {\n                if (used >= n_free_in)", "if (refcnt[tbl[i]] >= 1) {\n                if (used >= n_free_in)"),
    ("reserved block released", "} else if (i >= N_max - 1 && i != res) {", "} else if (i >= N_max - 1) {"),
    ("shared judged on live counts", "if (refcnt[p] > 1) {               /* shared at batch start", "if (cnt[p] > 1) {               /* shared at batch start"),
    ("targets released", "} else if (i >= N_max - 1 && i != res) {", "} else if (i != res) {"),
    ("decode attention without scale", "a[t] = acc / sqrt((double)d);", "a[t] = acc;"),
    ("history used on a first compression", "const int has_hist = ex->compressed && ex->compressed[n];", "const int has_hist = 1;"),
    ("history applied to the last block too", "if (has_hist && t < vl) {", "if (has_hist) {"),
    ("decay forgotten", "double old = ex->alpha * (double)ex->F[fi];", "double old = (double)ex->F[fi];"),
    ("cache stores the pooled score", "                ex->F[fi] = (float)v;\n                S[t] = v;", "                S[t] = v;"),
    ("pool window one short", "for (int q = j - r; q <= j + r; q++)", "for (int q = j - r; q < j + r; q++)"),
    ("first-only switch ignored", "if (ex->pool_kernel > 1 && !(ex->pool_first_only && has_hist)) {", "if (ex->pool_kernel > 1) {"),
    ("first-only switch inverted", "if (ex->pool_kernel > 1 && !(ex->pool_first_only && has_hist)) {", "if (ex->pool_kernel > 1 && !(ex->pool_first_only && !has_hist)) {"),
    ("first instead of last entry above p", "for (int r = b - 1; r >= 0; r--)\n                        if (Cm", "for (int r = 0; r < b; r++)\n                        if (Cm"),
    ("diagonal kept", "if (r != c && live_index(tr", "if (live_index(tr"),
    ("row sums not divided by the length", "tmp[j] = acc / (double)Tv;", "tmp[j] = acc;"),
    ("temperature ignored", "z += exp(tmp[j] / ex->tau - m);", "z += exp(tmp[j] - m);"),
    ("redundancy added instead of subtracted", "S[pos[j]] -= ex->lambda", "S[pos[j]] += ex->lambda"),
    ("similarity across blocks", "size_t ro = kv_row(s, l, tbl[i], r, h), co = kv_row(s, l, tbl[i], c, h);", "size_t ro = kv_row(s, l, tbl[i], r, h), co = kv_row(s, l, tbl[(i + 1) % N], c, h);"),
    ("global cache not moved", "for (int r = 0; r < k; r++) F[f_index(s, l, dst[r / b], r % b, h)] = snap[r];", ""),
]


def pins():
    out = [
        lambda: ts.test_g1_is_column_mean_of_textbook_causal_attention(False),
        lambda: ts.test_g1_is_column_mean_of_textbook_causal_attention(True),
        ts.test_w1_is_max_over_group_of_single_softmax_rows,
        ts.test_gqa_grouping_and_reduction_order_bruteforce,
        ts.test_identical_keys_closed_form_pins_mask_direction_and_offsets,
        ts.test_one_hot_keys_closed_form,
        ts.test_invariants_sum_range_and_window_mass,
        ts.test_block_table_permutation_invariance,
        ts.test_stale_gap_equals_packed_sequence,
        tc.test_window_always_kept_and_counts_inside_k,
        tc.test_ties_go_to_lower_position,
        tc.test_nan_inf_and_negative_zero,
        tc.test_stale_positions_never_kept_and_window_follows_live_sequence,
        lambda: tc.test_matches_stable_argsort_and_dominance(0),
        lambda: tc.test_gather_form_equals_in_place_sequential_move(0, False),
        tc.test_logical_content_after_compaction_and_untouched_bytes,
        tc.test_compaction_into_separate_targets_leaves_sources_alone,
        tp.test_first_figure_structure,
        tp.test_shared_prefix_shorter_than_budget,
        tp.test_shared_prefix_covering_all_targets,
        tp.test_two_sharers_in_one_batch_release_the_prefix_together,
        lambda: tp.test_conservation_laws(0),
        tp.test_decode_attention_is_textbook_softmax_attention,
        te.test_global_score_first_compression_only_stores,
        te.test_global_score_decayed_max_on_the_live_prefix_only,
        lambda: te.test_pooling_is_library_maxpool1d_along_the_live_sequence(3),
        te.test_pooling_at_the_first_compression_only,
        lambda: te.test_lightning_redundancy_matches_matrix_formulation(0, 0.2),
        te.test_redundancy_closed_forms,
        te.test_order_of_the_refinements,
        te.test_global_cache_moves_with_the_kept_entries,
    ]
    return out


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(name, old, new, tmp_path, monkeypatch):
    text = open(SRC).read()
    assert text.count(old) >= 1, "mutation site not found: " + name
    src = tmp_path / "mutant.c"
    src.write_text(text.replace(old, new))
    lib = tmp_path / "mutant.so"
    subprocess.check_call(["gcc", "-O1", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-w", "-o", str(lib), str(src), "-lm"])
    mutant = ctypes.CDLL(str(lib))
    oracle._load()
    monkeypatch.setattr(oracle, "_lib", mutant)
    caught = 0
    for pin in pins():
        try:
            pin()
        except (AssertionError, ValueError, MemoryError):
            caught += 1
    assert caught >= 1, "no pin noticed the planted mistake: " + name
