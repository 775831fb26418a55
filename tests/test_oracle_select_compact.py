"""Pins for the oracle's selection and compaction steps.

Selection (Method, "The Compression Process Pipeline": window gets +inf, top-k kept) is
pinned by a stable argsort, an O(T^2) dominance check and hand-made tie cases.
Compaction (appendix "KV Cache Compression") is pinned by a sequential in-place move
that keeps no snapshot (the oracle gathers from one), plus whole-pool byte equality
and idempotence.
"""
import numpy as np
import pytest

import oracle
from tests.util import random_problem


def live_positions(N, b, vl):
    return list(range(vl)) + list(range((N - 1) * b, N * b))


def brute_select(S, N, b, w, k, vl):
    """Stable argsort of the filled scores, first k, ascending."""
    T = N * b
    live = live_positions(N, b, vl)
    v = np.full(T, -np.inf, dtype=np.float32)
    v[live] = np.where(np.isnan(S[live]), -np.inf, S[live])
    v[live[-w:]] = np.inf
    order = np.argsort(-v, kind="stable")     # descending score, ties by ascending position
    return np.sort(order[:k]), v


def run_select(S_rows, *, b, N_max, w, keep=None, N=None, vl=None):
    """Oracle selection on hand-made score rows for one (request, layer) with len(S_rows) heads."""
    H = len(S_rows)
    N = N_max if N is None else N
    p = random_problem(0, h_kv=H, G=1, d=4, b=b, N_max=N_max, w=w, extra_blocks=N - N_max)
    if keep is not None:
        p.keep = np.array(keep, dtype=np.int32).reshape(1, 1, H)
    if vl is not None:
        p.valid_len = np.array(vl, dtype=np.int32).reshape(1, 1, H)
    S = np.array(S_rows, dtype=np.float32).reshape(1, 1, H, N * b)
    return oracle.select(p, S)


@pytest.mark.parametrize("seed", range(6))
def test_matches_stable_argsort_and_dominance(seed):
    rng = np.random.default_rng(seed)
    b, N_max, w, N = 4, 4, 3, 6
    H = 3
    S = rng.random((H, N * b)).astype(np.float32)
    S[:, rng.integers(0, N * b, 5)] = 0.5          # exact ties
    keep = [rng.integers(w, (N_max - 1) * b + 1) for _ in range(H)]
    idx, ln = run_select(S, b=b, N_max=N_max, w=w, keep=keep, N=N)
    for h in range(H):
        want, filled = brute_select(S[h], N, b, w, keep[h], (N - 1) * b)
        got = idx[0, 0, h]
        assert ln[0, 0, h] == keep[h]
        assert np.array_equal(got[: keep[h]], want) and (got[keep[h]:] == -1).all()
        kept = set(want.tolist())
        for a in kept:                              # every kept (score, -pos) dominates every dropped one
            for d_ in set(range(N * b)) - kept:
                assert (filled[a], -a) > (filled[d_], -d_)


def test_window_always_kept_and_counts_inside_k():
    b, N_max, w = 4, 3, 2
    S = np.linspace(1.0, 0.0, 12, dtype=np.float32)[None]      # window (last two) has the lowest raw scores
    idx, ln = run_select(S, b=b, N_max=N_max, w=w, keep=[[2]])
    assert idx[0, 0, 0, :2].tolist() == [10, 11] and ln[0, 0, 0] == 2          # k = w: only the window
    idx, _ = run_select(S, b=b, N_max=N_max, w=w, keep=[[5]])
    assert idx[0, 0, 0, :5].tolist() == [0, 1, 2, 10, 11]                      # window + 3 best


def test_ties_go_to_lower_position():
    b, N_max, w = 4, 3, 1
    S = np.zeros((1, 12), dtype=np.float32)                    # all equal
    idx, _ = run_select(S, b=b, N_max=N_max, w=w, keep=[[4]])
    assert idx[0, 0, 0, :4].tolist() == [0, 1, 2, 11]
    S = np.array([[0.1, 0.9, 0.9, 0.9, 0.1, 0.9, 0, 0, 0, 0, 0, 0]], dtype=np.float32)
    idx, _ = run_select(S, b=b, N_max=N_max, w=w, keep=[[4]])
    assert idx[0, 0, 0, :4].tolist() == [1, 2, 3, 11]          # three of the four 0.9s, the lowest positions


def test_nan_inf_and_negative_zero():
    b, N_max, w = 4, 3, 1
    S = np.array([[np.nan, np.inf, -np.inf, 0.0, -0.0, 1e-40, -1.0, np.nan, 2.0, 3.0, 0.5, 0.25]], dtype=np.float32)
    idx, _ = run_select(S, b=b, N_max=N_max, w=w, keep=[[8]])
    want, _ = brute_select(S[0], 3, b, w, 8, 8)
    assert np.array_equal(idx[0, 0, 0, :8], want)
    # NaN ranks with -inf: never preferred over any finite score
    assert 0 not in idx[0, 0, 0, :8].tolist() and 7 not in idx[0, 0, 0, :8].tolist()
    # +0.0 and -0.0 compare equal: the tie goes to the lower position
    idx6, _ = run_select(S, b=b, N_max=N_max, w=w, keep=[[7]])
    assert 3 in idx6[0, 0, 0, :7].tolist() and 4 not in idx6[0, 0, 0, :7].tolist()


def test_stale_positions_never_kept_and_window_follows_live_sequence():
    b, N_max, w, N = 4, 3, 6, 5
    S = np.full((1, N * b), 0.5, dtype=np.float32)
    S[0, 8:16] = 9.0                                           # stale region has the best raw scores
    idx, ln = run_select(S, b=b, N_max=N_max, w=w, keep=[[7]], N=N, vl=[[8]])
    # live = [0,8) ++ [16,20); window = last 6 live entries = {6,7,16,17,18,19}; one more: position 0
    assert idx[0, 0, 0, :7].tolist() == [0, 6, 7, 16, 17, 18, 19] and ln[0, 0, 0] == 7


def test_full_budget_when_keep_absent():
    b, N_max, w, N = 4, 3, 2, 4
    rng = np.random.default_rng(5)
    S = rng.random((2, N * b)).astype(np.float32)
    idx, ln = run_select(S, b=b, N_max=N_max, w=w, N=N)
    assert (ln == 8).all() and (idx >= 0).all()
    for h in range(2):
        assert np.array_equal(idx[0, 0, h], brute_select(S[h], N, b, w, 8, 12)[0])


# ---------------------------------------------------------------- compaction

def in_place_sequential_move(K, V, tbl_src, tbl_dst, kept_mask, l, h, b):
    """Order-preserving removal done in place, one row at a time, with no snapshot (appendix "KV Cache Compression"):
    the kept logical positions are visited in ascending order and the r-th of them lands on logical row r of the
    targets.  Because it overwrites the pool while it still reads from it, it only agrees with a gather from a
    snapshot if no row is overwritten before it has been read, which is what the test below establishes."""
    src_addr = [(tbl_src[t // b], t % b) for t in range(len(tbl_src) * b)]     # logical position -> (physical block, slot)
    rank = 0
    for t in np.flatnonzero(kept_mask.reshape(-1)):
        blk, slot = src_addr[t]
        K[l, tbl_dst[rank // b], rank % b, h] = K[l, blk, slot, h]
        V[l, tbl_dst[rank // b], rank % b, h] = V[l, blk, slot, h]
        rank += 1
    return rank


@pytest.mark.parametrize("seed,bf16", [(0, False), (1, True), (2, False), (3, True)])
def test_gather_form_equals_in_place_sequential_move(seed, bf16):
    p = random_problem(seed, B=2, L=2, h_kv=2, G=2, d=8, b=4, N_max=4, w=2, bf16=bf16, num_blocks=[6, 4])
    rng = np.random.default_rng(seed)
    p.keep = rng.integers(2, 13, size=(2, 2, 2)).astype(np.int32)
    K0, V0 = p.K.copy(), p.V.copy()
    S = oracle.score(p)
    idx, ln = oracle.select(p, S.astype(np.float32))
    oracle.compact(p, idx, ln)
    Kr, Vr = K0.copy(), V0.copy()
    for n in range(2):
        N = int(p.num_blocks[n])
        for l in range(2):
            for h in range(2):
                tag = np.zeros((N, 4), dtype=np.int8)
                kept = idx[n, l, h, : ln[n, l, h]]
                tag[kept // 4, kept % 4] = 1
                moved = in_place_sequential_move(Kr, Vr, p.block_table[n, :N], p.block_table[n, :3], tag, l, h, 4)
                assert moved == ln[n, l, h] == p.keep[n, l, h]       # the paper's count: k reads and writes
    assert np.array_equal(p.K, Kr) and np.array_equal(p.V, Vr)        # whole pool, stale tails and bystanders included
    assert not np.array_equal(p.K, K0)


def test_logical_content_after_compaction_and_untouched_bytes():
    p = random_problem(7, B=1, L=1, h_kv=2, G=1, d=4, b=4, N_max=3, w=2, extra_blocks=1)
    K0, V0 = p.K.copy(), p.V.copy()
    idx = np.array([[[[1, 2, 5, 9, 14, 15, -1, -1], [0, 1, 2, 3, 4, 14, 15, -1]]]], dtype=np.int32)
    ln = np.array([[[6, 7]]], dtype=np.int32)
    oracle.compact(p, idx, ln)
    tbl = p.block_table[0]
    changed = np.zeros(p.K.shape[:4], dtype=bool)
    for h in range(2):
        for r in range(ln[0, 0, h]):
            t = idx[0, 0, h, r]
            assert np.array_equal(p.K[0, tbl[r // 4], r % 4, h], K0[0, tbl[t // 4], t % 4, h])
            assert np.array_equal(p.V[0, tbl[r // 4], r % 4, h], V0[0, tbl[t // 4], t % 4, h])
            changed[0, tbl[r // 4], r % 4, h] = True
    assert np.array_equal(p.K[~changed], K0[~changed]) and np.array_equal(p.V[~changed], V0[~changed])
    # rows 0..4 of head 1 were already in place: nothing moved there
    assert np.array_equal(p.K[0, tbl[0], :, 1], K0[0, tbl[0], :, 1])


def test_idempotent_when_nothing_is_evicted():
    p = random_problem(8, B=1, L=1, h_kv=1, G=1, d=4, b=4, N_max=3, w=2)
    K0, V0 = p.K.copy(), p.V.copy()
    idx = np.arange(8, dtype=np.int32).reshape(1, 1, 1, 8)
    oracle.compact(p, idx, np.array([[[8]]], dtype=np.int32))
    assert np.array_equal(p.K, K0) and np.array_equal(p.V, V0)


def test_compaction_into_separate_targets_leaves_sources_alone():
    p = random_problem(9, B=1, L=1, h_kv=1, G=1, d=4, b=2, N_max=3, w=1, extra_blocks=1, N_total=10)
    free = [x for x in range(10) if x not in p.block_table[0].tolist()]
    p.dst_table = np.array([[free[0], p.block_table[0, 1]]], dtype=np.int32)    # block 0 "shared": redirected
    K0 = p.K.copy()
    idx = np.array([[[[1, 3, 6, 7]]]], dtype=np.int32)
    oracle.compact(p, idx, np.array([[[4]]], dtype=np.int32))
    tbl = p.block_table[0]
    assert np.array_equal(p.K[0, tbl[0]], K0[0, tbl[0]])                         # the shared source block is intact
    assert np.array_equal(p.K[0, free[0], 0, 0], K0[0, tbl[0], 1, 0])
    assert np.array_equal(p.K[0, free[0], 1, 0], K0[0, tbl[1], 1, 0])
    assert np.array_equal(p.K[0, tbl[1], 0, 0], K0[0, tbl[3], 0, 0])
    assert np.array_equal(p.K[0, tbl[1], 1, 0], K0[0, tbl[3], 1, 0])


def test_rejects_unsorted_or_out_of_range_indices():
    p = random_problem(10, B=1, L=1, h_kv=1, G=1, d=4, b=4, N_max=3, w=2)
    bad = np.array([[[[3, 2, 5, 6, 7, 8, 9, 10]]]], dtype=np.int32)
    with pytest.raises(ValueError):
        oracle.compact(p, bad, np.array([[[8]]], dtype=np.int32))
    bad = np.array([[[[0, 1, 2, 3, 4, 5, 6, 12]]]], dtype=np.int32)
    with pytest.raises(ValueError):
        oracle.compact(p, bad, np.array([[[8]]], dtype=np.int32))


def test_end_to_end_permutation_invariance_of_logical_result():
    p = random_problem(11, B=1, L=1, h_kv=2, G=2, d=8, b=4, N_max=3, w=2, extra_blocks=2)
    rng = np.random.default_rng(3)
    perm = rng.permutation(p.K.shape[1])
    inv = np.empty_like(perm)
    inv[perm] = np.arange(perm.size)
    p2 = oracle.Problem(K=np.ascontiguousarray(p.K[:, perm]), V=np.ascontiguousarray(p.V[:, perm]), Q=p.Q.copy(),
                        block_table=inv[p.block_table].astype(np.int32), num_blocks=p.num_blocks, q_slot=p.q_slot, N_max=3)
    _, idx1, ln1 = oracle.compress(p)
    _, idx2, ln2 = oracle.compress(p2)
    assert np.array_equal(idx1, idx2) and np.array_equal(ln1, ln2)
    for h in range(2):
        a = p.K[0, p.block_table[0, :2], :, h]
        c = p2.K[0, p2.block_table[0, :2], :, h]
        assert np.array_equal(a, c)
