"""Pins for the oracle's scoring step (appendix "Paged Attention Score").

None of these re-types the oracle's loop nest: each compares against a library
formulation of textbook attention, a closed form, an invariant or a pure-Python
brute force on a tiny case, chosen so that a wrong mask direction, a transposed
operand, a swapped reduction order or a wrong head grouping fails.
"""
import math

import numpy as np
import pytest

import oracle
from tests.util import logical_keys, random_problem, window_queries, f32_to_bf16_bits


def textbook_causal_rows(q, k, first_query_pos):
    """softmax(q k^T / sqrt d + causal mask) for queries at positions first_query_pos + u (numpy, matrix form)."""
    T, d = k.shape
    logits = q @ k.T / math.sqrt(d)
    pos = np.arange(T)[None, :]
    qpos = first_query_pos + np.arange(q.shape[0])[:, None]
    logits = np.where(pos > qpos, -np.inf, logits)
    logits -= logits.max(axis=1, keepdims=True)
    e = np.exp(logits)
    return e / e.sum(axis=1, keepdims=True)


@pytest.mark.parametrize("bf16", [False, True])
def test_g1_is_column_mean_of_textbook_causal_attention(bf16):
    # no grouping: S is the mean over the window rows of an ordinary causal attention matrix
    p = random_problem(1, B=2, L=2, h_kv=3, G=1, d=16, b=4, N_max=4, w=3, extra_blocks=1, bf16=bf16)
    S = oracle.score(p)
    for n in range(2):
        for l in range(2):
            for h in range(3):
                k = logical_keys(p, n, l, h)
                T = k.shape[0]
                P = textbook_causal_rows(window_queries(p, n, l, h), k, T - 3)
                np.testing.assert_allclose(S[n, l, h, :T], P.mean(axis=0), rtol=1e-12, atol=1e-15)


def test_w1_is_max_over_group_of_single_softmax_rows():
    p = random_problem(2, h_kv=2, G=3, d=8, b=4, N_max=3, w=1)
    S = oracle.score(p)
    for h in range(2):
        k = logical_keys(p, 0, 0, h)
        rows = [textbook_causal_rows(window_queries(p, 0, 0, h * 3 + g), k, k.shape[0] - 1)[0] for g in range(3)]
        np.testing.assert_allclose(S[0, 0, h, : k.shape[0]], np.max(rows, axis=0), rtol=1e-12)


def test_gqa_grouping_and_reduction_order_bruteforce():
    # pure-Python loops, max over the group BEFORE the mean over the window; heads grouped contiguously
    p = random_problem(3, h_kv=2, G=2, d=4, b=2, N_max=3, w=2)
    S = oracle.score(p)
    T, w, G, d = 6, 2, 2, 4
    for h in range(2):
        k = logical_keys(p, 0, 0, h)
        probs = {}
        for g in range(G):
            q = window_queries(p, 0, 0, h * G + g)
            for u in range(w):
                vis = [t for t in range(T) if t <= T - w + u]
                e = {t: math.exp(sum(q[u][c] * k[t][c] for c in range(d)) / math.sqrt(d)) for t in vis}
                z = sum(e.values())
                for t in range(T):
                    probs[g, u, t] = e[t] / z if t in e else 0.0
        for t in range(T):
            want = sum(max(probs[g, u, t] for g in range(G)) for u in range(w)) / w
            assert S[0, 0, h, t] == pytest.approx(want, rel=1e-12)
        # the other order (mean over window, then max over group) differs on this input: the pin is discriminating
        other = [max(sum(probs[g, u, t] for u in range(w)) / w for g in range(G)) for t in range(T)]
        assert not np.allclose(other, S[0, 0, h, :T])


def test_identical_keys_closed_form_pins_mask_direction_and_offsets():
    # all keys equal => each query attends uniformly to what it can see:
    # S[t] = (1/w) * sum over window rows u that see t of 1 / (T - w + u + 1)
    b, N, w, d = 4, 3, 3, 8
    p = random_problem(4, h_kv=1, G=2, d=d, b=b, N_max=N, w=w)
    p.K[...] = 0.37
    S = oracle.score(p)[0, 0, 0]
    T = N * b
    for t in range(T):
        want = sum(1.0 / (T - w + u + 1) for u in range(w) if t <= T - w + u) / w
        assert S[t] == pytest.approx(want, rel=1e-12)
    # the newest token is seen by the last window row only, the oldest window token by all
    assert S[T - 1] == pytest.approx(1.0 / (w * T))


def test_one_hot_keys_closed_form():
    # keys are c * e_{t mod d}; query = s * e_0: logit = c s / sqrt(d) on positions with t mod d == 0, else 0
    b, N, w, d = 4, 4, 1, 4
    p = random_problem(5, h_kv=1, G=1, d=d, b=b, N_max=N, w=w)
    T = N * b
    tbl = p.block_table[0]
    for t in range(T):
        row = np.zeros(d, dtype=np.float32)
        row[t % d] = 2.0
        p.K[0, tbl[t // b], t % b, 0] = row
    p.Q[...] = 0
    p.Q[0, p.q_slot[0], 0, 0, 0] = 3.0
    S = oracle.score(p)[0, 0, 0]
    hot = math.exp(2.0 * 3.0 / math.sqrt(d))
    z = (T // d) * hot + (T - T // d)
    for t in range(T):
        assert S[t] == pytest.approx((hot if t % d == 0 else 1.0) / z, rel=1e-12)


def test_invariants_sum_range_and_window_mass():
    G, w = 4, 5
    p = random_problem(6, B=2, L=2, h_kv=2, G=G, d=16, b=8, N_max=4, w=w, extra_blocks=2, heavy=3)
    S = oracle.score(p)
    T = 6 * 8
    assert (S >= 0).all()
    tot = S[..., :T].sum(axis=-1)
    assert (tot >= 1 - 1e-12).all() and (tot <= G + 1e-12).all()   # each of the w*G rows sums to 1
    assert (S[..., T:] == 0).all() if S.shape[-1] > T else True
    # position T-1 only receives mass from the last window row: at most 1/w
    assert (S[..., T - 1] <= 1.0 / w + 1e-15).all()


def test_rows_sum_to_one_when_group_is_one():
    p = random_problem(7, h_kv=2, G=1, d=8, b=4, N_max=5, w=4)
    S = oracle.score(p)
    np.testing.assert_allclose(S.sum(axis=-1), 1.0, rtol=1e-12)


def test_block_table_permutation_invariance():
    # same logical content under another physical placement => identical scores
    p = random_problem(8, B=1, L=2, h_kv=2, G=2, d=8, b=4, N_max=4, w=2, extra_blocks=1)
    S0 = oracle.score(p)
    rng = np.random.default_rng(99)
    perm = rng.permutation(p.K.shape[1])
    inv = np.empty_like(perm)
    inv[perm] = np.arange(perm.size)
    p2 = oracle.Problem(K=np.ascontiguousarray(p.K[:, perm]), V=np.ascontiguousarray(p.V[:, perm]), Q=p.Q,
                        block_table=np.where(p.block_table >= 0, inv[np.maximum(p.block_table, 0)], -1).astype(np.int32),
                        num_blocks=p.num_blocks, q_slot=p.q_slot, N_max=p.N_max)
    assert np.array_equal(oracle.score(p2), S0)


def test_heavy_keys_rank_high():
    # a key aligned with every window query and scaled up must collect far more than the average mass
    p = random_problem(9, h_kv=1, G=1, d=32, b=8, N_max=5, w=4)
    qbar = p.Q[0, p.q_slot[0], :, 0, :].mean(axis=0)
    p.K[0, p.block_table[0, 1], 3, 0] = 3.0 * qbar
    S = oracle.score(p)[0, 0, 0]
    assert np.argmax(S[: 40 - 4]) == 1 * 8 + 3
    assert S[11] > 5 * np.median(S[:36])


def test_stale_gap_equals_packed_sequence():
    # a head whose live data is [0, vl) ++ last block scores exactly like a request that holds only those blocks
    b, w = 4, 6   # window longer than a block: it reaches back into the live prefix
    p = random_problem(10, B=1, L=1, h_kv=2, G=2, d=8, b=b, N_max=3, w=w, extra_blocks=2)   # N = 5
    vl = np.array([[[8, 12]]], dtype=np.int32)      # heads differ; both multiples of b
    keep = np.array([[[6, 7]]], dtype=np.int32)
    p.valid_len, p.keep = vl, keep
    S = oracle.score(p)
    for h in range(2):
        nlive = vl[0, 0, h] // b
        blocks = list(p.block_table[0, :nlive]) + [p.block_table[0, 4]]
        tbl = np.array([blocks], dtype=np.int32)
        packed = oracle.Problem(K=p.K, V=p.V, Q=p.Q, block_table=tbl, num_blocks=np.array([len(blocks)], dtype=np.int32),
                                q_slot=p.q_slot, N_max=3)
        Sp = oracle.score(packed)[0, 0, h]
        live = list(range(vl[0, 0, h])) + list(range(16, 20))
        np.testing.assert_allclose(S[0, 0, h, live], Sp[: len(live)], rtol=1e-13)
        stale = [t for t in range(20) if t not in live]
        assert (S[0, 0, h, stale] == 0).all()


def test_bf16_inputs_are_widened_exactly():
    p = random_problem(11, h_kv=1, G=2, d=8, b=4, N_max=3, w=2, bf16=True)
    from tests.util import bf16_bits_to_f32
    pf = oracle.Problem(K=bf16_bits_to_f32(p.K), V=bf16_bits_to_f32(p.V), Q=bf16_bits_to_f32(p.Q), block_table=p.block_table,
                        num_blocks=p.num_blocks, q_slot=p.q_slot, N_max=p.N_max)
    assert np.array_equal(oracle.score(p), oracle.score(pf))
    assert f32_to_bf16_bits(np.array([1.0, -2.5, 3.140625], dtype=np.float32)).tolist() == [0x3F80, 0xC020, 0x4049]


def test_rejects_inconsistent_batches():
    p = random_problem(12, N_max=3)
    p.num_blocks = np.array([2], dtype=np.int32)           # fewer than N_max blocks
    with pytest.raises(ValueError):
        oracle.score(p)
    p = random_problem(12, N_max=3)
    p.keep = np.array([[[1]]], dtype=np.int32)             # keep < w
    with pytest.raises(ValueError):
        oracle.score(p)
    p = random_problem(12, N_max=3)
    p.block_table = p.block_table.copy()
    p.block_table[0, 0] = p.K.shape[1]                     # block id out of range
    with pytest.raises(ValueError):
        oracle.score(p)
