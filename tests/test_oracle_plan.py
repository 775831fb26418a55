"""Pins for the oracle's block bookkeeping (Method, "Compressed PagedAttention" and
"Shared Prefix Cache for Compressed PagedAttention") and for the check-only decode attention."""
import math
import os

import numpy as np
import pytest

import oracle
from tests.util import as_float, random_problem

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "fig1_compressed_pagedattention.txt")


def read_golden():
    out = {}
    for line in open(GOLDEN):
        if line.strip() and not line.startswith("#"):
            k, v = line.split()
            out[k] = int(v)
    return out


def test_first_figure_structure():
    g = read_golden()
    N_max, b, w = g["N_max"], g["b"], g["w"]
    # two requests that overflowed during prefill: 6 and 5 blocks
    p = random_problem(0, B=g["requests"], L=1, h_kv=1, G=1, d=4, b=b, N_max=N_max, w=w, num_blocks=[6, 5])
    refcnt = np.zeros(p.K.shape[1], dtype=np.int32)
    for n in range(2):
        refcnt[p.block_table[n, : p.num_blocks[n]]] += 1
    r = oracle.plan(p.block_table, p.num_blocks, N_max, refcnt, [])
    for n, N in enumerate([6, 5]):
        tbl = p.block_table[n]
        assert r["new_table"][n].tolist() == tbl[:N_max].tolist()          # first three + the fourth, reserved
        assert len(r["new_table"][n]) == g["blocks_held_after"]
        assert r["dst_table"][n].tolist() == tbl[: g["blocks_holding_kept_entries"]].tolist()
        assert r["new_table"][n][g["reserved_block_index"]] == tbl[N_max - 1]
    assert r["freed"].tolist() == p.block_table[0, 4:6].tolist() + p.block_table[1, 4:5].tolist()   # the rest, in order
    assert r["n_free_used"] == 0
    # kept entries really end up in the first three blocks and the budget is (N_max-1)*b
    _, idx, ln = oracle.compress(p)
    assert (ln == (N_max - 1) * b).all() and idx.shape[-1] == 12
    assert (idx[0, 0, 0, -w:] == [22, 23]).all() and (idx[1, 0, 0, -w:] == [18, 19]).all()   # window kept last


def test_exactly_nmax_blocks_releases_nothing():
    r = oracle.plan(np.array([[5, 2, 7, 1]], dtype=np.int32), [4], 4, np.array([0, 1, 1, 0, 0, 1, 0, 1], dtype=np.int32), [0, 3])
    assert r["freed"].size == 0 and r["new_table"].tolist() == [[5, 2, 7, 1]] and r["n_free_used"] == 0
    assert r["refcnt"].tolist() == [0, 1, 1, 0, 0, 1, 0, 1]


def test_shared_prefix_shorter_than_budget():
    # blocks 10, 11 are a prefix shared by requests A (compressing) and a bystander: refcount 2
    refcnt = np.zeros(20, dtype=np.int32)
    A = [10, 11, 3, 4, 5, 6]
    refcnt[A] += 1
    refcnt[[10, 11, 15]] += 1                              # bystander holds 10, 11, 15
    r = oracle.plan(np.array([A], dtype=np.int32), [6], 4, refcnt, [17, 18, 19])
    # N_prefix = 2 < N_max-1 = 3: two fresh blocks + one reused; shared blocks are not written
    assert r["dst_table"].tolist() == [[17, 18, 3]]
    assert r["new_table"].tolist() == [[17, 18, 3, 4]]
    assert r["n_free_used"] == 2                           # = min(N_prefix, N_max-1)
    assert r["freed"].tolist() == [5, 6]
    assert r["refcnt"][[10, 11]].tolist() == [1, 1]        # no longer shared, still held by the bystander
    assert r["refcnt"][[17, 18, 3, 4, 5, 6, 19]].tolist() == [1, 1, 1, 1, 0, 0, 0]


def test_shared_prefix_covering_all_targets():
    refcnt = np.zeros(16, dtype=np.int32)
    A = [1, 2, 3, 4, 5, 6]                                 # first five shared, the last private
    refcnt[A] += 1
    refcnt[[1, 2, 3, 4, 5]] += 2
    r = oracle.plan(np.array([A], dtype=np.int32), [6], 4, refcnt, [9, 10, 11, 12])
    assert r["dst_table"].tolist() == [[9, 10, 11]]        # N_prefix >= N_max-1: N_max-1 new blocks
    assert r["new_table"].tolist() == [[9, 10, 11, 6]]     # reserved = first private block at index >= N_max-1
    assert r["freed"].size == 0 and r["n_free_used"] == 3
    assert r["refcnt"][[1, 2, 3, 4, 5]].tolist() == [2] * 5


def test_two_sharers_in_one_batch_release_the_prefix_together():
    refcnt = np.zeros(16, dtype=np.int32)
    A, Bq = [1, 2, 3, 4], [1, 5, 6, 7]                     # block 1 shared by exactly these two
    refcnt[A] += 1
    refcnt[Bq] += 1
    r = oracle.plan(np.array([A, Bq], dtype=np.int32), [4, 4], 4, refcnt, [9, 10, 11])
    assert r["dst_table"].tolist() == [[9, 2, 3], [10, 5, 6]]   # both judged on the counts at batch start
    assert r["freed"].tolist() == [1]                          # released by the second decrement
    assert r["refcnt"][1] == 0 and r["n_free_used"] == 2


def test_free_list_exhaustion_changes_nothing():
    refcnt = np.zeros(8, dtype=np.int32)
    A = [1, 2, 3, 4]
    refcnt[A] += 1
    refcnt[[1, 2]] += 1
    before = refcnt.copy()
    with pytest.raises(MemoryError):
        oracle.plan(np.array([A], dtype=np.int32), [4], 4, refcnt, [7])
    assert np.array_equal(refcnt, before)


@pytest.mark.parametrize("seed", range(5))
def test_conservation_laws(seed):
    rng = np.random.default_rng(seed)
    N_max, N_total, B = 5, 200, 6
    perm = rng.permutation(N_total)
    prefix = perm[:3]
    pos, rows, nbs = 3, [], []
    refcnt = np.zeros(N_total, dtype=np.int32)
    for n in range(B):
        N = int(rng.integers(N_max, N_max + 4))
        share = int(rng.integers(0, 4)) if n % 2 == 0 else 0
        row = list(prefix[:share]) + list(perm[pos:pos + N - share])
        pos += N - share
        refcnt[row] += 1
        rows.append(row + [-1] * (9 - N))
        nbs.append(N)
    refcnt[prefix] += 1                                    # a bystander keeps the prefix shared
    free = perm[pos:]
    r = oracle.plan(np.array(rows, dtype=np.int32), nbs, N_max, refcnt, free)
    held_before = sum(nbs)
    n_shared = sum(1 for n in range(B) for i in range(nbs[n]) if refcnt[rows[n][i]] > 1)
    fresh = sum(1 for n in range(B) for i in range(N_max - 1) if refcnt[rows[n][i]] > 1)
    assert r["n_free_used"] == fresh
    assert (r["new_table"] >= 0).all() and r["new_table"].shape == (B, N_max)       # every request holds N_max blocks
    assert len(r["freed"]) == held_before - n_shared + fresh - B * N_max            # unshared case: N - N_max per request
    assert r["refcnt"].sum() == refcnt.sum() - n_shared + fresh - len(r["freed"])
    # no block appears twice among new tables, freed blocks and the unused free list
    live = r["new_table"].reshape(-1).tolist() + r["freed"].tolist() + free[r["n_free_used"]:].tolist()
    assert len(live) == len(set(live))
    assert (r["refcnt"][r["freed"]] == 0).all() and (r["refcnt"][r["new_table"]] == 1).all()


def test_decode_attention_is_textbook_softmax_attention():
    p = random_problem(3, B=2, L=2, h_kv=2, G=2, d=8, b=4, N_max=3, w=2, bf16=True)
    rng = np.random.default_rng(0)
    from tests.util import f32_to_bf16_bits
    q = f32_to_bf16_bits(rng.standard_normal((2, 2, 4, 8)).astype(np.float32))
    ln = rng.integers(1, 9, size=(2, 2, 2)).astype(np.int32)
    out = oracle.decode_attention(p.K, p.V, q, p.block_table, ln, 4)
    for n in range(2):
        for l in range(2):
            for hq in range(4):
                h = hq // 2
                k = as_float(p.K[l, p.block_table[n], :, h]).reshape(-1, 8)[: ln[n, l, h]]
                v = as_float(p.V[l, p.block_table[n], :, h]).reshape(-1, 8)[: ln[n, l, h]]
                a = k @ as_float(q[n, l, hq]) / math.sqrt(8)
                e = np.exp(a - a.max())
                np.testing.assert_allclose(out[n, l, hq], (e / e.sum()) @ v, rtol=1e-12, atol=1e-14)
