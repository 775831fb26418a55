"""Pins for the oracle's score refinements (appendix "Global Score", "Pooling at the Sequence Dimension",
"Lightning Redundancy", "Combining All These Techniques").  The attention score they start from is pinned in
test_oracle_score.py; here each added step is checked against a library routine (torch max_pool1d, scipy softmax),
an independent matrix formulation in numpy, or a closed form."""
import numpy as np
import pytest
import scipy.special
import torch

import oracle
from tests.util import logical_keys, random_problem


def live_positions(N, b, vl):
    return np.array(list(range(vl)) + list(range((N - 1) * b, N * b)))


def F_of(p):
    return np.zeros(p.K.shape[:4], dtype=np.float32)


def test_global_score_first_compression_only_stores():
    p = random_problem(1, B=2, L=2, h_kv=2, G=2, d=8, b=4, N_max=4, w=3, extra_blocks=1)
    S0 = oracle.score(p)
    F = F_of(p)
    F[...] = 7.0                                      # stale garbage: a first compression must not read it
    S1 = oracle.score_ex(p, oracle.Extras(F=F, compressed=np.zeros(2, dtype=np.int32), alpha=0.8))
    assert np.array_equal(S1, S0)
    for n in range(2):
        for l in range(2):
            for h in range(2):
                tbl = p.block_table[n, :5]
                assert np.array_equal(F[l, tbl, :, h].reshape(-1), S0[n, l, h, :20].astype(np.float32))
    touched = np.zeros(F.shape, dtype=bool)
    touched[:, p.block_table[p.block_table >= 0]] = True
    assert (F[~touched] == 7.0).all()


def test_global_score_decayed_max_on_the_live_prefix_only():
    b, N = 4, 5
    p = random_problem(2, B=2, L=1, h_kv=2, G=1, d=8, b=b, N_max=4, w=2, extra_blocks=1)
    p.valid_len = np.array([[[16, 12]], [[16, 8]]], dtype=np.int32)
    p.keep = np.full((2, 1, 2), 4, dtype=np.int32)
    S0 = oracle.score(p)
    rng = np.random.default_rng(0)
    F = (rng.random(p.K.shape[:4]) * S0.max() * 2).astype(np.float32)
    F0 = F.copy()
    comp = np.array([1, 0], dtype=np.int32)           # request 0 has history, request 1 has not
    alpha = 0.6
    S1 = oracle.score_ex(p, oracle.Extras(F=F, compressed=comp, alpha=alpha))
    for n in range(2):
        for h in range(2):
            vl = int(p.valid_len[n, 0, h])
            tbl = p.block_table[n, :N]
            hist = F0[0, tbl, :, h].reshape(-1).astype(np.float64)
            want = S0[n, 0, h, : N * b].copy()
            if comp[n]:
                want[:vl] = np.maximum(alpha * hist[:vl], want[:vl])       # the last block has no history
            live = live_positions(N, b, vl)
            np.testing.assert_allclose(S1[n, 0, h, live], want[live], rtol=1e-15)
            assert np.array_equal(F[0, tbl, :, h].reshape(-1)[live], want[live].astype(np.float32))
            stale = np.setdiff1d(np.arange(N * b), live)
            assert np.array_equal(F[0, tbl, :, h].reshape(-1)[stale], F0[0, tbl, :, h].reshape(-1)[stale])
            assert (S1[n, 0, h, stale] == 0).all()
    assert (S1[0] >= S0[0]).all() and np.array_equal(S1[1], S0[1])


@pytest.mark.parametrize("m", [3, 7])
def test_pooling_is_library_maxpool1d_along_the_live_sequence(m):
    b, N = 4, 6
    p = random_problem(3, B=1, L=1, h_kv=2, G=2, d=8, b=b, N_max=4, w=2, extra_blocks=2)
    p.valid_len = np.array([[[20, 9]]], dtype=np.int32)
    p.keep = np.full((1, 1, 2), 5, dtype=np.int32)
    S0 = oracle.score(p)
    S1 = oracle.score_ex(p, oracle.Extras(pool_kernel=m))
    for h in range(2):
        live = live_positions(N, b, int(p.valid_len[0, 0, h]))
        want = torch.nn.functional.max_pool1d(torch.from_numpy(S0[0, 0, h, live])[None, None], m, stride=1, padding=m // 2)[0, 0].numpy()
        assert np.array_equal(S1[0, 0, h, live], want)
    assert np.array_equal(oracle.score_ex(p, oracle.Extras(pool_kernel=1)), S0)
    with pytest.raises(ValueError):
        oracle.score_ex(p, oracle.Extras(pool_kernel=4))


def test_pooling_at_the_first_compression_only():
    b, N = 4, 5
    p = random_problem(4, B=2, L=1, h_kv=1, G=2, d=8, b=b, N_max=4, w=2, extra_blocks=1)
    S0 = oracle.score(p)
    comp = np.array([1, 0], dtype=np.int32)
    S1 = oracle.score_ex(p, oracle.Extras(compressed=comp, pool_kernel=3, pool_first_only=True))
    want = torch.nn.functional.max_pool1d(torch.from_numpy(S0[1, 0, 0, : N * b])[None, None], 3, stride=1, padding=1)[0, 0].numpy()
    assert np.array_equal(S1[0], S0[0])                          # has history: left alone
    assert np.array_equal(S1[1, 0, 0, : N * b], want) and not np.array_equal(S1[1], S0[1])
    S2 = oracle.score_ex(p, oracle.Extras(compressed=comp, pool_kernel=3))
    assert np.array_equal(S2[1], S1[1]) and not np.array_equal(S2[0], S0[0])   # without the switch every request is pooled


def matrix_redundancy(keys, b, live_mask, p_thr, tau):
    """Independent formulation: full cosine matrix, same-block mask, 'last above p per column' rule, row sums / Tv, softmax."""
    T = keys.shape[0]
    norm = np.linalg.norm(keys, axis=1)
    unit = np.where(norm[:, None] > 0, keys / np.maximum(norm[:, None], 1e-300), 0.0)
    C = unit @ unit.T
    same_block = np.kron(np.eye(T // b), np.ones((b, b))) > 0
    C = np.where(same_block & live_mask[:, None] & live_mask[None, :], C, 0.0)
    np.fill_diagonal(C, 0.0)
    above = C > p_thr
    rows = np.arange(T)[:, None]
    last = np.where(above, rows, -1).max(axis=0)                      # per column: highest row above the threshold
    cols = np.flatnonzero(last >= 0)
    C[last[cols], cols] = 0.0
    Tv = int(live_mask.sum())
    r = C.sum(axis=1)[live_mask] / Tv
    return scipy.special.softmax(r / tau)


@pytest.mark.parametrize("seed,thr", [(0, 0.2), (1, 0.05), (2, 0.6)])
def test_lightning_redundancy_matches_matrix_formulation(seed, thr):
    b, N = 8, 5
    p = random_problem(10 + seed, B=1, L=1, h_kv=2, G=2, d=6, b=b, N_max=3, w=3, extra_blocks=2)
    rng = np.random.default_rng(seed)
    tbl = p.block_table[0]
    for _ in range(6):                                                # near-duplicate neighbours inside blocks
        blk, s1, s2 = tbl[rng.integers(N)], rng.integers(b), rng.integers(b)
        p.K[0, blk, s2] = p.K[0, blk, s1] + 0.05 * rng.standard_normal(p.K.shape[3:]).astype(np.float32)
    p.valid_len = np.array([[[32, 21]]], dtype=np.int32)
    p.keep = np.full((1, 1, 2), 6, dtype=np.int32)
    S0 = oracle.score(p)
    lam, tau = 0.3, 0.4
    S1 = oracle.score_ex(p, oracle.Extras(lam=lam, tau=tau, p=thr))
    for h in range(2):
        vl = int(p.valid_len[0, 0, h])
        live = live_positions(N, b, vl)
        mask = np.zeros(N * b, dtype=bool)
        mask[live] = True
        R = matrix_redundancy(logical_keys(p, 0, 0, h), b, mask, thr, tau)
        assert R.sum() == pytest.approx(1.0)
        np.testing.assert_allclose(S1[0, 0, h, live], S0[0, 0, h, live] - lam * R, rtol=1e-12, atol=1e-15)
        stale = np.setdiff1d(np.arange(N * b), live)
        assert (S1[0, 0, h, stale] == 0).all()


def test_redundancy_closed_forms():
    b, N, d = 4, 3, 8
    p = random_problem(20, B=1, L=1, h_kv=1, G=1, d=d, b=b, N_max=3, w=2)
    S0 = oracle.score(p)[0, 0, 0]
    T = N * b
    tbl = p.block_table[0]
    # (a) mutually orthogonal keys inside every block: no similarity, R is uniform
    for t in range(T):
        row = np.zeros(d, dtype=np.float32)
        row[t % b] = 1.0 + t
        p.K[0, tbl[t // b], t % b, 0] = row
    Sa0 = oracle.score(p)[0, 0, 0]
    Sa = oracle.score_ex(p, oracle.Extras(lam=0.5, tau=0.3, p=0.9))[0, 0, 0]
    np.testing.assert_allclose(Sa, Sa0 - 0.5 / T, rtol=1e-12)
    # (b) identical keys inside every block, p below 1: every column loses its newest similar entry, so the row sums
    #     of a block are [b-1, ..., b-1, b-2, 0] (the newest token collects nothing, the one before it loses one)
    for t in range(T):
        p.K[0, tbl[t // b], t % b, 0] = np.full(d, 1.0 + t // b, dtype=np.float32)
    Sb0 = oracle.score(p)[0, 0, 0]
    tau = 0.25
    Sb = oracle.score_ex(p, oracle.Extras(lam=1.0, tau=tau, p=0.5))[0, 0, 0]
    r = np.tile(np.array([b - 1] * (b - 2) + [b - 2, 0], dtype=np.float64), N) / T
    np.testing.assert_allclose(Sb, Sb0 - scipy.special.softmax(r / tau), rtol=1e-12)
    # with the threshold above every similarity nothing is zeroed: all rows equal, R uniform again
    Sc = oracle.score_ex(p, oracle.Extras(lam=1.0, tau=tau, p=1.5))[0, 0, 0]
    np.testing.assert_allclose(Sc, Sb0 - 1.0 / T, rtol=1e-12)


def test_order_of_the_refinements():
    # global update first (what the cache stores), then pooling, then redundancy
    p = random_problem(30, B=1, L=1, h_kv=1, G=2, d=8, b=4, N_max=4, w=2)
    F = F_of(p)
    F[...] = 1.0                                                     # history larger than any score
    ex = oracle.Extras(F=F, compressed=np.ones(1, dtype=np.int32), alpha=0.5, pool_kernel=3, lam=0.2, tau=0.5, p=0.3)
    S = oracle.score_ex(p, ex)[0, 0, 0]
    S_att = oracle.score(p)[0, 0, 0]
    g = S_att.copy()
    g[:12] = np.maximum(0.5, g[:12])                                  # global
    assert np.array_equal(F[0, p.block_table[0], :, 0].reshape(-1), g.astype(np.float32))   # cache = after global, before pooling
    pooled = torch.nn.functional.max_pool1d(torch.from_numpy(g)[None, None], 3, stride=1, padding=1)[0, 0].numpy()
    R = matrix_redundancy(logical_keys(p, 0, 0, 0), 4, np.ones(16, dtype=bool), 0.3, 0.5)
    np.testing.assert_allclose(S, pooled - 0.2 * R, rtol=1e-12)


def test_global_cache_moves_with_the_kept_entries():
    p = random_problem(40, B=2, L=2, h_kv=2, G=1, d=4, b=4, N_max=3, w=2, extra_blocks=1)
    rng = np.random.default_rng(1)
    F = rng.random(p.K.shape[:4]).astype(np.float32)
    F0 = F.copy()
    p.keep = rng.integers(2, 9, size=(2, 2, 2)).astype(np.int32)
    S = oracle.score(p)
    idx, ln = oracle.select(p, S.astype(np.float32))
    oracle.compact_global(p, F, idx, ln)
    want = F0.copy()
    for n in range(2):
        tbl = p.block_table[n]
        for l in range(2):
            for h in range(2):
                for r in range(ln[n, l, h]):
                    t = idx[n, l, h, r]
                    want[l, tbl[r // 4], r % 4, h] = F0[l, tbl[t // 4], t % 4, h]
    assert np.array_equal(F, want) and not np.array_equal(F, F0)


def test_redundancy_threshold_at_the_margin_moves_scores_by_a_bounded_amount():
    """The device takes the `similarity > p` decision in fp32, the oracle in fp64; the GPU cases keep every similarity
    away from p so that the decision is unique.  What a decision AT the margin can change is bounded.  A similarity value
    sits at (i, j) and (j, i); when p crosses it, in each of the two columns the entry that is zeroed moves to another
    entry (or to none), so at most two entries (values <= 1) change in each column: a row sum / Tv moves by at most
    2 / Tv, the softmax normaliser by a factor within exp(+-2 / (Tv tau)), every entry of R by a factor within
    exp(+-4 / (Tv tau)), and S - lambda R by at most lambda R (e^{4/(Tv tau)} - 1).  Checked here on the oracle by
    putting p just below and just above similarities at which a decision does flip.  At the benchmark's size and the
    recommended settings (Tv = 4112, tau = 0.4) the factor is 1.0024, i.e. a score moves by less than 2.5e-3 lambda R,
    well inside the 1e-3 (|S| + lambda R) of the GPU comparison whenever lambda R < 0.4 |S|."""
    b, N = 8, 5
    p = random_problem(77, B=1, L=1, h_kv=1, G=2, d=6, b=b, N_max=3, w=3, extra_blocks=2)
    rng = np.random.default_rng(5)
    tbl = p.block_table[0]
    for _ in range(6):
        blk, s1, s2 = tbl[rng.integers(N)], rng.integers(b), rng.integers(b)
        p.K[0, blk, s2] = p.K[0, blk, s1] + 0.05 * rng.standard_normal(p.K.shape[3:]).astype(np.float32)
    keys = logical_keys(p, 0, 0, 0)
    unit = keys / np.linalg.norm(keys, axis=1, keepdims=True)
    C = unit @ unit.T
    same_block = np.kron(np.eye(N), np.ones((b, b))) > 0
    np.fill_diagonal(C, -2.0)
    cand = np.sort(np.unique(C[same_block & (C > 0.3)]))
    gaps = np.diff(cand)
    lam, tau, Tv, eps = 0.3, 0.4, N * b, 1e-9
    base = oracle.score(p)[0, 0, 0]
    flips = 0
    for c_star in cand[1:][gaps > 1e-6]:                               # similarities with clear air below them
        lo = oracle.score_ex(p, oracle.Extras(lam=lam, tau=tau, p=float(c_star - eps)))[0, 0, 0]
        hi = oracle.score_ex(p, oracle.Extras(lam=lam, tau=tau, p=float(c_star + eps)))[0, 0, 0]
        if np.array_equal(lo, hi):                                     # not the last entry above p of its column: nothing flips
            continue
        flips += 1
        check_margin_pair(base, lo, hi, lam, tau, Tv, c_star)
    assert flips >= 3, "too few thresholds at which a decision flips"
    # the same bound at the benchmark's size and recommended settings
    assert np.exp(4.0 / (4112 * 0.4)) - 1.0 < 2.5e-3


def check_margin_pair(base, lo, hi, lam, tau, Tv, c_star):
    R_lo, R_hi = (base - lo) / lam, (base - hi) / lam
    factor = np.exp(4.0 / (Tv * tau))
    assert np.all(R_hi <= R_lo * factor * (1 + 1e-12)) and np.all(R_lo <= R_hi * factor * (1 + 1e-12))
    assert np.abs(hi - lo).max() <= lam * max(R_lo.max(), R_hi.max()) * (factor - 1.0) * (1 + 1e-9)
