"""GPU test plumbing: put a workload / problem on the device, run the library, compare with the oracle.

Parity protocol used throughout:
  P1  device scores vs fp64 oracle scores, |d| <= 1e-3 |ref| + 1e-9
  P2  oracle selection applied to the DEVICE's fp32 score bits == device keep_idx / len, exactly
  P3  oracle compaction of that kept set == device pools, byte for byte (whole pool)
  P4  fused zp_compress == staged zp_score -> zp_select_topk -> zp_compact_kv, bit for bit
  P5  fully independent run (oracle scores -> oracle set): sets equal, or every swap is a near tie
"""
from __future__ import annotations

import numpy as np
import torch

import oracle
from paper_2603_08743_amd import binding
from paper_2603_08743_amd.workloads import Workload, to_host_bits

_ctx = None


def ctx() -> binding.Context:
    global _ctx
    if _ctx is None:
        _ctx = binding.Context()
    return _ctx


def dev_i32(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def to_device(p: oracle.Problem):
    """oracle.Problem (host) -> (Pool, Batch) on the device, same bits."""
    def up(a):
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
        return torch.from_numpy(a).cuda()
    pool = binding.Pool(k=up(p.K), v=up(p.V), q=up(p.Q))
    batch = binding.Batch(block_table=dev_i32(p.block_table), num_blocks=dev_i32(p.num_blocks), q_slot=dev_i32(p.q_slot),
                          N_max=p.N_max, L=p.K.shape[0], dst_table=dev_i32(p.dst_table), valid_len=dev_i32(p.valid_len),
                          keep=dev_i32(p.keep))
    return pool, batch


def workload_problem(w: Workload, layer0: int = 0, L_slab=None, device="cuda"):
    """Materialise a workload slab on the device and mirror it on the host for the oracle."""
    Ls = w.L - layer0 if L_slab is None else L_slab
    K, V, Q = w.pools(device, layer0, Ls)
    sl = slice(layer0, layer0 + Ls)
    keep = None if w.keep is None else np.ascontiguousarray(w.keep[:, sl])
    vl = None if w.valid_len is None else np.ascontiguousarray(w.valid_len[:, sl])
    p = oracle.Problem(K=to_host_bits(K), V=to_host_bits(V), Q=to_host_bits(Q), block_table=w.block_table.copy(),
                       num_blocks=w.num_blocks.copy(), q_slot=w.q_slot.copy(), N_max=w.N_max, valid_len=vl, keep=keep)
    pool = binding.Pool(k=K, v=V, q=Q, layer0=0)
    batch = binding.Batch(block_table=dev_i32(w.block_table), num_blocks=dev_i32(w.num_blocks), q_slot=dev_i32(w.q_slot),
                          N_max=w.N_max, L=Ls, valid_len=dev_i32(vl), keep=dev_i32(keep))
    return p, pool, batch


def clone_pool(pool: binding.Pool) -> binding.Pool:
    return binding.Pool(k=pool.k.clone(), v=pool.v.clone(), q=pool.q, layer0=pool.layer0)


def alloc_outputs(pool: binding.Pool, batch: binding.Batch):
    Ls, _, b, h_kv, _ = pool.k.shape
    B, max_blocks = batch.block_table.shape
    scores = torch.full((B, Ls, h_kv, max_blocks * b), float("nan"), dtype=torch.float32, device="cuda")
    keep_idx = torch.full((B, Ls, h_kv, (batch.N_max - 1) * b), -7, dtype=torch.int32, device="cuda")
    ln = torch.full((B, Ls, h_kv), -7, dtype=torch.int32, device="cuda")
    return scores, keep_idx, ln


def run_staged(pool, batch):
    c = ctx()
    scores, keep_idx, ln = alloc_outputs(pool, batch)
    c.zp_score(pool, batch, scores)
    c.zp_select_topk(scores, pool, batch, keep_idx, ln)
    c.zp_compact_kv(pool, batch, keep_idx, ln)
    c.zp_sync_status()
    return scores, keep_idx, ln


def run_fused(pool, batch, debug=True):
    c = ctx()
    scores, keep_idx, ln = alloc_outputs(pool, batch)
    c.zp_compress(pool, batch, ln, scores if debug else None, keep_idx if debug else None)
    c.zp_sync_status()
    return scores, keep_idx, ln


def pool_bits(t: torch.Tensor) -> np.ndarray:
    return to_host_bits(t)


def check_scores(gpu_scores: np.ndarray, ref: np.ndarray, rtol=1e-3, atol=1e-9):
    assert np.isfinite(gpu_scores).all(), "P1: device scores hold NaN/inf (unwritten or broken entries)"
    err = np.abs(gpu_scores.astype(np.float64) - ref)
    bad = err > rtol * np.abs(ref) + atol
    assert not bad.any(), "P1: %d scores off; worst rel %.3g" % (bad.sum(), (err / (np.abs(ref) + 1e-300))[bad].max())
    return float((err / (np.abs(ref) + atol)).max())


def full_protocol(p: oracle.Problem, pool: binding.Pool, batch: binding.Batch, exact_p5: bool = False):
    """Runs staged and fused on copies of the pool and checks P1..P5.  Returns a small report dict."""
    staged_pool, fused_pool = clone_pool(pool), clone_pool(pool)
    s_scores, s_idx, s_len = run_staged(staged_pool, batch)
    f_scores, f_idx, f_len = run_fused(fused_pool, batch)
    s_scores_h, s_idx_h, s_len_h = s_scores.cpu().numpy(), s_idx.cpu().numpy(), s_len.cpu().numpy()
    # P4
    assert torch.equal(s_scores.view(torch.int32), f_scores.view(torch.int32)), "P4: fused scores differ from staged"
    assert torch.equal(s_idx, f_idx) and torch.equal(s_len, f_len), "P4: fused kept set differs from staged"
    assert torch.equal(staged_pool.k.view(torch.int16) if staged_pool.k.dtype == torch.bfloat16 else staged_pool.k,
                       fused_pool.k.view(torch.int16) if fused_pool.k.dtype == torch.bfloat16 else fused_pool.k), "P4: K differs"
    assert torch.equal(staged_pool.v.view(torch.int16) if staged_pool.v.dtype == torch.bfloat16 else staged_pool.v,
                       fused_pool.v.view(torch.int16) if fused_pool.v.dtype == torch.bfloat16 else fused_pool.v), "P4: V differs"
    # P1
    ref = oracle.score(p)
    worst = check_scores(s_scores_h, ref)
    # P2
    o_idx, o_len = oracle.select(p, s_scores_h)
    assert np.array_equal(o_len, s_len_h), "P2: lengths differ"
    assert np.array_equal(o_idx, s_idx_h), "P2: kept sets differ on identical score bits"
    # P3
    q = oracle.Problem(K=p.K.copy(), V=p.V.copy(), Q=p.Q, block_table=p.block_table, num_blocks=p.num_blocks, q_slot=p.q_slot,
                       N_max=p.N_max, valid_len=p.valid_len, keep=p.keep, dst_table=p.dst_table)
    oracle.compact(q, o_idx, o_len)
    assert np.array_equal(pool_bits(fused_pool.k), q.K), "P3: K pool bytes differ"
    assert np.array_equal(pool_bits(fused_pool.v), q.V), "P3: V pool bytes differ"
    # P5
    i_idx, i_len = oracle.select(p, ref.astype(np.float32))
    assert np.array_equal(i_len, s_len_h)
    mism_units = 0
    flat_g, flat_o = s_idx_h.reshape(-1, s_idx_h.shape[-1]), i_idx.reshape(-1, i_idx.shape[-1])
    flat_ref = ref.reshape(-1, ref.shape[-1])
    for un in range(flat_g.shape[0]):
        if np.array_equal(flat_g[un], flat_o[un]):
            continue
        mism_units += 1
        assert not exact_p5, "P5: independent kept set differs in unit %d" % un
        a = set(flat_g[un][flat_g[un] >= 0].tolist())
        o = set(flat_o[un][flat_o[un] >= 0].tolist())
        only_g, only_o = sorted(a - o), sorted(o - a)
        assert len(only_g) == len(only_o)
        sg, so = flat_ref[un][only_g], flat_ref[un][only_o]
        # every swapped pair must be a near tie in the reference scores
        assert np.all(np.abs(np.sort(sg) - np.sort(so)) <= 2e-3 * np.maximum(np.sort(sg), np.sort(so)) + 1e-9), "P5: swap is not a near tie"
    return dict(worst_rel=worst, p5_mismatch_units=mism_units, units=flat_g.shape[0])
