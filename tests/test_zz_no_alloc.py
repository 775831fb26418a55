"""zp_compress_static (the entry point for callers that cannot allocate) against zp_compress, through the C ABI.

Two calls in a row, the second on a smaller input: the device array the call keeps its status words in is shared by
every call on the GPU and keeps the previous call's contents, so the second call must not be disturbed by the first.
Bar: bit-exact lengths and K/V pool bytes (integer and byte work).
"""
import numpy as np
import pytest
import torch

from paper_2603_08743_amd import binding, workloads
from tests import gpu_util as G

pytestmark = pytest.mark.gpu


def bits(t):
    return t.view(torch.int16) if t.dtype == torch.bfloat16 else t.view(torch.int32)


def both_ways(w):
    """Run the same batch through zp_compress (context) and zp_compress_static on copies of the pool."""
    _, pool, batch = G.workload_problem(w)
    a, b = G.clone_pool(pool), G.clone_pool(pool)
    units = w.B * w.L * w.h_kv
    ln_ctx = torch.full((units,), -7, dtype=torch.int32, device="cuda")
    ln_static = torch.full((units,), -7, dtype=torch.int32, device="cuda")
    G.ctx().zp_compress(a, batch, ln_ctx)
    G.ctx().zp_sync_status()
    binding.zp_compress_static(b, batch, ln_static)
    torch.cuda.synchronize()
    assert torch.equal(ln_ctx, ln_static), "lengths differ"
    assert (ln_ctx >= w.w).all()
    assert torch.equal(bits(a.k), bits(b.k)) and torch.equal(bits(a.v), bits(b.v)), "compacted pools differ"
    assert not torch.equal(bits(a.k), bits(pool.k)), "nothing was compacted"
    return batch, pool


def test_static_entry_point_matches_zp_compress_on_two_calls_in_a_row():
    big = workloads.config(2, B=3, L=2, N_total=900)                 # 48 units of the 8B-like shape, per-head keep counts
    small = workloads.config(1, B=1, L=1, N_total=200)               # then 4 units of the 7B-like shape
    both_ways(big)
    both_ways(small)


def test_static_entry_point_after_a_call_that_skipped_a_unit():
    """A call whose batch holds a bad keep count raises the flag in the shared status words; the next call starts clean."""
    w = workloads.config(2, B=2, L=1, N_total=600)
    _, pool, batch = G.workload_problem(w)
    keep = batch.keep.clone()
    keep.view(-1)[3] = 1                                             # below the window: the kernel skips this unit
    bad = binding.Batch(block_table=batch.block_table, num_blocks=batch.num_blocks, q_slot=batch.q_slot, N_max=batch.N_max, L=batch.L, keep=keep)
    units = w.B * w.L * w.h_kv
    ln = torch.full((units,), -7, dtype=torch.int32, device="cuda")
    binding.zp_compress_static(G.clone_pool(pool), bad, ln)
    torch.cuda.synchronize()
    got = ln.cpu().numpy()
    assert got[3] == -1 and (np.delete(got, 3) >= w.w).all()
    both_ways(workloads.config(2, B=1, L=1, N_total=300))


def test_static_entry_point_refuses_bad_arguments_without_launching():
    w = workloads.config(1, B=1, L=1, N_total=200)
    _, pool, batch = G.workload_problem(w)
    with pytest.raises(AssertionError):
        binding.zp_compress_static(pool, batch, torch.zeros(1, dtype=torch.int32, device="cuda"))   # wrong length: caught by the binding
    lib = binding.load_library()
    import ctypes
    p, b = pool.c(), batch.c()
    rc = lib.zp_compress_static(ctypes.byref(p), ctypes.byref(b), ctypes.c_void_p(None), ctypes.c_void_p(None))
    assert rc == binding.ZP_EINVAL and b"len_out" in lib.zp_last_error(None)


def test_static_entry_point_inside_a_hip_graph():
    """The callers this entry point is for include code under HIP graph capture: captured after one eager call (which
    resolves the status array's address), every replay, with eager work and synchronisations in between, must give the
    eager call's lengths and pool bytes."""
    w = workloads.config(2, B=2, L=1, N_total=600)
    _, pool, batch = G.workload_problem(w)
    units = w.B * w.L * w.h_kv
    K0, V0 = pool.k.clone(), pool.v.clone()
    ln_e = torch.full((units,), -7, dtype=torch.int32, device="cuda")
    binding.zp_compress_static(pool, batch, ln_e)                    # eager
    torch.cuda.synchronize()
    Ke, Ve = pool.k.clone(), pool.v.clone()
    assert (ln_e >= w.w).all() and not torch.equal(bits(Ke), bits(K0))
    ln_g = torch.full((units,), -7, dtype=torch.int32, device="cuda")
    pool.k.copy_(K0)
    pool.v.copy_(V0)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        binding.zp_compress_static(pool, batch, ln_g)
    for rep in range(3):
        pool.k.copy_(K0)
        pool.v.copy_(V0)
        ln_g.fill_(-7)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(ln_g, ln_e), "replay %d" % rep
        assert torch.equal(bits(pool.k), bits(Ke)) and torch.equal(bits(pool.v), bits(Ve)), "replay %d" % rep
