"""GPU parity of the HIP path against the CPU oracle, through the C ABI (protocol P1..P5 in tests/gpu_util.py)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_08743_amd import binding, workloads
from tests import gpu_util as G
from tests.util import random_problem

pytestmark = pytest.mark.gpu


SPLIT_OFF = ("the split path (several workgroups per unit) is switched off in the library: its bounded wait expired "
             "intermittently on MI355X (reported cleanly, nothing faulted) and the cause is not established")


@pytest.fixture(autouse=True, params=[pytest.param(1, marks=pytest.mark.skip(reason=SPLIT_OFF)), 0], ids=["split", "single"])
def split_mode(request):
    """Every case is written to run on both bf16 kernels: several workgroups per unit and one per unit."""
    G.ctx().zp_set_option(binding.ZP_OPT_SPLIT, request.param)
    yield request.param
    G.ctx().zp_set_option(binding.ZP_OPT_SPLIT, -1)


def test_split_option_is_refused():
    with pytest.raises(binding.ZpError) as e:
        G.ctx().zp_set_option(binding.ZP_OPT_SPLIT, 1)
    assert e.value.status == binding.ZP_EUNSUPPORTED


def test_config0_tiny_fp32_exact():
    w = workloads.config(0)
    p, pool, batch = G.workload_problem(w)
    rep = G.full_protocol(p, pool, batch, exact_p5=True)
    assert rep["units"] == 2 and rep["worst_rel"] < 1e-4
    # the two heavy key positions are kept in both heads
    _, idx, ln = oracle.compress(p)
    heavy_t = [t for t in range(16) if w.heavy[w.block_table[0, t // 4], t % 4]]
    assert len(heavy_t) == 2 and all(t in idx[0, 0, h] for t in heavy_t for h in range(2))


@pytest.mark.parametrize("cfg,kw", [
    (1, dict(B=2, L=2, N_total=300)),      # G=7, w=32, budget 2048
    (2, dict(B=2, L=1, N_total=600)),      # G=4, w=64, budget 4096, per-head keep counts
    (4, dict(B=1, L=1, N_total=600)),      # G=5, w=128, budget 8192
    (5, dict(B=2, L=2, N_total=30)),       # the paper's own geometry: block size 256, window 16, budget 2048
], ids=["cfg1", "cfg2", "cfg4", "paper-geometry"])
def test_benchmark_shapes_reduced_batch(cfg, kw):
    w = workloads.config(cfg, **kw)
    p, pool, batch = G.workload_problem(w)
    rep = G.full_protocol(p, pool, batch)
    print("cfg%d: %s" % (cfg, rep))
    assert rep["worst_rel"] < 1e-3
    assert rep["p5_mismatch_units"] <= max(1, rep["units"] // 4)


@pytest.mark.parametrize("seed,kw", [
    (0, dict(B=2, L=2, h_kv=2, G=2, d=16, b=4, N_max=4, w=3, extra_blocks=1)),
    (1, dict(B=1, L=1, h_kv=3, G=1, d=8, b=5, N_max=3, w=2, extra_blocks=2)),            # b not a power of two
    (2, dict(B=3, L=1, h_kv=1, G=3, d=32, b=8, N_max=5, w=11, num_blocks=[5, 9, 6])),    # w > b, overflowed prefill
    (3, dict(B=1, L=2, h_kv=2, G=2, d=64, b=16, N_max=6, w=4, bf16=True)),               # bf16 but d/G off the MFMA menu? (G=2: runtime-G MFMA)
    (4, dict(B=2, L=1, h_kv=2, G=1, d=24, b=8, N_max=4, w=5, bf16=True)),                # bf16, d=24: generic path
    (5, dict(B=1, L=1, h_kv=1, G=6, d=256, b=4, N_max=9, w=7)),                          # 1 KiB rows
], ids=lambda v: str(v) if isinstance(v, int) else "")
def test_small_random_problems(seed, kw):
    p = random_problem(100 + seed, heavy=3, **kw)
    pool, batch = G.to_device(p)
    rep = G.full_protocol(p, pool, batch, exact_p5=not kw.get("bf16", False))
    assert rep["worst_rel"] < 1e-3


@pytest.mark.parametrize("Gq,w,d,b,N_max,extra", [
    (1, 1, 128, 16, 5, 0), (1, 40, 64, 16, 9, 2), (2, 16, 128, 16, 6, 1), (3, 5, 128, 8, 12, 0), (4, 16, 128, 256, 2, 1),
    (5, 32, 64, 16, 20, 3), (6, 9, 128, 24, 7, 0), (7, 32, 128, 16, 17, 0), (8, 16, 64, 32, 5, 1), (16, 3, 128, 16, 4, 0),
    (4, 200, 128, 16, 30, 0), (8, 128, 64, 16, 12, 0),
    (4, 64, 128, 128, 3, 1), (8, 32, 64, 64, 4, 0),      # eight-wave workgroups with blocks larger than / equal to a key tile
])
def test_mfma_path_shape_sweep(Gq, w, d, b, N_max, extra):
    p = random_problem(200 + Gq * 7 + w, B=2, L=1, h_kv=2, G=Gq, d=d, b=b, N_max=N_max, w=w, extra_blocks=extra, bf16=True, heavy=4)
    rng = np.random.default_rng(w)
    budget = (N_max - 1) * b
    p.keep = rng.integers(w, budget + 1, size=(2, 1, 2)).astype(np.int32)
    pool, batch = G.to_device(p)
    rep = G.full_protocol(p, pool, batch)
    assert rep["worst_rel"] < 1e-3


@pytest.mark.parametrize("bf16", [False, True])
def test_stale_gaps_and_per_head_keep(bf16):
    # re-compression: heads with different live prefixes; window longer than a block reaches into the prefix
    b, N_max, w = 16, 6, 40
    p = random_problem(300, B=2, L=2, h_kv=2, G=4, d=128 if bf16 else 32, b=b, N_max=N_max, w=w, extra_blocks=1, bf16=bf16, heavy=5)
    rng = np.random.default_rng(1)
    N = N_max + 1
    vl = rng.integers(w - b, (N - 1) * b + 1, size=(2, 2, 2)).astype(np.int32)
    vl[0, 0, 0], vl[1, 1, 1] = (N - 1) * b, w - b                    # extremes: no gap / shortest legal sequence
    cap = np.minimum((N_max - 1) * b, vl + b)
    keep = (w + (rng.random(vl.shape) * (cap - w + 1)).astype(np.int32)).clip(w, cap).astype(np.int32)
    p.valid_len, p.keep = vl, keep
    pool, batch = G.to_device(p)
    rep = G.full_protocol(p, pool, batch)
    assert rep["worst_rel"] < 1e-3


def test_run_to_run_determinism():
    w = workloads.config(2, B=2, L=1, N_total=600)
    _, pool, batch = G.workload_problem(w)
    outs = []
    for _ in range(3):
        pl = G.clone_pool(pool)
        s, i, l = G.run_fused(pl, batch)
        outs.append((s.clone(), i.clone(), pl.k.clone(), pl.v.clone()))
    for o in outs[1:]:
        assert all(torch.equal(a.view(torch.int16) if a.dtype == torch.bfloat16 else a,
                               c.view(torch.int16) if c.dtype == torch.bfloat16 else c) for a, c in zip(outs[0], o))


def test_duplicate_keys_tie_break_end_to_end():
    # identical key rows give bitwise-equal scores on the device too; the lower position must win
    p = random_problem(400, B=1, L=1, h_kv=1, G=4, d=128, b=16, N_max=5, w=8, bf16=True)
    tbl = p.block_table[0]
    row = p.K[0, tbl[1], 3, 0].copy()
    for t in (5, 21, 22, 40, 41, 57):
        p.K[0, tbl[t // 16], t % 16, 0] = row
    pool, batch = G.to_device(p)
    s, idx, ln = G.run_fused(G.clone_pool(pool), batch)
    sh = s.cpu().numpy()[0, 0, 0]
    assert len({sh[t].tobytes() for t in (5, 19, 21, 22, 40, 41, 57)}) == 1
    o_idx, _ = oracle.select(p, s.cpu().numpy())
    assert np.array_equal(o_idx, idx.cpu().numpy())


def test_logit_spike_late_in_the_sequence():
    # one late key is a large multiple of a window query: its logit exceeds everything before it by hundreds of
    # binary orders of magnitude, which forces the running softmax reference of sweep 1 to be re-based mid-sequence
    from tests.util import bf16_bits_to_f32, f32_to_bf16_bits
    p = random_problem(500, B=1, L=1, h_kv=2, G=4, d=128, b=16, N_max=40, w=16, bf16=True)
    tbl = p.block_table[0]
    for h, t in ((0, 300), (1, 37)):
        q = bf16_bits_to_f32(p.Q[0, p.q_slot[0], 5, h * 4 + 1])
        p.K[0, tbl[t // 16], t % 16, h] = f32_to_bf16_bits(30.0 * q)
    pool, batch = G.to_device(p)
    rep = G.full_protocol(p, pool, batch)
    assert rep["worst_rel"] < 1e-3


def test_workgroup_to_unit_map_does_not_change_results():
    # 21 units: not a multiple of the 8 XCDs, so the ragged branch of the map is exercised; both maps must give the same bits
    p = random_problem(600, B=3, L=1, h_kv=7, G=4, d=128, b=16, N_max=6, w=16, extra_blocks=1, bf16=True, heavy=4)
    rng = np.random.default_rng(0)
    p.keep = rng.integers(16, 81, size=(3, 1, 7)).astype(np.int32)
    pool, batch = G.to_device(p)
    outs = []
    for mode in (0, 1):
        G.ctx().zp_set_option(binding.ZP_OPT_XCD_MAP, mode)
        pl = G.clone_pool(pool)
        s, i, l = G.run_fused(pl, batch)
        outs.append((s, i, l, pl.k, pl.v))
    G.ctx().zp_set_option(binding.ZP_OPT_XCD_MAP, 1)
    for a, c in zip(*outs):
        assert torch.equal(a.view(torch.int16) if a.dtype == torch.bfloat16 else a, c.view(torch.int16) if c.dtype == torch.bfloat16 else c)
    rep = G.full_protocol(p, pool, batch)
    assert rep["worst_rel"] < 1e-3


@pytest.mark.parametrize("seed", range(24))
def test_seeded_random_shapes(seed):
    """Shapes, live prefixes and keep counts drawn from a seed: whatever geometry the library picks must pass the protocol."""
    rng = np.random.default_rng(7000 + seed)
    Gq = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 16]))
    b = int(rng.choice([4, 8, 16, 32]))
    d = int(rng.choice([64, 128]))
    N_max = int(rng.integers(3, 13))
    extra = int(rng.integers(0, 4))
    budget = (N_max - 1) * b
    w = int(rng.integers(1, min(96, budget) + 1))
    B, L, h_kv = int(rng.integers(1, 4)), int(rng.integers(1, 3)), int(rng.integers(1, 4))
    p = random_problem(7100 + seed, B=B, L=L, h_kv=h_kv, G=Gq, d=d, b=b, N_max=N_max, w=w, extra_blocks=extra, bf16=True, heavy=4)
    N = N_max + extra
    if seed % 2:
        vl = rng.integers(max(0, w - b), (N - 1) * b + 1, size=(B, L, h_kv)).astype(np.int32)
        p.valid_len = vl
    else:
        vl = np.full((B, L, h_kv), (N - 1) * b, dtype=np.int32)
    cap = np.minimum(budget, vl + b)
    p.keep = (w + (rng.random(vl.shape) * (cap - w + 1)).astype(np.int32)).clip(w, cap).astype(np.int32)
    pool, batch = G.to_device(p)
    rep = G.full_protocol(p, pool, batch)
    assert rep["worst_rel"] < 1e-3


@pytest.mark.parametrize("w,N_max", [(64, 20), (128, 36)])
def test_keys_whose_logits_jump_far_above_everything_before_them(w, N_max):
    """Massive activations: sweep 1 keeps each row's sum of exp2 against a reference that only moves when the sum leaves
    the safe range, which late keys with logits more than 2^100 above everything before them force; the softmax then is
    nearly one-hot.  A few keys in later blocks are scaled by 128 (exact in bf16): logits of the order of +-200 in base 2."""
    p = random_problem(910 + w, B=1, L=1, h_kv=2, G=4 if w == 64 else 5, d=128, b=16, N_max=N_max, w=w, extra_blocks=1, bf16=True, heavy=2)
    tbl = p.block_table[0]
    for blk, slot in ((5, 3), (N_max // 2, 9), (N_max - 3, 0), (N_max - 3, 15)):
        p.K[0, tbl[blk], slot] += np.uint16(7 << 7)                  # exponent + 7: times 128
    pool, batch = G.to_device(p)
    rep = G.full_protocol(p, pool, batch)
    assert rep["worst_rel"] < 1e-3
