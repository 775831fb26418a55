"""GPU parity of the score refinements (global score, max pooling, lightning redundancy, moving the global cache)
against the CPU oracle, through the C ABI.

Protocol, on top of P1..P4 of tests/gpu_util.py:
  E1  zp_score_ex vs oracle.score_ex (fully independent): |d| <= 1e-3 (|ref| + lambda R_ref) + 1e-9, and the cache F
      within 1e-3 relative at the positions the oracle wrote, untouched elsewhere
  E2  zp_score_ex vs oracle.refine applied to the DEVICE's attention scores: bit-exact (scores and F) when only the
      global score and pooling are on (they are max / one exact product), 1e-5 of (|S| + lambda R) with redundancy
  E3  the `similarity > p` decision is taken in fp32 on the device and fp64 in the oracle: the cases are built so that
      no within-block cosine similarity lies within 1e-5 of p (checked here in numpy), which makes the decision unique
  E4  fused zp_compress_ex == zp_score_ex -> zp_select_topk -> zp_compact_kv_ex bit for bit (scores, lists, K, V, F)
  E5  oracle.select on the device's refined score bits == device lists; oracle.compact / compact_global applied to
      the device's F after scoring == device pools and F, byte for byte
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_08743_amd import binding, workloads
from tests import gpu_util as G
from tests.util import as_float, random_problem

pytestmark = pytest.mark.gpu


def plant_similar_keys(p, rng, count, noise=0.05):
    """Near-duplicate keys inside blocks, so that some similarities exceed the threshold."""
    L, N_total, b, h_kv, d = p.K.shape
    from tests.util import bf16_bits_to_f32, f32_to_bf16_bits
    for _ in range(count):
        l, blk, h, s1, s2 = rng.integers(L), rng.integers(N_total), rng.integers(h_kv), rng.integers(b), rng.integers(b)
        if s1 == s2:
            continue
        if p.K.dtype == np.uint16:
            src = bf16_bits_to_f32(p.K[l, blk, s1, h])
            p.K[l, blk, s2, h] = f32_to_bf16_bits(src + noise * rng.standard_normal(d).astype(np.float32))
        else:
            p.K[l, blk, s2, h] = p.K[l, blk, s1, h] + noise * rng.standard_normal(d).astype(np.float32)


def threshold_margin(p, thr):
    """Smallest |cos - thr| over all pairs of keys that share a physical block (numpy fp64, every block of the pool)."""
    K = as_float(p.K)                                            # [L, N_total, b, h_kv, d]
    Kt = np.moveaxis(K, 3, 2)                                    # [L, N_total, h_kv, b, d]
    nrm = np.linalg.norm(Kt, axis=-1, keepdims=True)
    unit = np.where(nrm > 0, Kt / np.maximum(nrm, 1e-300), 0.0)
    C = unit @ np.swapaxes(unit, -1, -2)
    return float(np.abs(C - thr).min())


def pick_threshold(p, candidates):
    for thr in candidates:
        if threshold_margin(p, thr) > 1e-5:
            return thr
    raise AssertionError("no threshold with a safe margin among %s" % (candidates,))


def bits(t):
    return t.view(torch.int16) if t.dtype == torch.bfloat16 else t.view(torch.int32)


def run_extras_protocol(p, ex_kw, history=True, seed=0, check_fused=True):
    """ex_kw: alpha, pool_kernel, lam, tau, p, use_F.  Returns a small report."""
    rng = np.random.default_rng(seed)
    pool, batch = G.to_device(p)
    c = G.ctx()
    B = p.block_table.shape[0]
    use_F = ex_kw.pop("use_F", True)
    alpha = float(np.float32(ex_kw.pop("alpha", 0.8)))           # the same fp32 value on both sides
    lam = float(np.float32(ex_kw.get("lam", 0.0)))
    tau = float(np.float32(ex_kw.get("tau", 1.0)))
    thr = float(np.float32(ex_kw.get("p", 1.0)))
    m = ex_kw.get("pool_kernel", 1)
    first_only = ex_kw.get("pool_first_only", False)
    if lam != 0.0:
        assert threshold_margin(p, thr) > 1e-5, "E3: a similarity lies too close to the threshold"
    S_att = oracle.score(p)
    F0 = comp = None
    if use_F:
        F0 = (rng.random(p.K.shape[:4]) * 2.0 * S_att.max()).astype(np.float32)
        comp = (rng.random(B) < 0.6).astype(np.int32) if history else np.zeros(B, dtype=np.int32)
        if history:
            comp[0] = 1
            if B > 1:
                comp[-1] = 0                                      # a mix of first and repeated compressions

    def o_extras(F):
        return oracle.Extras(F=F, compressed=comp, alpha=alpha, pool_kernel=m, lam=lam, tau=tau, p=thr, pool_first_only=first_only)

    def d_extras(F):
        return binding.Extras(F=F, compressed=G.dev_i32(comp), alpha=alpha, pool_kernel=m, lam=lam, tau=tau, p=thr, pool_first_only=first_only)

    def fresh_F():
        return None if F0 is None else torch.from_numpy(F0).cuda()

    # device: attention scores, refined scores
    s0, _, _ = G.alloc_outputs(pool, batch)
    c.zp_score(pool, batch, s0)
    s1, _, _ = G.alloc_outputs(pool, batch)
    F1 = fresh_F()
    c.zp_score_ex(pool, batch, d_extras(F1), s1)
    c.zp_sync_status()
    s0_h, s1_h = s0.cpu().numpy(), s1.cpu().numpy()
    assert np.isfinite(s1_h).all()
    # E1: fully independent
    F_or = None if F0 is None else F0.copy()
    ref = oracle.score_ex(p, o_extras(F_or))
    scale = np.abs(ref)
    if lam != 0.0:
        ex_nor = o_extras(None if F0 is None else F0.copy())
        ex_nor.lam = 0.0
        scale = np.abs(oracle.score_ex(p, ex_nor)) + np.abs(oracle.score_ex(p, ex_nor) - ref)
    err = np.abs(s1_h - ref)
    assert (err <= 1e-3 * scale + 1e-9).all(), "E1: worst %.3g" % (err / (scale + 1e-9)).max()
    if F0 is not None:
        F1_h = F1.cpu().numpy()
        wrote = F_or != F0
        assert np.array_equal(F1_h[~wrote], F0[~wrote]), "E1: the device wrote cache entries the oracle left alone"
        assert (np.abs(F1_h - F_or) <= 1e-3 * np.abs(F_or) + 1e-9).all(), "E1: cache values off"
    # E2: the refinements alone, from the device's attention scores
    F_rf = None if F0 is None else F0.copy()
    ref2 = oracle.refine(p, o_extras(F_rf), s0_h)
    if lam == 0.0:
        assert np.array_equal(s1_h, ref2.astype(np.float32)), "E2: global score / pooling are exact operations"
    else:
        ex_nor = o_extras(None if F0 is None else F0.copy())
        ex_nor.lam = 0.0
        base = oracle.refine(p, ex_nor, s0_h)
        sc2 = np.abs(base) + np.abs(base - ref2)
        assert (np.abs(s1_h - ref2) <= 1e-5 * sc2 + 1e-12).all(), "E2: worst %.3g" % (np.abs(s1_h - ref2) / (sc2 + 1e-12)).max()
    if F0 is not None:
        assert np.array_equal(F1.cpu().numpy(), F_rf), "E2: cache after the global update must be bit-exact"
    rep = dict(worst=float((err / (scale + 1e-9)).max()))
    if not check_fused:
        return rep
    # staged: select on the refined scores, compaction that moves F
    st_pool = G.clone_pool(pool)
    _, s_idx, s_len = G.alloc_outputs(pool, batch)
    c.zp_select_topk(s1, st_pool, batch, s_idx, s_len)
    F_st = None if F1 is None else F1.clone()
    if F_st is not None:
        c.zp_compact_kv_ex(st_pool, batch, F_st, s_idx, s_len)
    else:
        c.zp_compact_kv(st_pool, batch, s_idx, s_len)
    # fused
    fu_pool = G.clone_pool(pool)
    f_s, f_idx, f_len = G.alloc_outputs(pool, batch)
    F_fu = fresh_F()
    c.zp_compress_ex(fu_pool, batch, d_extras(F_fu), f_len, f_s, f_idx)
    c.zp_sync_status()
    # E4
    assert torch.equal(bits(f_s), bits(s1)), "E4: fused refined scores differ from zp_score_ex"
    assert torch.equal(f_idx, s_idx) and torch.equal(f_len, s_len), "E4: kept sets differ"
    assert torch.equal(bits(fu_pool.k), bits(st_pool.k)) and torch.equal(bits(fu_pool.v), bits(st_pool.v)), "E4: pools differ"
    if F_fu is not None:
        assert torch.equal(bits(F_fu), bits(F_st)), "E4: global cache differs"
    # E5
    o_idx, o_len = oracle.select(p, s1_h)
    assert np.array_equal(o_len, f_len.cpu().numpy()) and np.array_equal(o_idx, f_idx.cpu().numpy()), "E5: selection"
    q = oracle.Problem(K=p.K.copy(), V=p.V.copy(), Q=p.Q, block_table=p.block_table, num_blocks=p.num_blocks, q_slot=p.q_slot,
                       N_max=p.N_max, valid_len=p.valid_len, keep=p.keep, dst_table=p.dst_table)
    oracle.compact(q, o_idx, o_len)
    assert np.array_equal(G.pool_bits(fu_pool.k), q.K) and np.array_equal(G.pool_bits(fu_pool.v), q.V), "E5: pools"
    if F_fu is not None:
        F_want = F1.cpu().numpy().copy()
        oracle.compact_global(q, F_want, o_idx, o_len)
        assert np.array_equal(F_fu.cpu().numpy(), F_want), "E5: moved global cache"
    return rep


# ------------------------------------------------------------------ generic kernel (fp32, odd shapes)

@pytest.mark.parametrize("seed,kw,ex", [
    (0, dict(B=2, L=2, h_kv=2, G=2, d=16, b=4, N_max=4, w=3, extra_blocks=1), dict(alpha=0.75)),
    (1, dict(B=2, L=1, h_kv=2, G=1, d=8, b=5, N_max=3, w=2, extra_blocks=2), dict(use_F=False, pool_kernel=5)),
    (2, dict(B=2, L=1, h_kv=1, G=3, d=32, b=8, N_max=5, w=11, num_blocks=[5, 9]), dict(alpha=0.9, pool_kernel=3)),
    (3, dict(B=2, L=2, h_kv=2, G=2, d=16, b=8, N_max=4, w=3, extra_blocks=1), dict(use_F=False, lam=0.3, tau=0.4, p=0.2)),
    (4, dict(B=2, L=1, h_kv=2, G=2, d=12, b=6, N_max=4, w=4, extra_blocks=2), dict(alpha=0.8, pool_kernel=7, lam=0.5, tau=0.05, p=0.35)),
    (5, dict(B=1, L=1, h_kv=2, G=1, d=24, b=8, N_max=4, w=5, bf16=True), dict(alpha=0.5, pool_kernel=3, lam=0.2, tau=0.1, p=0.3)),
    (6, dict(B=1, L=1, h_kv=1, G=2, d=8, b=4, N_max=4, w=2), dict(use_F=False, lam=0.2, tau=0.3, p=-0.5)),     # p < 0: zero entries count
    (7, dict(B=4, L=1, h_kv=2, G=2, d=16, b=4, N_max=4, w=3, extra_blocks=1), dict(alpha=0.75, pool_kernel=3, pool_first_only=True)),
], ids=lambda v: str(v) if isinstance(v, int) else "")
def test_refinements_small_problems(seed, kw, ex):
    p = random_problem(700 + seed, heavy=3, **kw)
    rng = np.random.default_rng(seed)
    plant_similar_keys(p, rng, 12)
    if "p" in ex:
        ex = dict(ex, p=pick_threshold(p, [ex["p"], ex["p"] + 0.013, ex["p"] + 0.029]))
    run_extras_protocol(p, dict(ex), seed=seed)


def test_refinements_with_stale_gaps_fp32():
    b, N_max, w = 8, 5, 11
    p = random_problem(720, B=2, L=1, h_kv=2, G=2, d=16, b=b, N_max=N_max, w=w, extra_blocks=2, heavy=3)
    rng = np.random.default_rng(3)
    N = N_max + 2
    vl = rng.integers(w - b, (N - 1) * b + 1, size=(2, 1, 2)).astype(np.int32)
    vl[0, 0, 0], vl[1, 0, 1] = (N - 1) * b, w - b
    cap = np.minimum((N_max - 1) * b, vl + b)
    p.valid_len = vl
    p.keep = (w + (rng.random(vl.shape) * (cap - w + 1)).astype(np.int32)).clip(w, cap).astype(np.int32)
    plant_similar_keys(p, rng, 20)
    thr = pick_threshold(p, [0.25, 0.26, 0.27])
    run_extras_protocol(p, dict(alpha=0.7, pool_kernel=3, lam=0.4, tau=0.1, p=thr), seed=1)


# ------------------------------------------------------------------ matrix-core kernel (bf16)

@pytest.mark.parametrize("Gq,w,d,b,N_max,extra,gaps", [
    (4, 16, 128, 16, 6, 1, False),      # T = 112: not a multiple of 32
    (4, 16, 128, 16, 7, 2, True),       # stale gaps, prefix lengths off the 32 grid
    (2, 8, 64, 32, 4, 1, True),         # one block per 32-row group
    (8, 16, 128, 8, 9, 0, True),        # four blocks per group
    (1, 40, 64, 16, 9, 2, True),        # window longer than a block
    (4, 16, 128, 64, 3, 1, True),       # block size off the matrix-core menu: vector-ALU redundancy inside the MFMA kernel
    (5, 32, 64, 4, 30, 3, True),
    (4, 32, 128, 16, 8, 1, True),       # four waves: the tile's four blocks go to one wave each
    (2, 8, 64, 16, 5, 1, True),         # a single wave takes all four blocks of a tile
])
@pytest.mark.parametrize("first_only", [False, True], ids=["pool-always", "pool-first"])
def test_refinements_bf16(Gq, w, d, b, N_max, extra, gaps, first_only):
    p = random_problem(800 + Gq * 7 + w + b, B=2, L=2, h_kv=2, G=Gq, d=d, b=b, N_max=N_max, w=w, extra_blocks=extra, bf16=True, heavy=4)
    rng = np.random.default_rng(w + b)
    N = N_max + extra
    budget = (N_max - 1) * b
    if gaps:
        vl = rng.integers(max(0, w - b), (N - 1) * b + 1, size=(2, 2, 2)).astype(np.int32)
        vl[0, 0, 0] = (N - 1) * b
        p.valid_len = vl
        cap = np.minimum(budget, vl + b)
        p.keep = (w + (rng.random(vl.shape) * (cap - w + 1)).astype(np.int32)).clip(w, cap).astype(np.int32)
    else:
        p.keep = rng.integers(w, budget + 1, size=(2, 2, 2)).astype(np.int32)
    plant_similar_keys(p, rng, 40, noise=0.1)
    thr = pick_threshold(p, [0.4, 0.41, 0.42, 0.43])
    rep = run_extras_protocol(p, dict(alpha=0.8, pool_kernel=5, lam=0.3, tau=0.02, p=thr, pool_first_only=first_only), seed=b)
    assert rep["worst"] < 1e-3


@pytest.mark.parametrize("ex", [dict(alpha=0.8), dict(use_F=False, pool_kernel=7), dict(use_F=False, lam=0.3, tau=2e-4, p=0.3),
                                dict(alpha=0.6, pool_kernel=3, lam=0.3, tau=2e-4, p=0.3)], ids=["global", "pool", "redundancy", "all"])
def test_refinements_benchmark_shape(ex):
    w = workloads.config(2, B=2, L=1, N_total=600)
    p, _, _ = G.workload_problem(w)
    rng = np.random.default_rng(5)
    plant_similar_keys(p, rng, 300, noise=0.1)
    if "p" in ex:
        ex = dict(ex, p=pick_threshold(p, [0.4, 0.41, 0.42, 0.43]))
    rep = run_extras_protocol(p, dict(ex), seed=2)
    print("cfg2 reduced, %s: worst relative error %.2e" % (sorted(ex), rep["worst"]))


def test_refinements_off_equal_the_plain_calls():
    p = random_problem(900, B=2, L=1, h_kv=2, G=4, d=128, b=16, N_max=5, w=8, bf16=True)
    pool, batch = G.to_device(p)
    c = G.ctx()
    s0, _, _ = G.alloc_outputs(pool, batch)
    s1, _, _ = G.alloc_outputs(pool, batch)
    c.zp_score(pool, batch, s0)
    c.zp_score_ex(pool, batch, binding.Extras(), s1)
    c.zp_sync_status()
    assert torch.equal(bits(s0), bits(s1))


def test_global_cache_with_shared_prefix_blocks():
    """Two requests share their leading blocks (copy-on-write targets): in the fused call every request's kept
    entries carry its own global scores to its own targets, although the shared source blocks are written by both."""
    b, N_max = 16, 4
    p = random_problem(910, B=2, L=1, h_kv=2, G=4, d=128, b=b, N_max=N_max, w=8, extra_blocks=1, bf16=True, N_total=20)
    p.block_table[1, :2] = p.block_table[0, :2]                     # shared prefix of two blocks
    used = set(p.block_table.reshape(-1).tolist())
    free = [x for x in range(20) if x not in used]
    dst = p.block_table[:, : N_max - 1].copy()
    dst[0, :2], dst[1, :2] = free[0:2], free[2:4]
    p.dst_table = dst
    pool, batch = G.to_device(p)
    c = G.ctx()
    F = torch.full(p.K.shape[:4], -1.0, dtype=torch.float32, device="cuda")
    s, idx, ln = G.alloc_outputs(pool, batch)
    fu = G.clone_pool(pool)
    c.zp_compress_ex(fu, batch, binding.Extras(F=F, alpha=0.8), ln, s, idx)
    c.zp_sync_status()
    s_h, idx_h, ln_h, F_h = s.cpu().numpy(), idx.cpu().numpy(), ln.cpu().numpy(), F.cpu().numpy()
    G.check_scores(s_h, oracle.score(p))                              # first compression: the global score is the attention score
    o_idx, o_len = oracle.select(p, s_h)
    assert np.array_equal(o_idx, idx_h) and np.array_equal(o_len, ln_h)
    for n in range(2):
        for h in range(2):
            k = ln_h[n, 0, h]
            got = F_h[0, dst[n], :, h].reshape(-1)[:k]
            assert np.array_equal(got, s_h[n, 0, h, idx_h[n, 0, h, :k]]), "request %d head %d" % (n, h)
    q = oracle.Problem(K=p.K.copy(), V=p.V.copy(), Q=p.Q, block_table=p.block_table, num_blocks=p.num_blocks, q_slot=p.q_slot,
                       N_max=p.N_max, dst_table=dst)
    oracle.compact(q, o_idx, o_len)
    assert np.array_equal(G.pool_bits(fu.k), q.K) and np.array_equal(G.pool_bits(fu.v), q.V)


def test_extras_argument_errors():
    p = random_problem(920, B=1, L=1, h_kv=1, G=1, d=8, b=4, N_max=3, w=2)
    pool, batch = G.to_device(p)
    c = G.ctx()
    s, _, _ = G.alloc_outputs(pool, batch)
    for bad in (dict(pool_kernel=4), dict(pool_kernel=0), dict(lam=0.1, tau=0.0), dict(lam=0.1, tau=-1.0)):
        with pytest.raises(binding.ZpError) as e:
            c.zp_score_ex(pool, batch, binding.Extras(**bad), s)
        assert e.value.status == binding.ZP_EINVAL


@pytest.mark.parametrize("seed", range(12))
def test_refinements_seeded_random_shapes(seed):
    rng = np.random.default_rng(8000 + seed)
    Gq = int(rng.choice([1, 2, 4, 5, 8]))
    b = int(rng.choice([8, 16, 16, 32]))
    d = int(rng.choice([64, 128]))
    N_max = int(rng.integers(3, 10))
    extra = int(rng.integers(0, 3))
    budget = (N_max - 1) * b
    w = int(rng.integers(1, min(64, budget) + 1))
    B, L, h_kv = 2, int(rng.integers(1, 3)), int(rng.integers(1, 3))
    p = random_problem(8100 + seed, B=B, L=L, h_kv=h_kv, G=Gq, d=d, b=b, N_max=N_max, w=w, extra_blocks=extra, bf16=True, heavy=4)
    N = N_max + extra
    vl = rng.integers(max(0, w - b), (N - 1) * b + 1, size=(B, L, h_kv)).astype(np.int32)
    if seed % 3 == 0:
        vl[...] = (N - 1) * b
    p.valid_len = vl
    cap = np.minimum(budget, vl + b)
    p.keep = (w + (rng.random(vl.shape) * (cap - w + 1)).astype(np.int32)).clip(w, cap).astype(np.int32)
    plant_similar_keys(p, rng, 30, noise=0.1)
    ex = dict(alpha=0.8, use_F=bool(seed % 2 == 0), pool_kernel=int(rng.choice([1, 3, 5])), pool_first_only=bool(seed % 4 == 1))
    if seed % 3 != 1:
        ex.update(lam=0.3, tau=0.02, p=pick_threshold(p, [0.4, 0.41, 0.42, 0.43, 0.44]))
    run_extras_protocol(p, ex, seed=seed)
