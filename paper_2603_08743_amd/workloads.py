"""Seeded synthetic inputs for the compression step (shapes of reasoning-decode workloads).

This module holds *no* arithmetic of the method: it only produces paged K/V
pools, a window-query cache, block tables, per-head keep counts and reference
counts.  It serves the HIP path (device tensors) and the CPU oracle (the same
bits on the host), and imports neither.

Values come from a counter-based integer hash of (seed, tensor id, flat element
index), so any sub-range of a tensor can be regenerated bit-for-bit on either
device: twelve 10-bit uniforms are summed (Irwin-Hall) into
``z = (s - 6138) / 1024`` (exact in fp32, mean 0, unit variance), multiplied by
3 at "heavy" key positions, then rounded to the storage type.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional, Tuple

import numpy as np
import torch

_M64 = (1 << 64) - 1


def _s64(x: int) -> int:
    """Python int -> the int64 with the same low 64 bits."""
    x &= _M64
    return x - (1 << 64) if x >= (1 << 63) else x


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix64(x: torch.Tensor) -> torch.Tensor:
    """splitmix64 finaliser on int64 tensors (wrap-around arithmetic)."""
    z = x + _s64(0x9E3779B97F4A7C15)
    z = (z ^ _lsr(z, 30)) * _s64(0xBF58476D1CE4E5B9)
    z = (z ^ _lsr(z, 27)) * _s64(0x94D049BB133111EB)
    return z ^ _lsr(z, 31)


def _sum6x10(h: torch.Tensor) -> torch.Tensor:
    """Sum of the six 10-bit fields in bits 0..59 of h."""
    m = 0x3FF | (0x3FF << 20) | (0x3FF << 40)
    a = (h & m) + ((h >> 10) & m)
    return (a & 0xFFFFF) + ((a >> 20) & 0xFFFFF) + ((a >> 40) & 0xFFFFF)


def hashed_normal(seed: int, tensor_id: int, start: int, count: int, device) -> torch.Tensor:
    """fp32 values z(i), i in [start, start+count): approximately N(0,1), multiples of 1/1024."""
    idx = torch.arange(start, start + count, dtype=torch.int64, device=device)
    key = _mix64(idx ^ _s64((seed * 0x100000001B3 + tensor_id) * 0x9E3779B97F4A7C15))
    s = _sum6x10(key) + _sum6x10(_mix64(key ^ _s64(0xD6E8FEB86659FD93)))
    return (s - 6138).to(torch.float32) * (1.0 / 1024.0)


def hashed_uniform16(seed: int, tensor_id: int, count: int) -> np.ndarray:
    """count 16-bit uniforms (host, numpy int64), same hash family."""
    idx = torch.arange(0, count, dtype=torch.int64)
    key = _mix64(idx ^ _s64((seed * 0x100000001B3 + tensor_id) * 0x9E3779B97F4A7C15))
    return (key & 0xFFFF).numpy()


_TID_K, _TID_V, _TID_Q, _TID_HEAVY, _TID_KEEP, _TID_QDEC = 1, 2, 3, 4, 5, 6
_CHUNK = 1 << 25  # elements generated per step (bounds temporaries to a few GiB on the device)


@dataclass
class Workload:
    """One compression batch plus the pool it lives in (all host metadata; tensors made on demand)."""

    name: str
    L: int
    h_kv: int
    h_q: int
    d: int
    dtype: str              # "f32" or "bf16"
    b: int
    N_max: int
    w: int
    N_total: int
    M: int                  # query slots
    block_table: np.ndarray  # [B, max_blocks] int32, -1 padded
    num_blocks: np.ndarray   # [B] int32
    q_slot: np.ndarray       # [B] int32
    heavy: np.ndarray        # [N_total, b] bool: key rows scaled x3
    refcnt: np.ndarray       # [N_total] int32 (all tables of the pool, bystanders included)
    free_list: np.ndarray    # [n_free] int32
    seed: int
    keep: Optional[np.ndarray] = None       # [B, L, h_kv] int32
    valid_len: Optional[np.ndarray] = None  # [B, L, h_kv] int32
    bystander_tables: list = field(default_factory=list)  # block id arrays of requests not in the batch

    @property
    def B(self) -> int:
        return int(self.block_table.shape[0])

    @property
    def max_blocks(self) -> int:
        return int(self.block_table.shape[1])

    @property
    def budget(self) -> int:
        return (self.N_max - 1) * self.b

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    @property
    def esize(self) -> int:
        return 4 if self.dtype == "f32" else 2

    def _fill(self, tid: int, shape: Tuple[int, ...], layer0: int, per_layer: int, device, heavy=None) -> torch.Tensor:
        out = torch.empty(shape, dtype=self.torch_dtype, device=device)
        flat = out.view(-1)
        total = flat.numel()
        hv = None
        if heavy is not None:  # [N_total, b] -> scale per (block, slot), broadcast over heads and dims
            hv = torch.from_numpy(heavy.reshape(-1)).to(device)
        row = self.h_kv * self.d
        for o in range(0, total, _CHUNK):
            c = min(_CHUNK, total - o)
            z = hashed_normal(self.seed, tid, layer0 * per_layer + o, c, device)
            if hv is not None:
                rows = (torch.arange(o, o + c, dtype=torch.int64, device=device) // row) % hv.numel()
                z = torch.where(hv[rows], z * 3.0, z)
            flat[o:o + c] = z.to(self.torch_dtype)
        return out

    def pools(self, device, layer0: int = 0, L_slab: Optional[int] = None):
        """K, V ``[L_slab, N_total, b, h_kv, d]`` and Q ``[L_slab, M, w, h_q, d]`` for global layers [layer0, layer0+L_slab)."""
        Ls = self.L - layer0 if L_slab is None else L_slab
        kv_shape = (Ls, self.N_total, self.b, self.h_kv, self.d)
        per_layer_kv = self.N_total * self.b * self.h_kv * self.d
        per_layer_q = self.M * self.w * self.h_q * self.d
        K = self._fill(_TID_K, kv_shape, layer0, per_layer_kv, device, heavy=self.heavy)
        V = self._fill(_TID_V, kv_shape, layer0, per_layer_kv, device)
        Q = self._fill(_TID_Q, (Ls, self.M, self.w, self.h_q, self.d), layer0, per_layer_q, device)
        return K, V, Q

    def decode_queries(self, device, layer0: int = 0, L_slab: Optional[int] = None) -> torch.Tensor:
        """One seeded query per (request, layer, query head) for the check-only decode attention: [B, L_slab, h_q, d]."""
        Ls = self.L - layer0 if L_slab is None else L_slab
        full = self._fill(_TID_QDEC, (self.B, self.L, self.h_q, self.d), 0, 0, device)
        return full[:, layer0:layer0 + Ls].contiguous()

    def subset(self, requests) -> "Workload":
        """The same pool with only the given batch rows (other requests become bystanders)."""
        requests = np.asarray(requests, dtype=np.int64)
        rest = [self.block_table[n, : self.num_blocks[n]].copy() for n in range(self.B) if n not in set(requests.tolist())]
        return Workload(
            name=self.name + "[sub]", L=self.L, h_kv=self.h_kv, h_q=self.h_q, d=self.d, dtype=self.dtype, b=self.b,
            N_max=self.N_max, w=self.w, N_total=self.N_total, M=self.M, block_table=self.block_table[requests].copy(),
            num_blocks=self.num_blocks[requests].copy(), q_slot=self.q_slot[requests].copy(), heavy=self.heavy,
            refcnt=self.refcnt, free_list=self.free_list, seed=self.seed,
            keep=None if self.keep is None else self.keep[requests].copy(),
            valid_len=None if self.valid_len is None else self.valid_len[requests].copy(),
            bystander_tables=self.bystander_tables + rest)


def to_host_bits(t: torch.Tensor) -> np.ndarray:
    """Device/host tensor -> contiguous numpy array the oracle accepts (bf16 as uint16 bit patterns)."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def make_workload(name: str, *, L: int, h_kv: int, h_q: int, d: int, dtype: str, b: int, N_max: int, w: int, B: int,
                  N_total: int, seed: int, num_blocks=None, keep_range: Optional[Tuple[int, int]] = None,
                  heavy_frac: float = 0.05, heavy_exact: Optional[int] = None, M: Optional[int] = None,
                  shared_prefix_blocks: int = 0, shared_frac: float = 0.0, n_bystanders: int = 0,
                  bystander_blocks: Optional[Tuple[int, int]] = None) -> Workload:
    """Build a batch: shuffled block tables dealt from a seeded permutation of the pool.

    num_blocks: per-request block counts (default: every request at exactly N_max).
    keep_range: per (request, layer, head) keep counts uniform in [lo, hi] (default: the budget for all).
    shared_prefix_blocks / shared_frac: the first ``shared_frac`` of the requests (batch and bystanders alike,
      interleaved by a seeded draw) share their leading ``shared_prefix_blocks`` physical blocks.
    n_bystanders: further requests that hold blocks of the pool but are not compressing.
    """
    rng = np.random.default_rng(seed)
    nb = np.full(B, N_max, dtype=np.int32) if num_blocks is None else np.asarray(num_blocks, dtype=np.int32)
    assert nb.shape == (B,) and (nb >= N_max).all()
    by_nb = np.zeros(0, dtype=np.int32)
    if n_bystanders:
        lo, hi = bystander_blocks if bystander_blocks else (1, N_max - 1)
        by_nb = rng.integers(lo, hi + 1, size=n_bystanders).astype(np.int32)
    perm = rng.permutation(N_total).astype(np.int32)
    pos = 0
    prefix = None
    n_all = B + n_bystanders
    is_sharer = np.zeros(n_all, dtype=bool)
    if shared_prefix_blocks and shared_frac > 0:
        prefix = perm[:shared_prefix_blocks].copy()
        pos = shared_prefix_blocks
        is_sharer[rng.permutation(n_all)[: int(round(shared_frac * n_all))]] = True
    max_blocks = int(nb.max())
    table = np.full((B, max_blocks), -1, dtype=np.int32)
    refcnt = np.zeros(N_total, dtype=np.int32)
    bystanders = []
    for r in range(n_all):
        N = int(nb[r]) if r < B else int(by_nb[r - B])
        row = np.empty(N, dtype=np.int32)
        k0 = 0
        if is_sharer[r] and prefix is not None:
            k0 = min(N - 1 if r < B else N, shared_prefix_blocks)  # a compressing request's last block is private
            row[:k0] = prefix[:k0]
        need = N - k0
        if pos + need > N_total:
            raise ValueError("pool of %d blocks too small for workload %s" % (N_total, name))
        row[k0:] = perm[pos:pos + need]
        pos += need
        np.add.at(refcnt, row, 1)
        if r < B:
            table[r, :N] = row
        else:
            bystanders.append(row)
    free_list = perm[pos:].copy()
    M = B if M is None else M
    q_slot = rng.permutation(M)[:B].astype(np.int32)
    if heavy_exact is not None:  # exactly this many heavy logical positions in request 0
        heavy = np.zeros((N_total, b), dtype=bool)
        tpos = rng.choice(int(nb[0]) * b - w, size=heavy_exact, replace=False)
        heavy[table[0, tpos // b], tpos % b] = True
    else:
        u = hashed_uniform16(seed, _TID_HEAVY, N_total * b).reshape(N_total, b)
        heavy = u < int(heavy_frac * 65536)
    keep = None
    if keep_range is not None:
        lo, hi = keep_range
        u = hashed_uniform16(seed, _TID_KEEP, B * L * h_kv).reshape(B, L, h_kv)
        keep = (lo + (u * (hi - lo + 1) >> 16)).astype(np.int32)
    return Workload(name=name, L=L, h_kv=h_kv, h_q=h_q, d=d, dtype=dtype, b=b, N_max=N_max, w=w, N_total=N_total, M=M,
                    block_table=table, num_blocks=nb, q_slot=q_slot, heavy=heavy, refcnt=refcnt, free_list=free_list,
                    seed=seed, keep=keep, bystander_tables=bystanders)


_BASE_SEED = 20260308


def config(i: int, *, B: Optional[int] = None, L: Optional[int] = None, N_total: Optional[int] = None,
           compress_frac: float = 1.0) -> Workload:
    """The five benchmark configurations (B, L, N_total may be reduced for parity tests; shapes per unit stay real), and as
    number 5 the geometry of the paper's own runs (experimental setup: block size 256, window 16)."""
    seed = _BASE_SEED + i
    if i == 0:   # tiny fp32 case: 16 cached tokens, budget 12
        return make_workload("cfg0-tiny-f32", L=1, h_kv=2, h_q=4, d=64, dtype="f32", b=4, N_max=4, w=2, B=1,
                             N_total=16, seed=seed, heavy_exact=2)
    if i == 1:   # 7B-like decode shape, budget 2048
        Bv = 64 if B is None else B
        return make_workload("cfg1-7b-budget2048", L=28 if L is None else L, h_kv=4, h_q=28, d=128, dtype="bf16", b=16,
                             N_max=129, w=32, B=Bv, N_total=(16384 if N_total is None else N_total), seed=seed)
    if i == 2:   # 8B-like decode shape, budget 4096, per-head keep counts
        Bv = 256 if B is None else B
        return make_workload("cfg2-8b-budget4096", L=32 if L is None else L, h_kv=8, h_q=32, d=128, dtype="bf16", b=16,
                             N_max=257, w=64, B=Bv, N_total=(131072 if N_total is None else N_total), seed=seed,
                             keep_range=(1024, 4096))
    if i == 3:   # prefix-cache mix: 75 % of the requests share a 1024-token prefix; a fraction compresses this step
        n_req = 512 if B is None else B
        n_comp = max(1, int(round(compress_frac * n_req)))
        return make_workload("cfg3-prefix-mix", L=32 if L is None else L, h_kv=8, h_q=32, d=128, dtype="bf16", b=16,
                             N_max=257, w=64, B=n_comp, N_total=(132096 if N_total is None else N_total), seed=seed,
                             shared_prefix_blocks=64, shared_frac=0.75, n_bystanders=n_req - n_comp,
                             bystander_blocks=(65, 256), M=n_req)
    if i == 4:   # 14B-like long-reasoning shape, budget 8192
        Bv = 128 if B is None else B
        return make_workload("cfg4-14b-budget8192", L=48 if L is None else L, h_kv=8, h_q=40, d=128, dtype="bf16", b=16,
                             N_max=513, w=128, B=Bv, N_total=(65792 if N_total is None else N_total), seed=seed,
                             keep_range=(2048, 8192))
    if i == 5:   # the geometry the paper itself runs (block size 256, window 16), budget 2048, 8B-like heads
        Bv = 256 if B is None else B
        return make_workload("paper-geometry-b256-w16", L=36 if L is None else L, h_kv=8, h_q=32, d=128, dtype="bf16", b=256,
                             N_max=9, w=16, B=Bv, N_total=(Bv * 9 + 64 if N_total is None else N_total), seed=seed)
    raise ValueError("config index must be 0..5")
