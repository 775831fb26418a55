"""Helpers shared by the tests: small random problems on the host, bf16 bit conversion.

Input preparation only - none of the method's arithmetic lives here.
"""
from __future__ import annotations

import numpy as np

import oracle


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    r = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return r.astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << 16).view(np.float32)


def as_float(a: np.ndarray) -> np.ndarray:
    """Pool / query tensor -> float64 values, whatever the storage type."""
    return (bf16_bits_to_f32(a) if a.dtype == np.uint16 else a).astype(np.float64)


def random_problem(seed, *, B=1, L=1, h_kv=1, G=1, d=8, b=4, N_max=3, w=2, extra_blocks=0, bf16=False,
                   N_total=None, valid_len=None, keep=None, num_blocks=None, heavy=0) -> oracle.Problem:
    """A seeded problem with shuffled block tables.  num_blocks: list per request (default N_max + extra_blocks)."""
    rng = np.random.default_rng(seed)
    nb = np.full(B, N_max + extra_blocks, dtype=np.int32) if num_blocks is None else np.asarray(num_blocks, dtype=np.int32)
    need = int(nb.sum())
    N_total = need + 3 if N_total is None else N_total
    perm = rng.permutation(N_total).astype(np.int32)
    table = np.full((B, int(nb.max())), -1, dtype=np.int32)
    pos = 0
    for n in range(B):
        table[n, : nb[n]] = perm[pos:pos + nb[n]]
        pos += nb[n]
    h_q = h_kv * G
    K = rng.standard_normal((L, N_total, b, h_kv, d)).astype(np.float32)
    V = rng.standard_normal((L, N_total, b, h_kv, d)).astype(np.float32)
    Q = rng.standard_normal((L, B + 1, w, h_q, d)).astype(np.float32)
    for _ in range(heavy):
        K[:, rng.integers(N_total), rng.integers(b)] *= 3.0
    if bf16:
        K, V, Q = f32_to_bf16_bits(K), f32_to_bf16_bits(V), f32_to_bf16_bits(Q)
    q_slot = rng.permutation(B + 1)[:B].astype(np.int32)
    return oracle.Problem(K=K, V=V, Q=Q, block_table=table, num_blocks=nb, q_slot=q_slot, N_max=N_max,
                          valid_len=valid_len, keep=keep)


def logical_keys(p: oracle.Problem, n: int, l: int, h: int, tensor: str = "K") -> np.ndarray:
    """Rows of request n in logical order: [T, d] float64."""
    src = getattr(p, tensor)
    N = int(p.num_blocks[n])
    blocks = p.block_table[n, :N]
    return as_float(src[l, blocks, :, h, :]).reshape(N * src.shape[2], src.shape[4])


def window_queries(p: oracle.Problem, n: int, l: int, hq: int) -> np.ndarray:
    """[w, d] float64."""
    return as_float(p.Q[l, p.q_slot[n], :, hq, :])
