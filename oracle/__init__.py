"""CPU oracle for the compression step of Compressed PagedAttention (numpy front end).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke()``
and by the ``cpu_baseline`` leg of ``bench.py``.  The product (the HIP library
and its binding) never imports this package, and this package imports nothing
of the product.

The arithmetic lives in ``zp_oracle.c`` (plain C, fp64, one loop nest per step
of the paper); this file only marshals numpy arrays into it.  Shapes follow the
paper's notation: K, V ``[L, N_total, b, h_kv, d]``; Q ``[L, M, w, h_q, d]``.
bf16 tensors are passed as ``uint16`` bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "zp_oracle.c")
_LIB = os.path.join(_HERE, "libzp_oracle.so")

F32, BF16 = 0, 1
OK, EINVAL, ENOMEM = 0, -1, -2


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP over independent units)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


class _Shape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("L", "N_total", "b", "h_kv", "h_q", "d", "M", "w", "dtype")]


class _Batch(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("N_max", ctypes.c_int32), ("max_blocks", ctypes.c_int32)] + [
        (n, ctypes.c_void_p) for n in ("block_table", "dst_table", "num_blocks", "q_slot", "valid_len", "keep")
    ]


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        for name in ("zo_score", "zo_select", "zo_compact", "zo_plan", "zo_decode_attention", "zo_threads", "zo_score_ex", "zo_refine", "zo_compact_global"):
            getattr(_lib, name).restype = ctypes.c_int
    return _lib


def threads() -> int:
    """Number of host threads the oracle's loops over units run on."""
    return int(_load().zo_threads())


@dataclass
class Problem:
    """One compression batch on host memory (numpy).  dtype: F32 or BF16 (uint16 bits)."""

    K: np.ndarray            # [L, N_total, b, h_kv, d]
    V: np.ndarray
    Q: np.ndarray            # [L, M, w, h_q, d]
    block_table: np.ndarray  # [B, max_blocks] int32
    num_blocks: np.ndarray   # [B] int32
    q_slot: np.ndarray       # [B] int32
    N_max: int
    valid_len: Optional[np.ndarray] = None  # [B, L, h_kv] int32
    keep: Optional[np.ndarray] = None       # [B, L, h_kv] int32
    dst_table: Optional[np.ndarray] = None  # [B, N_max-1] int32

    @property
    def dtype(self) -> int:
        return F32 if self.K.dtype == np.float32 else BF16

    @property
    def dims(self):
        L, N_total, b, h_kv, d = self.K.shape
        _, M, w, h_q, _ = self.Q.shape
        return L, N_total, b, h_kv, h_q, d, M, w

    @property
    def budget(self) -> int:
        return (self.N_max - 1) * self.K.shape[2]


def _i32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


def _ptr(a):
    return None if a is None else a.ctypes.data


def _structs(p: Problem):
    L, N_total, b, h_kv, h_q, d, M, w = p.dims
    assert p.K.dtype in (np.float32, np.uint16) and p.Q.dtype == p.K.dtype and p.V.dtype == p.K.dtype
    assert p.K.flags.c_contiguous and p.V.flags.c_contiguous and p.Q.flags.c_contiguous
    sh = _Shape(L, N_total, b, h_kv, h_q, d, M, w, p.dtype)
    keepalive = [_i32(p.block_table), _i32(p.dst_table), _i32(p.num_blocks), _i32(p.q_slot), _i32(p.valid_len), _i32(p.keep)]
    B, max_blocks = keepalive[0].shape
    bt = _Batch(B, p.N_max, max_blocks, *[_ptr(a) for a in keepalive])
    return sh, bt, keepalive


def _check(rc: int, what: str):
    if rc != OK:
        raise ValueError("%s: oracle status %d (%s)" % (what, rc, {EINVAL: "invalid argument", ENOMEM: "out of memory"}.get(rc, "?")))


def score(p: Problem) -> np.ndarray:
    """fp64 scores S ``[B, L, h_kv, max_blocks*b]`` (softmax -> max over group -> mean over window)."""
    sh, bt, keepalive = _structs(p)
    L, _, b, h_kv = p.K.shape[:4]
    out = np.empty((bt.B, L, h_kv, bt.max_blocks * b), dtype=np.float64)
    _check(_load().zo_score(ctypes.byref(sh), ctypes.byref(bt), ctypes.c_void_p(p.K.ctypes.data),
                            ctypes.c_void_p(p.Q.ctypes.data), ctypes.c_void_p(out.ctypes.data)), "score")
    return out


class _Extras(ctypes.Structure):
    _fields_ = [("F", ctypes.c_void_p), ("compressed", ctypes.c_void_p), ("alpha", ctypes.c_double), ("pool_kernel", ctypes.c_int32),
                ("lam", ctypes.c_double), ("tau", ctypes.c_double), ("p", ctypes.c_double), ("pool_first_only", ctypes.c_int32)]


@dataclass
class Extras:
    """Score refinements: global score (cache F, updated in place), max pooling, lightning redundancy."""
    F: Optional[np.ndarray] = None            # [L, N_total, b, h_kv] float32
    compressed: Optional[np.ndarray] = None   # [B] int32, nonzero = the request was compressed before
    alpha: float = 0.8
    pool_kernel: int = 1
    lam: float = 0.0
    tau: float = 1.0
    p: float = 1.0
    pool_first_only: bool = False             # pool only the requests without history


def score_ex(p: Problem, ex: Extras) -> np.ndarray:
    """Attention score followed by global score, pooling and S - lambda R (fp64); ex.F is updated in place."""
    sh, bt, keepalive = _structs(p)
    L, _, b, h_kv = p.K.shape[:4]
    if ex.F is not None:
        assert ex.F.dtype == np.float32 and ex.F.flags.c_contiguous and ex.F.shape == p.K.shape[:4]
    comp = _i32(ex.compressed)
    cx = _Extras(_ptr(ex.F), _ptr(comp), ex.alpha, ex.pool_kernel, ex.lam, ex.tau, ex.p, int(ex.pool_first_only))
    out = np.empty((bt.B, L, h_kv, bt.max_blocks * b), dtype=np.float64)
    _check(_load().zo_score_ex(ctypes.byref(sh), ctypes.byref(bt), ctypes.c_void_p(p.K.ctypes.data), ctypes.c_void_p(p.Q.ctypes.data),
                               ctypes.byref(cx), ctypes.c_void_p(out.ctypes.data)), "score_ex")
    return out


def refine(p: Problem, ex: Extras, scores: np.ndarray) -> np.ndarray:
    """The refinements of score_ex applied to given scores (any float type; computed in fp64); ex.F is updated in place."""
    sh, bt, keepalive = _structs(p)
    L, _, b, h_kv = p.K.shape[:4]
    if ex.F is not None:
        assert ex.F.dtype == np.float32 and ex.F.flags.c_contiguous and ex.F.shape == p.K.shape[:4]
    comp = _i32(ex.compressed)
    cx = _Extras(_ptr(ex.F), _ptr(comp), ex.alpha, ex.pool_kernel, ex.lam, ex.tau, ex.p, int(ex.pool_first_only))
    out = np.ascontiguousarray(scores, dtype=np.float64).copy()
    assert out.shape == (bt.B, L, h_kv, bt.max_blocks * b)
    _check(_load().zo_refine(ctypes.byref(sh), ctypes.byref(bt), ctypes.c_void_p(p.K.ctypes.data), ctypes.byref(cx),
                             ctypes.c_void_p(out.ctypes.data)), "refine")
    return out


def compact_global(p: Problem, F: np.ndarray, keep_idx: np.ndarray, ln: np.ndarray) -> None:
    """Move the cached global scores of the kept entries into the targets, in place in F."""
    sh, bt, keepalive = _structs(p)
    idx = np.ascontiguousarray(keep_idx, dtype=np.int32)
    ln = np.ascontiguousarray(ln, dtype=np.int32)
    assert F.dtype == np.float32 and F.flags.c_contiguous and F.shape == p.K.shape[:4]
    _check(_load().zo_compact_global(ctypes.byref(sh), ctypes.byref(bt), ctypes.c_void_p(F.ctypes.data),
                                     ctypes.c_void_p(idx.ctypes.data), ctypes.c_void_p(ln.ctypes.data)), "compact_global")


def select(p: Problem, scores_f32: np.ndarray):
    """Top-k_h selection on fp32 scores.  Returns (keep_idx [B,L,h_kv,budget] ascending, -1 padded; len [B,L,h_kv])."""
    sh, bt, keepalive = _structs(p)
    L, _, b, h_kv = p.K.shape[:4]
    s = np.ascontiguousarray(scores_f32, dtype=np.float32)
    assert s.shape[:3] == (bt.B, L, h_kv)
    idx = np.empty((bt.B, L, h_kv, p.budget), dtype=np.int32)
    ln = np.empty((bt.B, L, h_kv), dtype=np.int32)
    _check(_load().zo_select(ctypes.byref(sh), ctypes.byref(bt), ctypes.c_void_p(s.ctypes.data), ctypes.c_int32(s.shape[3]),
                             ctypes.c_void_p(idx.ctypes.data), ctypes.c_void_p(ln.ctypes.data)), "select")
    return idx, ln


def compact(p: Problem, keep_idx: np.ndarray, ln: np.ndarray) -> None:
    """Move the kept K and V rows into the targets, in place in ``p.K`` / ``p.V``."""
    sh, bt, keepalive = _structs(p)
    idx = np.ascontiguousarray(keep_idx, dtype=np.int32)
    ln = np.ascontiguousarray(ln, dtype=np.int32)
    assert idx.shape[-1] == p.budget
    _check(_load().zo_compact(ctypes.byref(sh), ctypes.byref(bt), ctypes.c_void_p(p.K.ctypes.data), ctypes.c_void_p(p.V.ctypes.data),
                              ctypes.c_void_p(idx.ctypes.data), ctypes.c_void_p(ln.ctypes.data)), "compact")


def compress(p: Problem):
    """score -> select -> compact.  Returns (scores fp64, keep_idx, len); p.K / p.V are compacted in place."""
    s = score(p)
    idx, ln = select(p, s.astype(np.float32))
    compact(p, idx, ln)
    return s, idx, ln


def plan(block_table, num_blocks, N_max: int, refcnt, free_in):
    """Targets, new tables, freed blocks and reference counts after a compression batch.

    Returns dict(dst_table, new_table, freed, n_free_used, refcnt) ; raises
    MemoryError when the free list runs out (nothing is changed then).
    """
    tbl = _i32(block_table)
    nb = _i32(num_blocks)
    rc_arr = np.array(refcnt, dtype=np.int32, copy=True)
    fr = _i32(np.asarray(free_in, dtype=np.int32).reshape(-1))
    B, max_blocks = tbl.shape
    dst = np.full((B, N_max - 1), -1, dtype=np.int32)
    new = np.full((B, N_max), -1, dtype=np.int32)
    freed = np.full((max(1, int(nb.sum())),), -1, dtype=np.int32)
    used = ctypes.c_int32(0)
    nfreed = ctypes.c_int32(0)
    rc = _load().zo_plan(ctypes.c_int32(B), ctypes.c_int32(N_max), ctypes.c_int32(max_blocks), ctypes.c_int32(rc_arr.shape[0]),
                         ctypes.c_void_p(tbl.ctypes.data), ctypes.c_void_p(nb.ctypes.data), ctypes.c_void_p(rc_arr.ctypes.data),
                         ctypes.c_void_p(fr.ctypes.data if fr.size else None), ctypes.c_int32(fr.size), ctypes.byref(used),
                         ctypes.c_void_p(dst.ctypes.data), ctypes.c_void_p(new.ctypes.data),
                         ctypes.c_void_p(freed.ctypes.data), ctypes.byref(nfreed))
    if rc == ENOMEM:
        raise MemoryError("plan: free list exhausted")
    _check(rc, "plan")
    return dict(dst_table=dst, new_table=new, freed=freed[: nfreed.value].copy(), n_free_used=used.value, refcnt=rc_arr)


def decode_attention(K, V, q, table, ln, h_q: int) -> np.ndarray:
    """Check-only paged decode attention: out[B, L, h_q, d] fp64 over the first len rows per kv head."""
    L, N_total, b, h_kv, d = K.shape
    tbl = _i32(table)
    ln = _i32(ln)
    B = tbl.shape[0]
    assert q.shape == (B, L, h_q, d) and q.dtype == K.dtype and q.flags.c_contiguous
    sh = _Shape(L, N_total, b, h_kv, h_q, d, 0, 0, F32 if K.dtype == np.float32 else BF16)
    out = np.empty((B, L, h_q, d), dtype=np.float64)
    _check(_load().zo_decode_attention(ctypes.byref(sh), ctypes.c_int32(B), ctypes.c_int32(tbl.shape[1]), ctypes.c_void_p(tbl.ctypes.data),
                                       ctypes.c_void_p(ln.ctypes.data), ctypes.c_void_p(K.ctypes.data), ctypes.c_void_p(V.ctypes.data),
                                       ctypes.c_void_p(q.ctypes.data), ctypes.c_void_p(out.ctypes.data)), "decode_attention")
    return out
