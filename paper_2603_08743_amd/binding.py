"""Thin ctypes binding over libzp.so: same names as the C ABI (include/zp.h), argument marshalling only.

PyTorch supplies device memory and the stream; every step of the path runs in the HIP
kernels of the library.  There is no CPU fallback: a missing library or GPU raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libzp.so")

ZP_OK, ZP_EINVAL, ZP_ENOMEM, ZP_EHIP, ZP_EUNSUPPORTED = 0, -1, -2, -3, -4
ZP_F32, ZP_BF16 = 0, 1
ZP_OPT_SPLIT, ZP_OPT_SPIN_LIMIT, ZP_OPT_STREAMS, ZP_OPT_XCD_MAP = 1, 2, 3, 4

EXPORTS = ("zp_create", "zp_destroy", "zp_last_error", "zp_scratch_bytes", "zp_score", "zp_select_topk", "zp_compact_kv",
           "zp_compress", "zp_sync_status", "zp_validate_batch", "zp_plan", "zp_set_option", "zp_decode_attention", "zp_score_ex",
           "zp_compact_kv_ex", "zp_compress_ex", "zp_compress_static")


class ZpError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("zp status %d: %s" % (status, message))
        self.status = status


class _Pool(ctypes.Structure):
    _fields_ = [("k", ctypes.c_void_p), ("v", ctypes.c_void_p), ("q", ctypes.c_void_p)] + [
        (n, ctypes.c_int32) for n in ("layer0", "L_slab", "N_total", "b", "h_kv", "h_q", "d", "M", "w", "dtype")]


class _Batch(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("B", "N_max", "max_blocks", "L")] + [
        (n, ctypes.c_void_p) for n in ("block_table", "dst_table", "num_blocks", "q_slot", "valid_len", "keep")]


class _Extras(ctypes.Structure):
    _fields_ = [("F", ctypes.c_void_p), ("compressed", ctypes.c_void_p), ("alpha", ctypes.c_float), ("pool_kernel", ctypes.c_int32),
                ("lam", ctypes.c_float), ("tau", ctypes.c_float), ("p", ctypes.c_float), ("pool_first_only", ctypes.c_int32)]


_lib = None


def load_library() -> ctypes.CDLL:
    """Load libzp.so (built in tree by ``paper_2603_08743_amd.build``); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError("%s not built: run `python -m paper_2603_08743_amd.build` (needs hipcc)" % LIB_PATH)
        lib = ctypes.CDLL(LIB_PATH)
        for name in EXPORTS:
            getattr(lib, name).restype = ctypes.c_int
        lib.zp_last_error.restype = ctypes.c_char_p
        lib.zp_last_error.argtypes = [ctypes.c_void_p]
        lib.zp_scratch_bytes.restype = ctypes.c_size_t
        lib.zp_destroy.restype = None
        lib.zp_destroy.argtypes = [ctypes.c_void_p]
        _lib = lib
    return _lib


@dataclass
class Pool:
    """Device tensors of one layer slab: K, V ``[L_slab, N_total, b, h_kv, d]``, Q ``[L_slab, M, w, h_q, d]``."""
    k: torch.Tensor
    v: torch.Tensor
    q: torch.Tensor
    layer0: int = 0

    def c(self) -> _Pool:
        k, v, q = self.k, self.v, self.q
        assert k.is_cuda and v.is_cuda and q.is_cuda and k.is_contiguous() and v.is_contiguous() and q.is_contiguous()
        assert k.dtype == v.dtype == q.dtype and k.dtype in (torch.float32, torch.bfloat16) and k.shape == v.shape
        Ls, N_total, b, h_kv, d = k.shape
        Lq, M, w, h_q, dq = q.shape
        assert Lq == Ls and dq == d
        return _Pool(k.data_ptr(), v.data_ptr(), q.data_ptr(), self.layer0, Ls, N_total, b, h_kv, h_q, d, M, w,
                     ZP_F32 if k.dtype == torch.float32 else ZP_BF16)


def _i32ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    assert t.is_cuda and t.dtype == torch.int32 and t.is_contiguous()
    return t.data_ptr()


@dataclass
class Batch:
    """Device int32 tensors of one compression batch (see zp_batch in include/zp.h)."""
    block_table: torch.Tensor          # [B, max_blocks]
    num_blocks: torch.Tensor           # [B]
    q_slot: torch.Tensor               # [B]
    N_max: int
    L: int                             # layers the per-unit arrays are laid out for
    dst_table: Optional[torch.Tensor] = None   # [B, N_max-1]
    valid_len: Optional[torch.Tensor] = None   # [B, L, h_kv]
    keep: Optional[torch.Tensor] = None        # [B, L, h_kv]

    def c(self) -> _Batch:
        B, max_blocks = self.block_table.shape
        return _Batch(B, self.N_max, max_blocks, self.L, _i32ptr(self.block_table), _i32ptr(self.dst_table),
                      _i32ptr(self.num_blocks), _i32ptr(self.q_slot), _i32ptr(self.valid_len), _i32ptr(self.keep))


@dataclass
class Extras:
    """Score refinements (see zp_extras in include/zp.h)."""
    F: Optional[torch.Tensor] = None            # [L_slab, N_total, b, h_kv] float32, updated in place
    compressed: Optional[torch.Tensor] = None   # [B] int32
    alpha: float = 0.8
    pool_kernel: int = 1
    lam: float = 0.0
    tau: float = 1.0
    p: float = 1.0
    pool_first_only: bool = False

    def c(self, pool: _Pool) -> _Extras:
        if self.F is not None:
            assert self.F.is_cuda and self.F.dtype == torch.float32 and self.F.is_contiguous()
            assert tuple(self.F.shape) == (pool.L_slab, pool.N_total, pool.b, pool.h_kv)
        return _Extras(None if self.F is None else self.F.data_ptr(), _i32ptr(self.compressed), self.alpha, self.pool_kernel,
                       self.lam, self.tau, self.p, int(self.pool_first_only))


def _stream() -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


class Context:
    """zp_ctx wrapper.  Methods carry the names of the C entry points."""

    def __init__(self):
        self.lib = load_library()
        if not torch.cuda.is_available():
            raise RuntimeError("libzp needs a GPU: no HIP device is visible")
        torch.cuda.init()
        h = ctypes.c_void_p()
        rc = self.lib.zp_create(ctypes.byref(h))
        if rc != ZP_OK:
            raise ZpError(rc, self.lib.zp_last_error(None).decode())
        self.h = h

    def close(self):
        if getattr(self, "h", None):
            self.lib.zp_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc: int):
        if rc != ZP_OK:
            raise ZpError(rc, self.lib.zp_last_error(self.h).decode())

    def zp_score(self, pool: Pool, batch: Batch, scores: torch.Tensor) -> None:
        assert scores.is_cuda and scores.dtype == torch.float32 and scores.is_contiguous()
        p, b = pool.c(), batch.c()
        assert scores.numel() == b.B * p.L_slab * p.h_kv * b.max_blocks * p.b
        self._check(self.lib.zp_score(self.h, ctypes.byref(p), ctypes.byref(b), ctypes.c_void_p(scores.data_ptr()), _stream()))

    def zp_select_topk(self, scores: torch.Tensor, pool: Pool, batch: Batch, keep_idx: torch.Tensor, len_out: torch.Tensor) -> None:
        assert scores.is_cuda and scores.dtype == torch.float32 and scores.is_contiguous()
        assert keep_idx.dtype == torch.int32 and len_out.dtype == torch.int32 and keep_idx.is_contiguous() and len_out.is_contiguous()
        p, b = pool.c(), batch.c()
        units = b.B * p.L_slab * p.h_kv
        assert keep_idx.numel() == units * (b.N_max - 1) * p.b and len_out.numel() == units
        self._check(self.lib.zp_select_topk(self.h, ctypes.c_void_p(scores.data_ptr()), ctypes.c_int32(scores.shape[-1]), ctypes.byref(p),
                                            ctypes.byref(b), ctypes.c_void_p(keep_idx.data_ptr()), ctypes.c_void_p(len_out.data_ptr()), _stream()))

    def zp_compact_kv(self, pool: Pool, batch: Batch, keep_idx: torch.Tensor, length: torch.Tensor) -> None:
        assert keep_idx.is_cuda and keep_idx.dtype == torch.int32 and length.dtype == torch.int32
        p, b = pool.c(), batch.c()
        units = b.B * p.L_slab * p.h_kv
        assert keep_idx.numel() == units * (b.N_max - 1) * p.b and length.numel() == units
        self._check(self.lib.zp_compact_kv(self.h, ctypes.byref(p), ctypes.byref(b), ctypes.c_void_p(keep_idx.data_ptr()),
                                           ctypes.c_void_p(length.data_ptr()), _stream()))

    def zp_compress(self, pool: Pool, batch: Batch, len_out: torch.Tensor, scores_dbg: Optional[torch.Tensor] = None,
                    keep_idx_dbg: Optional[torch.Tensor] = None) -> None:
        p, b = pool.c(), batch.c()
        units = b.B * p.L_slab * p.h_kv
        assert len_out.is_cuda and len_out.dtype == torch.int32 and len_out.numel() == units
        if scores_dbg is not None:
            assert scores_dbg.dtype == torch.float32 and scores_dbg.is_contiguous() and scores_dbg.numel() == units * b.max_blocks * p.b
        if keep_idx_dbg is not None:
            assert keep_idx_dbg.dtype == torch.int32 and keep_idx_dbg.is_contiguous() and keep_idx_dbg.numel() == units * (b.N_max - 1) * p.b
        self._check(self.lib.zp_compress(self.h, ctypes.byref(p), ctypes.byref(b), ctypes.c_void_p(len_out.data_ptr()),
                                         ctypes.c_void_p(scores_dbg.data_ptr() if scores_dbg is not None else None),
                                         ctypes.c_void_p(keep_idx_dbg.data_ptr() if keep_idx_dbg is not None else None), _stream()))

    def zp_score_ex(self, pool: Pool, batch: Batch, extras: Extras, scores: torch.Tensor) -> None:
        assert scores.is_cuda and scores.dtype == torch.float32 and scores.is_contiguous()
        p, b = pool.c(), batch.c()
        x = extras.c(p)
        assert scores.numel() == b.B * p.L_slab * p.h_kv * b.max_blocks * p.b
        self._check(self.lib.zp_score_ex(self.h, ctypes.byref(p), ctypes.byref(b), ctypes.byref(x), ctypes.c_void_p(scores.data_ptr()), _stream()))

    def zp_compact_kv_ex(self, pool: Pool, batch: Batch, F: torch.Tensor, keep_idx: torch.Tensor, length: torch.Tensor) -> None:
        assert keep_idx.is_cuda and keep_idx.dtype == torch.int32 and length.dtype == torch.int32
        p, b = pool.c(), batch.c()
        units = b.B * p.L_slab * p.h_kv
        assert keep_idx.numel() == units * (b.N_max - 1) * p.b and length.numel() == units
        assert F.is_cuda and F.dtype == torch.float32 and F.is_contiguous() and tuple(F.shape) == (p.L_slab, p.N_total, p.b, p.h_kv)
        self._check(self.lib.zp_compact_kv_ex(self.h, ctypes.byref(p), ctypes.byref(b), ctypes.c_void_p(F.data_ptr()),
                                              ctypes.c_void_p(keep_idx.data_ptr()), ctypes.c_void_p(length.data_ptr()), _stream()))

    def zp_compress_ex(self, pool: Pool, batch: Batch, extras: Extras, len_out: torch.Tensor, scores_dbg: Optional[torch.Tensor] = None,
                       keep_idx_dbg: Optional[torch.Tensor] = None) -> None:
        p, b = pool.c(), batch.c()
        x = extras.c(p)
        units = b.B * p.L_slab * p.h_kv
        assert len_out.is_cuda and len_out.dtype == torch.int32 and len_out.numel() == units
        if scores_dbg is not None:
            assert scores_dbg.dtype == torch.float32 and scores_dbg.is_contiguous() and scores_dbg.numel() == units * b.max_blocks * p.b
        if keep_idx_dbg is not None:
            assert keep_idx_dbg.dtype == torch.int32 and keep_idx_dbg.is_contiguous() and keep_idx_dbg.numel() == units * (b.N_max - 1) * p.b
        self._check(self.lib.zp_compress_ex(self.h, ctypes.byref(p), ctypes.byref(b), ctypes.byref(x), ctypes.c_void_p(len_out.data_ptr()),
                                            ctypes.c_void_p(scores_dbg.data_ptr() if scores_dbg is not None else None),
                                            ctypes.c_void_p(keep_idx_dbg.data_ptr() if keep_idx_dbg is not None else None), _stream()))

    def zp_decode_attention(self, pool: Pool, table: torch.Tensor, length: torch.Tensor, q: torch.Tensor, out: torch.Tensor) -> None:
        """Check-only paged decode attention; q [B, L_slab, h_q, d] (pool dtype), out fp32 of the same shape."""
        p = pool.c()
        B, stride = table.shape
        assert q.is_cuda and q.is_contiguous() and q.dtype == pool.k.dtype and tuple(q.shape) == (B, p.L_slab, p.h_q, p.d)
        assert out.is_cuda and out.is_contiguous() and out.dtype == torch.float32 and out.shape == q.shape
        assert length.numel() == B * p.L_slab * p.h_kv
        self._check(self.lib.zp_decode_attention(self.h, ctypes.byref(p), ctypes.c_int32(B), ctypes.c_int32(stride),
                                                 ctypes.c_void_p(_i32ptr(table)), ctypes.c_void_p(_i32ptr(length)),
                                                 ctypes.c_void_p(q.data_ptr()), ctypes.c_void_p(out.data_ptr()), _stream()))

    def zp_set_option(self, option: int, value: int) -> None:
        self._check(self.lib.zp_set_option(self.h, ctypes.c_int32(option), ctypes.c_int32(value)))

    def zp_sync_status(self) -> None:
        self._check(self.lib.zp_sync_status(self.h, _stream()))

    def zp_validate_batch(self, pool: Pool, batch: Batch) -> None:
        p, b = pool.c(), batch.c()
        self._check(self.lib.zp_validate_batch(self.h, ctypes.byref(p), ctypes.byref(b)))

    def zp_scratch_bytes(self, pool: Pool, batch: Batch) -> int:
        p, b = pool.c(), batch.c()
        return int(self.lib.zp_scratch_bytes(ctypes.byref(p), ctypes.byref(b)))


def zp_compress_static(pool: Pool, batch: Batch, len_out: torch.Tensor) -> None:
    """zp_compress without a context and without any allocation (see include/zp.h); asynchronous on the current stream."""
    lib = load_library()
    if not torch.cuda.is_available():
        raise RuntimeError("libzp needs a GPU: no HIP device is visible")
    p, b = pool.c(), batch.c()
    assert len_out.is_cuda and len_out.dtype == torch.int32 and len_out.is_contiguous() and len_out.numel() == b.B * p.L_slab * p.h_kv
    rc = lib.zp_compress_static(ctypes.byref(p), ctypes.byref(b), ctypes.c_void_p(len_out.data_ptr()), _stream())
    if rc != ZP_OK:
        raise ZpError(rc, lib.zp_last_error(None).decode())


def zp_plan(block_table: np.ndarray, num_blocks: np.ndarray, N_max: int, refcnt: np.ndarray, free_in: np.ndarray):
    """Host planner (no GPU needed).  refcnt is updated in place.  Returns dict(dst_table, new_table, freed, n_free_used)."""
    lib = load_library()
    tbl = np.ascontiguousarray(block_table, dtype=np.int32)
    nb = np.ascontiguousarray(num_blocks, dtype=np.int32)
    fr = np.ascontiguousarray(np.asarray(free_in).reshape(-1), dtype=np.int32)
    assert refcnt.dtype == np.int32 and refcnt.flags.c_contiguous
    B, max_blocks = tbl.shape
    dst = np.full((B, N_max - 1), -1, dtype=np.int32)
    new = np.full((B, N_max), -1, dtype=np.int32)
    freed = np.full((max(1, int(nb.sum())),), -1, dtype=np.int32)
    used, nfreed = ctypes.c_int32(0), ctypes.c_int32(0)
    p = lambda a: ctypes.c_void_p(a.ctypes.data if a.size else None)
    rc = lib.zp_plan(ctypes.c_int32(B), ctypes.c_int32(N_max), ctypes.c_int32(max_blocks), ctypes.c_int32(refcnt.shape[0]), p(tbl), p(nb),
                     p(refcnt), p(fr), ctypes.c_int32(fr.size), ctypes.byref(used), p(dst), p(new), p(freed), ctypes.byref(nfreed))
    if rc != ZP_OK:
        raise ZpError(rc, lib.zp_last_error(None).decode())
    return dict(dst_table=dst, new_table=new, freed=freed[: nfreed.value].copy(), n_free_used=used.value)
