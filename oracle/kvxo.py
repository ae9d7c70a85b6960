"""ctypes front end of the CPU oracle (oracle/kvxo.c).  TEST INFRASTRUCTURE ONLY.

Pools and buffers are numpy uint8 arrays; block tables are CSR (uint32 ids,
uint64 offsets).  Nothing here does any of the method's arithmetic: it marshals
arguments and calls the C functions, which follow section 3.6 of the paper.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import numpy as np

from . import build as _build

_lib = None


class _Pool(C.Structure):
    _fields_ = [("num_layers", C.c_uint32), ("num_kv_heads", C.c_uint32), ("head_dim", C.c_uint32),
                ("elem_bytes", C.c_uint32), ("page_tokens", C.c_uint32), ("num_pages", C.c_uint32),
                ("layout", C.c_uint32), ("inner", C.c_uint32),
                ("stride_layer", C.c_uint64), ("stride_kv", C.c_uint64),
                ("stride_page", C.c_uint64), ("stride_token", C.c_uint64)]


class _Batch(C.Structure):
    _fields_ = [("num_requests", C.c_uint32), ("reserved", C.c_uint32),
                ("seq_lens", C.c_void_p), ("block_ids", C.c_void_p), ("block_offsets", C.c_void_p)]


def lib():
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path):
            _build.build()
        _lib = C.CDLL(path)
        for name in ("kvxo_total_bytes", "kvxo_segment", "kvxo_pack", "kvxo_unpack", "kvxo_convert"):
            getattr(_lib, name).restype = C.c_int
    return _lib


@dataclass
class Pool:
    num_layers: int
    num_kv_heads: int
    head_dim: int
    elem_bytes: int
    page_tokens: int
    num_pages: int
    layout: int = 0
    stride_layer: int = 0
    stride_kv: int = 0
    stride_page: int = 0
    stride_token: int = 0
    inner: int = 0          # arrangement inside a page: 0 [token][head][dim], 1 [head][token][dim],
                            # 2 [head][dim/x][token][x] with x = 16/elem_bytes, 3 [head][dim][token]

    def c(self) -> _Pool:
        return _Pool(self.num_layers, self.num_kv_heads, self.head_dim, self.elem_bytes,
                     self.page_tokens, self.num_pages, self.layout, self.inner,
                     self.stride_layer, self.stride_kv, self.stride_page, self.stride_token)

    @property
    def row(self) -> int:
        return self.num_kv_heads * self.head_dim * self.elem_bytes

    @property
    def nbytes(self) -> int:
        """Size of a densely laid out pool of this geometry (named layouts only)."""
        return self.num_layers * 2 * self.num_pages * self.page_tokens * self.row


class Batch:
    """Keeps the numpy arrays alive for as long as the C struct is in use."""

    def __init__(self, seq_lens, block_ids, block_offsets):
        self.seq_lens = np.ascontiguousarray(seq_lens, dtype=np.uint32)
        self.block_ids = np.ascontiguousarray(block_ids, dtype=np.uint32)
        self.block_offsets = np.ascontiguousarray(block_offsets, dtype=np.uint64)
        assert self.block_offsets.shape[0] == self.seq_lens.shape[0] + 1

    def c(self) -> _Batch:
        return _Batch(len(self.seq_lens), 0, self.seq_lens.ctypes.data,
                      self.block_ids.ctypes.data, self.block_offsets.ctypes.data)


def _u8(a: np.ndarray) -> int:
    assert a.dtype == np.uint8 and a.flags.c_contiguous
    return a.ctypes.data


def total_bytes(pool: Pool, batch: Batch, l0: int, l1: int) -> int:
    out = C.c_uint64(0)
    p, b = pool.c(), batch.c()
    rc = lib().kvxo_total_bytes(C.byref(p), C.byref(b), C.c_uint32(l0), C.c_uint32(l1), C.byref(out))
    if rc:
        raise ValueError("kvxo_total_bytes: bad arguments")
    return out.value


def segment(pool: Pool, batch: Batch, l0: int, l1: int, r: int, layer: int):
    off, ln = C.c_uint64(0), C.c_uint64(0)
    p, b = pool.c(), batch.c()
    rc = lib().kvxo_segment(C.byref(p), C.byref(b), C.c_uint32(l0), C.c_uint32(l1),
                            C.c_uint32(r), C.c_uint32(layer), C.byref(off), C.byref(ln))
    if rc:
        raise ValueError("kvxo_segment: bad arguments")
    return off.value, ln.value


def pack(pool: Pool, batch: Batch, l0: int, l1: int, src_pool: np.ndarray, buf: np.ndarray,
         threads: int = 1) -> None:
    assert buf.nbytes >= total_bytes(pool, batch, l0, l1)
    p, b = pool.c(), batch.c()
    rc = lib().kvxo_pack(C.byref(p), C.byref(b), C.c_uint32(l0), C.c_uint32(l1),
                         C.c_void_p(_u8(src_pool)), C.c_void_p(_u8(buf)), C.c_int(threads))
    if rc:
        raise ValueError("kvxo_pack: block table does not cover the request or leaves the pool")


def unpack(pool: Pool, batch: Batch, l0: int, l1: int, buf: np.ndarray, dst_pool: np.ndarray,
           threads: int = 1) -> None:
    assert buf.nbytes >= total_bytes(pool, batch, l0, l1)
    p, b = pool.c(), batch.c()
    rc = lib().kvxo_unpack(C.byref(p), C.byref(b), C.c_uint32(l0), C.c_uint32(l1),
                           C.c_void_p(_u8(buf)), C.c_void_p(_u8(dst_pool)), C.c_int(threads))
    if rc:
        raise ValueError("kvxo_unpack: block table does not cover the request or leaves the pool")


def convert(spool: Pool, sbatch: Batch, dpool: Pool, dbatch: Batch, l0: int, l1: int,
            src: np.ndarray, dst: np.ndarray, threads: int = 1) -> None:
    ps, bs, pd, bd = spool.c(), sbatch.c(), dpool.c(), dbatch.c()
    rc = lib().kvxo_convert(C.byref(ps), C.byref(bs), C.byref(pd), C.byref(bd),
                            C.c_uint32(l0), C.c_uint32(l1),
                            C.c_void_p(_u8(src)), C.c_void_p(_u8(dst)), C.c_int(threads))
    if rc:
        raise ValueError("kvxo_convert: mismatched sides or bad block table")
