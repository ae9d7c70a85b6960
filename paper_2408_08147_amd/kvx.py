"""Thin ctypes binding of libkvx (include/kvx.h): argument marshalling only.

Every function has the name of the C entry point it calls.  Device memory is
passed as raw addresses (`tensor.data_ptr()`), streams as the integer value of
a hipStream_t (`torch.cuda.Stream().cuda_stream`).  There is no fallback: if
the HIP library cannot be loaded, importing a symbol from it raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence, Tuple

import numpy as np

from . import build as _build

(OK, ERR_INVALID_ARG, ERR_ALIGNMENT, ERR_BLOCK_TABLE, ERR_CAPACITY, ERR_UNSUPPORTED, ERR_DEVICE,
 ERR_BUSY, ERR_HOST_MEMORY) = range(9)
LAYOUT_LAYER_MAJOR, LAYOUT_PAGE_MAJOR = 0, 1
INNER_TOKEN_ROWS, INNER_HEAD_MAJOR, INNER_DIM_SPLIT_TOKEN, INNER_TOKEN_INNERMOST = 0, 1, 2, 3
OP_PACK, OP_UNPACK, OP_CONVERT = 0, 1, 2

EXPORTS = (
    "kvx_plan_workspace_bytes", "kvx_plan", "kvx_plan_destroy", "kvx_plan_total_bytes",
    "kvx_plan_segment", "kvx_plan_request_segment", "kvx_plan_get_tables", "kvx_plan_set_launch",
    "kvx_plan_get_launch", "kvx_plan_can_launch", "kvx_pack", "kvx_unpack", "kvx_convert", "kvx_pack_layers",
    "kvx_unpack_layers", "kvx_convert_layers", "kvx_pack_blockwise", "kvx_copy_yardstick",
    "kvx_retriever_arena_bytes", "kvx_retriever_create", "kvx_retriever_destroy", "kvx_retriever_acquire",
    "kvx_retriever_scatter", "kvx_retriever_abandon", "kvx_retriever_poll", "kvx_retriever_drain",
    "kvx_unpack_noalloc", "kvx_release_cached", "kvx_build_id", "kvx_status_string",
    "kvx_last_device_error",
)
NOALLOC_MAX_TABLE_WORDS = 896
INLINE_RUNS = 96
NOALLOC_SCRATCH_BYTES = 65536


class KvxError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        detail = ""
        if status == ERR_DEVICE:
            step = C.c_char_p(None)
            code = load().kvx_last_device_error(C.byref(step))
            detail = f"; hipError_t {code} at {(step.value or b'?').decode()}"
        super().__init__(f"{where}: {status_string(status)} (kvx_status {status}){detail}")


class PoolDesc(C.Structure):
    _fields_ = [("num_layers", C.c_uint32), ("num_kv_heads", C.c_uint32), ("head_dim", C.c_uint32),
                ("elem_bytes", C.c_uint32), ("page_tokens", C.c_uint32), ("num_pages", C.c_uint32),
                ("layout", C.c_uint32), ("inner", C.c_uint32),
                ("stride_layer", C.c_uint64), ("stride_kv", C.c_uint64),
                ("stride_page", C.c_uint64), ("stride_token", C.c_uint64)]

    @property
    def row_bytes(self) -> int:
        return self.num_kv_heads * self.head_dim * self.elem_bytes

    @property
    def dense_bytes(self) -> int:
        return self.num_layers * 2 * self.num_pages * self.page_tokens * self.row_bytes


class _BatchDesc(C.Structure):
    _fields_ = [("num_requests", C.c_uint32), ("reserved", C.c_uint32),
                ("seq_lens", C.c_void_p), ("block_ids", C.c_void_p), ("block_offsets", C.c_void_p)]


class LaunchCfg(C.Structure):
    _fields_ = [("unroll", C.c_uint32), ("nontemporal", C.c_uint32), ("order", C.c_uint32),
                ("xcd_swizzle", C.c_uint32), ("max_workgroups", C.c_uint32),
                ("threads", C.c_uint32), ("workgroups_per_cu", C.c_uint32), ("xcd_block_tiles", C.c_uint32)]


class PlanTables(C.Structure):
    _fields_ = [("token_prefix_off", C.c_uint64), ("run_prefix_off", C.c_uint64 * 3),
                ("runs_off", C.c_uint64 * 3), ("num_runs", C.c_uint64 * 3)]


RUN_DTYPE = np.dtype([("src_off", "<u8"), ("dst_off", "<u8"), ("bytes", "<u4"), ("seq_len", "<u4"),
                      ("request", "<u4"), ("token", "<u4")])


class BatchDesc:
    """Host-side batch (lengths + CSR block table); keeps its arrays alive."""

    def __init__(self, seq_lens, block_ids, block_offsets):
        self.seq_lens = np.ascontiguousarray(seq_lens, dtype=np.uint32)
        self.block_ids = np.ascontiguousarray(block_ids, dtype=np.uint32)
        self.block_offsets = np.ascontiguousarray(block_offsets, dtype=np.uint64)
        self._c = _BatchDesc(len(self.seq_lens), 0,
                             self.seq_lens.ctypes.data if self.seq_lens.size else None,
                             self.block_ids.ctypes.data if self.block_ids.size else None,
                             self.block_offsets.ctypes.data if self.block_offsets.size else None)

    def ref(self):
        return C.byref(self._c)


_lib = None


def lib_path() -> str:
    return _build.LIB


def load():
    """Loads libkvx.so.  A library that is missing, or was built from other sources than the ones beside
    it (the build bakes a hash of them in), is built first; if that cannot be done, loading fails."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if _build.is_stale():
        _build.build()
        if _build.is_stale():
            raise RuntimeError(f"{path} does not match the sources in {_build.CSRC} even after a rebuild")
    # The library must share ONE HIP runtime with whoever owns the streams and buffers it is handed.
    # PyTorch wheels carry their own copy of the runtime under another file name: were this library loaded
    # first, the loader would bring in the system copy for it and later PyTorch's for PyTorch, and a stream
    # or event of one is an invalid handle in the other.  With torch imported first, the dependency of this
    # library resolves (by soname) to the copy that is already in the process.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = C.CDLL(path)
    for name in EXPORTS:
        getattr(lib, name)  # raises AttributeError on a missing export
    lib.kvx_status_string.restype = C.c_char_p
    lib.kvx_status_string.argtypes = [C.c_int]
    lib.kvx_last_device_error.restype = C.c_int
    lib.kvx_last_device_error.argtypes = [C.POINTER(C.c_char_p)]
    lib.kvx_plan_destroy.restype = None
    lib.kvx_plan_destroy.argtypes = [C.c_void_p]
    lib.kvx_plan_workspace_bytes.argtypes = [C.c_void_p] * 4 + [C.POINTER(C.c_size_t)]
    lib.kvx_plan.argtypes = [C.c_void_p] * 4 + [C.c_uint32, C.c_uint32, C.c_void_p, C.c_size_t,
                                                 C.c_void_p, C.POINTER(C.c_void_p)]
    lib.kvx_plan_total_bytes.argtypes = [C.c_void_p, C.POINTER(C.c_uint64)]
    lib.kvx_plan_segment.argtypes = [C.c_void_p, C.c_uint32, C.c_uint32, C.POINTER(C.c_uint64),
                                     C.POINTER(C.c_uint64)]
    lib.kvx_plan_request_segment.argtypes = [C.c_void_p, C.c_uint32, C.POINTER(C.c_uint64),
                                             C.POINTER(C.c_uint64)]
    lib.kvx_plan_get_tables.argtypes = [C.c_void_p, C.POINTER(PlanTables)]
    lib.kvx_plan_set_launch.argtypes = [C.c_void_p, C.POINTER(LaunchCfg)]
    lib.kvx_plan_get_launch.argtypes = [C.c_void_p, C.POINTER(LaunchCfg)]
    lib.kvx_plan_can_launch.argtypes = [C.c_void_p, C.POINTER(C.c_int)]
    lib.kvx_pack.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p]
    lib.kvx_unpack.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p]
    lib.kvx_convert.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.kvx_pack_layers.argtypes = [C.c_void_p, C.c_uint32, C.c_uint32, C.c_void_p, C.c_void_p, C.c_uint64,
                                    C.c_void_p]
    lib.kvx_unpack_layers.argtypes = [C.c_void_p, C.c_uint32, C.c_uint32, C.c_void_p, C.c_uint64, C.c_void_p,
                                      C.c_void_p]
    lib.kvx_convert_layers.argtypes = [C.c_void_p, C.c_uint32, C.c_uint32, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.kvx_pack_blockwise.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64, C.c_uint32, C.c_void_p]
    lib.kvx_retriever_arena_bytes.argtypes = [C.c_uint32, C.c_uint64, C.c_uint64, C.POINTER(C.c_uint64)]
    lib.kvx_retriever_create.argtypes = [C.c_uint32, C.c_uint64, C.c_uint64, C.c_void_p, C.c_uint64,
                                         C.POINTER(C.c_void_p)]
    lib.kvx_retriever_destroy.argtypes = [C.c_void_p]
    lib.kvx_retriever_destroy.restype = None
    lib.kvx_retriever_acquire.argtypes = [C.c_void_p, C.c_uint64, C.c_uint64, C.POINTER(C.c_uint32),
                                          C.POINTER(C.c_void_p), C.POINTER(C.c_void_p)]
    lib.kvx_retriever_scatter.argtypes = [C.c_void_p, C.c_uint32, C.c_void_p, C.c_void_p, C.c_uint32, C.c_uint32,
                                          C.c_void_p, C.POINTER(LaunchCfg)]
    lib.kvx_retriever_abandon.argtypes = [C.c_void_p, C.c_uint32]
    lib.kvx_retriever_poll.argtypes = [C.c_void_p, C.POINTER(C.c_uint64), C.c_uint32, C.POINTER(C.c_uint32)]
    lib.kvx_retriever_drain.argtypes = [C.c_void_p]
    lib.kvx_copy_yardstick.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64, C.POINTER(LaunchCfg), C.c_void_p]
    lib.kvx_unpack_noalloc.argtypes = [C.c_void_p, C.c_void_p, C.c_uint32, C.c_uint32, C.c_void_p, C.c_uint64,
                                       C.c_void_p, C.c_void_p]
    lib.kvx_release_cached.argtypes = [C.POINTER(C.c_uint64)]
    lib.kvx_build_id.restype = C.c_char_p
    lib.kvx_build_id.argtypes = []
    for name in EXPORTS:
        if name not in ("kvx_status_string", "kvx_plan_destroy", "kvx_retriever_destroy", "kvx_last_device_error",
                        "kvx_build_id"):
            getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load().kvx_status_string(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != OK:
        raise KvxError(status, where)


def _ref(desc):
    if desc is None:
        return None
    return desc.ref() if isinstance(desc, BatchDesc) else C.cast(C.pointer(desc), C.c_void_p)


def kvx_plan_workspace_bytes(s: Optional[PoolDesc], sb: Optional[BatchDesc],
                             d: Optional[PoolDesc], db: Optional[BatchDesc]) -> int:
    out = C.c_size_t(0)
    _check(load().kvx_plan_workspace_bytes(_ref(s), _ref(sb), _ref(d), _ref(db), C.byref(out)),
           "kvx_plan_workspace_bytes")
    return out.value


class Plan:
    """Owns a kvx_plan_t*.  Destroyed explicitly or when collected."""

    def __init__(self, handle: int):
        self.handle = C.c_void_p(handle)

    def destroy(self) -> None:
        if self.handle:
            load().kvx_plan_destroy(self.handle)
            self.handle = C.c_void_p(None)

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def kvx_plan(s: Optional[PoolDesc], sb: Optional[BatchDesc], d: Optional[PoolDesc],
             db: Optional[BatchDesc], layer_begin: int, layer_end: int,
             dev_workspace: int = 0, workspace_bytes: int = 0, stream: int = 0) -> Plan:
    out = C.c_void_p(None)
    _check(load().kvx_plan(_ref(s), _ref(sb), _ref(d), _ref(db), layer_begin, layer_end,
                           C.c_void_p(dev_workspace or None), workspace_bytes,
                           C.c_void_p(stream or None), C.byref(out)), "kvx_plan")
    return Plan(out.value)


def kvx_plan_destroy(plan: Plan) -> None:
    plan.destroy()


def kvx_plan_total_bytes(plan: Plan) -> int:
    out = C.c_uint64(0)
    _check(load().kvx_plan_total_bytes(plan.handle, C.byref(out)), "kvx_plan_total_bytes")
    return out.value


def kvx_plan_segment(plan: Plan, request: int, layer: int) -> Tuple[int, int]:
    off, ln = C.c_uint64(0), C.c_uint64(0)
    _check(load().kvx_plan_segment(plan.handle, request, layer, C.byref(off), C.byref(ln)),
           "kvx_plan_segment")
    return off.value, ln.value


def kvx_plan_request_segment(plan: Plan, request: int) -> Tuple[int, int]:
    off, ln = C.c_uint64(0), C.c_uint64(0)
    _check(load().kvx_plan_request_segment(plan.handle, request, C.byref(off), C.byref(ln)),
           "kvx_plan_request_segment")
    return off.value, ln.value


def kvx_plan_get_tables(plan: Plan) -> PlanTables:
    t = PlanTables()
    _check(load().kvx_plan_get_tables(plan.handle, C.byref(t)), "kvx_plan_get_tables")
    return t


def kvx_plan_set_launch(plan: Plan, unroll: int = 0, nontemporal: int = 0, order: int = 0,
                        xcd_swizzle: int = 0, max_workgroups: int = 0, threads: int = 0,
                        workgroups_per_cu: int = 0, xcd_block_tiles: int = 0) -> None:
    cfg = LaunchCfg(unroll, nontemporal, order, xcd_swizzle, max_workgroups, threads, workgroups_per_cu,
                    xcd_block_tiles)
    _check(load().kvx_plan_set_launch(plan.handle, C.byref(cfg)), "kvx_plan_set_launch")


def kvx_plan_can_launch(plan: Plan) -> bool:
    out = C.c_int(0)
    _check(load().kvx_plan_can_launch(plan.handle, C.byref(out)), "kvx_plan_can_launch")
    return bool(out.value)


def kvx_plan_get_launch(plan: Plan) -> LaunchCfg:
    cfg = LaunchCfg()
    _check(load().kvx_plan_get_launch(plan.handle, C.byref(cfg)), "kvx_plan_get_launch")
    return cfg


def kvx_pack(plan: Plan, src_pool: int, buf: int, buf_bytes: int, stream: int = 0) -> None:
    _check(load().kvx_pack(plan.handle, C.c_void_p(src_pool or None), C.c_void_p(buf or None), buf_bytes,
                           C.c_void_p(stream or None)), "kvx_pack")


def kvx_unpack(plan: Plan, buf: int, buf_bytes: int, dst_pool: int, stream: int = 0) -> None:
    _check(load().kvx_unpack(plan.handle, C.c_void_p(buf or None), buf_bytes, C.c_void_p(dst_pool or None),
                             C.c_void_p(stream or None)), "kvx_unpack")


def kvx_convert(plan: Plan, src_pool: int, dst_pool: int, stream: int = 0) -> None:
    _check(load().kvx_convert(plan.handle, C.c_void_p(src_pool or None), C.c_void_p(dst_pool or None),
                              C.c_void_p(stream or None)), "kvx_convert")


def kvx_pack_layers(plan: Plan, layer_begin: int, layer_end: int, src_pool: int, buf: int, buf_bytes: int,
                    stream: int = 0) -> None:
    _check(load().kvx_pack_layers(plan.handle, layer_begin, layer_end, C.c_void_p(src_pool or None),
                                  C.c_void_p(buf or None), buf_bytes, C.c_void_p(stream or None)),
           "kvx_pack_layers")


def kvx_unpack_layers(plan: Plan, layer_begin: int, layer_end: int, buf: int, buf_bytes: int, dst_pool: int,
                      stream: int = 0) -> None:
    _check(load().kvx_unpack_layers(plan.handle, layer_begin, layer_end, C.c_void_p(buf or None), buf_bytes,
                                    C.c_void_p(dst_pool or None), C.c_void_p(stream or None)),
           "kvx_unpack_layers")


def kvx_convert_layers(plan: Plan, layer_begin: int, layer_end: int, src_pool: int, dst_pool: int,
                       stream: int = 0) -> None:
    _check(load().kvx_convert_layers(plan.handle, layer_begin, layer_end, C.c_void_p(src_pool or None),
                                     C.c_void_p(dst_pool or None), C.c_void_p(stream or None)),
           "kvx_convert_layers")


def kvx_pack_blockwise(plan: Plan, src_pool: int, buf: int, buf_bytes: int, confirm_every: int = 0,
                       stream: int = 0) -> None:
    _check(load().kvx_pack_blockwise(plan.handle, C.c_void_p(src_pool or None), C.c_void_p(buf or None),
                                     buf_bytes, confirm_every, C.c_void_p(stream or None)),
           "kvx_pack_blockwise")


def kvx_copy_yardstick(dst: int, src: int, nbytes: int, stream: int = 0, unroll: int = 0,
                       nontemporal: int = 0, max_workgroups: int = 0, threads: int = 0) -> None:
    cfg = LaunchCfg(unroll, nontemporal, 0, 0, max_workgroups, threads)
    _check(load().kvx_copy_yardstick(C.c_void_p(dst or None), C.c_void_p(src or None), nbytes, C.byref(cfg),
                                     C.c_void_p(stream or None)), "kvx_copy_yardstick")


def kvx_retriever_arena_bytes(num_slots: int, slot_buf_bytes: int, slot_ws_bytes: int) -> int:
    out = C.c_uint64(0)
    _check(load().kvx_retriever_arena_bytes(num_slots, slot_buf_bytes, slot_ws_bytes, C.byref(out)),
           "kvx_retriever_arena_bytes")
    return out.value


class Retriever:
    """Owns a kvx_retriever_t*."""

    def __init__(self, handle: int):
        self.handle = C.c_void_p(handle)

    def destroy(self) -> None:
        if self.handle:
            load().kvx_retriever_destroy(self.handle)
            self.handle = C.c_void_p(None)

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def kvx_retriever_create(num_slots: int, slot_buf_bytes: int, slot_ws_bytes: int, dev_arena: int,
                         arena_bytes: int) -> Retriever:
    out = C.c_void_p(None)
    _check(load().kvx_retriever_create(num_slots, slot_buf_bytes, slot_ws_bytes, C.c_void_p(dev_arena or None),
                                       arena_bytes, C.byref(out)), "kvx_retriever_create")
    return Retriever(out.value)


def kvx_retriever_destroy(ret: Retriever) -> None:
    ret.destroy()


def kvx_retriever_acquire(ret: Retriever, ticket: int, need_bytes: int) -> Tuple[int, int, int]:
    """Returns (slot, slot_buf address, slot stream handle)."""
    slot, buf, stream = C.c_uint32(0), C.c_void_p(None), C.c_void_p(None)
    _check(load().kvx_retriever_acquire(ret.handle, ticket, need_bytes, C.byref(slot), C.byref(buf),
                                        C.byref(stream)), "kvx_retriever_acquire")
    return slot.value, buf.value or 0, stream.value or 0


def kvx_retriever_scatter(ret: Retriever, slot: int, d: PoolDesc, db: BatchDesc, layer_begin: int,
                          layer_end: int, dst_pool: int, launch: Optional[LaunchCfg] = None) -> None:
    _check(load().kvx_retriever_scatter(ret.handle, slot, _ref(d), _ref(db), layer_begin, layer_end,
                                        C.c_void_p(dst_pool or None), C.byref(launch) if launch else None),
           "kvx_retriever_scatter")


def kvx_retriever_abandon(ret: Retriever, slot: int) -> None:
    _check(load().kvx_retriever_abandon(ret.handle, slot), "kvx_retriever_abandon")


def kvx_retriever_poll(ret: Retriever, capacity: int = 64):
    """Returns the list of tickets completed since they were last reported."""
    arr = (C.c_uint64 * max(capacity, 1))()
    n = C.c_uint32(0)
    _check(load().kvx_retriever_poll(ret.handle, arr, capacity, C.byref(n)), "kvx_retriever_poll")
    return [int(arr[i]) for i in range(n.value)]


def kvx_retriever_drain(ret: Retriever) -> None:
    _check(load().kvx_retriever_drain(ret.handle), "kvx_retriever_drain")


def kvx_unpack_noalloc(d: PoolDesc, db: BatchDesc, layer_begin: int, layer_end: int, buf: int, buf_bytes: int,
                       dst_pool: int, stream: int = 0) -> None:
    _check(load().kvx_unpack_noalloc(_ref(d), _ref(db), layer_begin, layer_end, C.c_void_p(buf or None), buf_bytes,
                                     C.c_void_p(dst_pool or None), C.c_void_p(stream or None)),
           "kvx_unpack_noalloc")


def kvx_release_cached() -> int:
    """Returns the pinned host bytes given back."""
    out = C.c_uint64(0)
    _check(load().kvx_release_cached(C.byref(out)), "kvx_release_cached")
    return out.value


def kvx_build_id() -> str:
    return load().kvx_build_id().decode()


def pool_desc(num_layers: int, num_kv_heads: int, head_dim: int, elem_bytes: int, page_tokens: int,
              num_pages: int, layout: int = LAYOUT_LAYER_MAJOR,
              strides: Sequence[int] = (0, 0, 0, 0), inner: int = INNER_TOKEN_ROWS) -> PoolDesc:
    return PoolDesc(num_layers, num_kv_heads, head_dim, elem_bytes, page_tokens, num_pages, layout, inner,
                    *strides)
