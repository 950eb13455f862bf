"""Thin ctypes binding over the C ABI of ``include/kvd.h``.

Argument marshalling only: every step of the transfer (address translation, coalescing, the
copy) runs in the library's HIP kernels.  Function names mirror the C names; ``Pool`` and
``Plan`` are small handle owners.  There is no fallback: if ``libkvd.so`` has not been built
(``python -m paper_2501_14743_amd.build``) every call raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libkvd.so")

KVD_OK = 0
KVD_ERR_INVALID, KVD_ERR_RANGE, KVD_ERR_MISMATCH = -1, -2, -3
KVD_ERR_ALIAS, KVD_ERR_CAPACITY, KVD_ERR_HIP = -4, -5, -6
KVD_LAYOUT_BHTD, KVD_LAYOUT_BTHD = 0, 1
KVD_NOALLOC_MAX_BLOCKS = 8192
KVD_NOALLOC_MAX_WORK_ITEMS = 1 << 19
KVD_PLAN_NO_COALESCE = 1
KVD_PLAN_PERSISTENT = 2
KVD_PLAN_WHOLE_BLOCKS = 4
KVD_PLAN_QUEUE_ORDER = 8
KVD_PLAN_DESTINATION_ORDER = 64
KVD_PLAN_WIDE_OFFSETS = 16
KVD_PLAN_COMPLETE_PER_REQUEST = 32
KVD_ORDER_QUEUE, KVD_ORDER_REGIONS, KVD_ORDER_SORTED = 0, 1, 2
LAYOUTS = {"BHTD": KVD_LAYOUT_BHTD, "BTHD": KVD_LAYOUT_BTHD}


class KvdError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"kvd error {code}: {message}")
        self.code = code


class kvd_pool_desc_t(ctypes.Structure):
    _fields_ = [
        ("base", ctypes.c_void_p),
        ("num_layers", ctypes.c_uint32), ("num_blocks", ctypes.c_uint32),
        ("block_tokens", ctypes.c_uint32), ("num_kv_heads", ctypes.c_uint32),
        ("head_dim", ctypes.c_uint32), ("elem_bytes", ctypes.c_uint32),
        ("layout", ctypes.c_int32),
        ("stride_layer", ctypes.c_int64), ("stride_kv", ctypes.c_int64),
        ("stride_block", ctypes.c_int64),
    ]


class kvd_span_t(ctypes.Structure):
    _fields_ = [("src_offset", ctypes.c_uint64), ("dst_offset", ctypes.c_uint64),
                ("bytes", ctypes.c_uint64)]


class kvd_piece_t(ctypes.Structure):
    _fields_ = [("src_block", ctypes.c_int32), ("src_token", ctypes.c_uint32),
                ("dst_block", ctypes.c_int32), ("dst_token", ctypes.c_uint32),
                ("num_tokens", ctypes.c_uint32)]


class kvd_stats_t(ctypes.Structure):
    _fields_ = [("num_requests", ctypes.c_uint32), ("relayout", ctypes.c_uint32),
                ("num_src_blocks", ctypes.c_uint64), ("num_dst_blocks", ctypes.c_uint64),
                ("num_transactions", ctypes.c_uint64), ("num_descriptors", ctypes.c_uint64),
                ("num_work_items", ctypes.c_uint64), ("payload_bytes", ctypes.c_uint64),
                ("work_order", ctypes.c_uint32), ("reserved", ctypes.c_uint32)]


_lib: Optional[ctypes.CDLL] = None


def lib() -> ctypes.CDLL:
    """Load libkvd.so (once).  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2501_14743_amd.build`; "
                           "there is no fallback path")
    L = ctypes.CDLL(LIB_PATH)
    vp, u32, u64, i32p = ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint64, ctypes.POINTER(ctypes.c_int32)
    L.kvd_last_error.restype = ctypes.c_char_p
    L.kvd_last_error.argtypes = []
    L.kvd_pool_create.argtypes = [ctypes.POINTER(kvd_pool_desc_t), ctypes.POINTER(vp)]
    L.kvd_plan_create.argtypes = [vp, vp, u32, u32, u32, ctypes.POINTER(vp)]
    L.kvd_build_descriptors.argtypes = [vp, i32p, u32, i32p, u32, u32, u32, u32, vp]
    L.kvd_build_descriptors_batch.argtypes = [vp, u32, ctypes.POINTER(i32p), ctypes.POINTER(u32),
                                              ctypes.POINTER(i32p), ctypes.POINTER(u32), ctypes.POINTER(u32),
                                              u32, u32, vp]
    L.kvd_pull.argtypes = [vp, vp]
    L.kvd_pull_layers.argtypes = [vp, u32, u32, vp]
    L.kvd_pull_noalloc.argtypes = [ctypes.POINTER(kvd_pool_desc_t), ctypes.POINTER(kvd_pool_desc_t), i32p, u32, i32p, u32,
                                   u32, u32, u32, u32, vp]
    L.kvd_complete.argtypes = [vp, u64, vp]
    L.kvd_pull_notify.argtypes = [vp, vp, u64, vp]
    L.kvd_plan_set_completion_granularity.argtypes = [vp, u32]
    L.kvd_pull_blockwise_memcpy.argtypes = [vp, vp]
    L.kvd_pull_staged.argtypes = [vp, vp, vp, u64, vp]
    L.kvd_plan_reset.argtypes = [vp]
    L.kvd_plan_stats.argtypes = [vp, vp, ctypes.POINTER(kvd_stats_t)]
    L.kvd_plan_get_descriptors.argtypes = [vp, vp, ctypes.POINTER(kvd_span_t), ctypes.POINTER(kvd_piece_t),
                                           u64, ctypes.POINTER(u64)]
    L.kvd_copy_plain.argtypes = [vp, vp, u64, vp]
    L.kvd_stream_probe.argtypes = [vp, vp, u64, u32, vp]
    L.kvd_free.argtypes = [vp]
    L.kvd_free.restype = None
    for name in ("kvd_pool_create", "kvd_plan_create", "kvd_build_descriptors", "kvd_build_descriptors_batch", "kvd_pull",
                 "kvd_pull_layers", "kvd_pull_noalloc", "kvd_complete", "kvd_pull_notify",
                 "kvd_plan_set_completion_granularity",
                 "kvd_pull_blockwise_memcpy", "kvd_pull_staged", "kvd_plan_reset", "kvd_plan_stats",
                 "kvd_plan_get_descriptors", "kvd_copy_plain", "kvd_stream_probe"):
        getattr(L, name).restype = ctypes.c_int
    _lib = L
    return L


def kvd_last_error() -> str:
    return lib().kvd_last_error().decode()


def _check(rc: int) -> None:
    if rc != KVD_OK:
        raise KvdError(rc, kvd_last_error())


def _table(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def _i32p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)) if a.size else None


# ---------------------------------------------------------------- functions, named as in kvd.h

def kvd_pool_create(base: int, num_layers: int, num_blocks: int, block_tokens: int, num_kv_heads: int,
                    head_dim: int, elem_bytes: int, layout, stride_layer: int, stride_kv: int,
                    stride_block: int) -> int:
    d = kvd_pool_desc_t(base, num_layers, num_blocks, block_tokens, num_kv_heads, head_dim, elem_bytes,
                        LAYOUTS.get(layout, layout), stride_layer, stride_kv, stride_block)
    out = ctypes.c_void_p()
    _check(lib().kvd_pool_create(ctypes.byref(d), ctypes.byref(out)))
    return out.value


def kvd_plan_create(src_pool: int, dst_pool: int, max_requests: int, max_total_blocks: int, flags: int = 0) -> int:
    out = ctypes.c_void_p()
    _check(lib().kvd_plan_create(src_pool, dst_pool, max_requests, max_total_blocks, flags, ctypes.byref(out)))
    return out.value


def kvd_build_descriptors(plan: int, src_block_table, dst_block_table, seq_len: int, layer_begin: int,
                          layer_end: int, stream: int = 0) -> None:
    st, dt = _table(src_block_table), _table(dst_block_table)
    _check(lib().kvd_build_descriptors(plan, _i32p(st), st.size, _i32p(dt), dt.size, seq_len,
                                       layer_begin, layer_end, stream))


def kvd_build_descriptors_batch(plan: int, src_block_tables: Sequence, dst_block_tables: Sequence,
                                seq_lens: Sequence[int], layer_begin: int, layer_end: int, stream: int = 0) -> None:
    n = len(seq_lens)
    assert len(src_block_tables) == n and len(dst_block_tables) == n
    sts, dts = [_table(t) for t in src_block_tables], [_table(t) for t in dst_block_tables]
    i32p = ctypes.POINTER(ctypes.c_int32)
    sp = (i32p * n)(*[_i32p(t) if t.size else i32p() for t in sts])
    dp = (i32p * n)(*[_i32p(t) if t.size else i32p() for t in dts])
    ns = (ctypes.c_uint32 * n)(*[t.size for t in sts])
    nd = (ctypes.c_uint32 * n)(*[t.size for t in dts])
    sl = (ctypes.c_uint32 * n)(*[int(x) for x in seq_lens])
    _check(lib().kvd_build_descriptors_batch(plan, n, sp, ns, dp, nd, sl, layer_begin, layer_end, stream))


def kvd_pull(plan: int, stream: int = 0) -> None:
    _check(lib().kvd_pull(plan, stream))


def kvd_pull_layers(plan: int, layer_begin: int, layer_end: int, stream: int = 0) -> None:
    _check(lib().kvd_pull_layers(plan, layer_begin, layer_end, stream))


def pool_desc(base: int, geometry, stride_layer=None, stride_kv=None, stride_block=None) -> kvd_pool_desc_t:
    """kvd_pool_desc_t of a pool at `base` with the given geometry (strides from the geometry unless given)."""
    g = geometry
    return kvd_pool_desc_t(base, g.num_layers, g.num_blocks, g.block_tokens, g.num_kv_heads, g.head_dim, g.elem_bytes,
                           LAYOUTS.get(g.layout, g.layout), g.stride_layer if stride_layer is None else stride_layer,
                           g.stride_kv if stride_kv is None else stride_kv,
                           g.stride_block if stride_block is None else stride_block)


def kvd_pull_noalloc(src_desc: kvd_pool_desc_t, dst_desc: kvd_pool_desc_t, src_block_table, dst_block_table,
                     seq_len: int, layer_begin: int, layer_end: int, flags: int = 0, stream: int = 0) -> None:
    st, dt = _table(src_block_table), _table(dst_block_table)
    _check(lib().kvd_pull_noalloc(ctypes.byref(src_desc), ctypes.byref(dst_desc), _i32p(st), st.size, _i32p(dt), dt.size,
                                  seq_len, layer_begin, layer_end, flags, stream))


def kvd_pull_notify(plan: int, words_ptr: int, value: int, stream: int = 0) -> None:
    _check(lib().kvd_pull_notify(plan, words_ptr, value, stream))


def kvd_plan_set_completion_granularity(plan: int, min_tokens: int) -> None:
    _check(lib().kvd_plan_set_completion_granularity(plan, min_tokens))


def kvd_complete(flag_ptr: int, value: int, stream: int = 0) -> None:
    _check(lib().kvd_complete(flag_ptr, value, stream))


def kvd_pull_blockwise_memcpy(plan: int, stream: int = 0) -> None:
    _check(lib().kvd_pull_blockwise_memcpy(plan, stream))


def kvd_pull_staged(plan: int, send_buffer: int, recv_buffer: int, buffer_bytes: int, stream: int = 0) -> None:
    _check(lib().kvd_pull_staged(plan, send_buffer, recv_buffer, buffer_bytes, stream))


def kvd_plan_reset(plan: int) -> None:
    _check(lib().kvd_plan_reset(plan))


def kvd_plan_stats(plan: int, stream: int = 0) -> dict:
    s = kvd_stats_t()
    _check(lib().kvd_plan_stats(plan, stream, ctypes.byref(s)))
    return {k: int(getattr(s, k)) for k, _ in kvd_stats_t._fields_}


def kvd_plan_get_descriptors(plan: int, stream: int = 0) -> np.ndarray:
    """Spans as an (n, 3) int64 array [src_offset, dst_offset, bytes] for byte-copy plans, pieces as
    an (n, 5) array [src_block, src_token, dst_block, dst_token, num_tokens] for re-layout plans."""
    relayout = kvd_plan_stats(plan, stream)["relayout"]
    n = ctypes.c_uint64()
    dummy_s, dummy_p = (kvd_span_t * 1)(), (kvd_piece_t * 1)()
    _check(lib().kvd_plan_get_descriptors(plan, stream, dummy_s, dummy_p, 0, ctypes.byref(n)))
    cap = max(int(n.value), 1)
    spans, pieces = (kvd_span_t * cap)(), (kvd_piece_t * cap)()
    _check(lib().kvd_plan_get_descriptors(plan, stream, spans, pieces, cap, ctypes.byref(n)))
    m = int(n.value)
    if relayout:
        return np.array([(p.src_block, p.src_token, p.dst_block, p.dst_token, p.num_tokens)
                         for p in pieces[:m]], dtype=np.int64).reshape(m, 5)
    return np.array([(s.src_offset, s.dst_offset, s.bytes) for s in spans[:m]], dtype=np.int64).reshape(m, 3)


def kvd_copy_plain(dst_ptr: int, src_ptr: int, nbytes: int, stream: int = 0) -> None:
    _check(lib().kvd_copy_plain(dst_ptr, src_ptr, nbytes, stream))


PROBE_MODES = {"copy": 0, "read": 1, "write": 2, "copy_persistent": 3, "read_persistent": 4, "write_persistent": 5}


def kvd_stream_probe(dst_ptr: int, src_ptr: int, nbytes: int, mode, stream: int = 0) -> None:
    _check(lib().kvd_stream_probe(dst_ptr, src_ptr, nbytes, PROBE_MODES.get(mode, mode), stream))


def kvd_free(handle: Optional[int]) -> None:
    if handle:
        lib().kvd_free(handle)


# ---------------------------------------------------------------- handle owners

class Pool:
    """Registered tensor metadata of one paged pool whose memory the caller owns."""

    def __init__(self, base: int, geometry, stride_layer=None, stride_kv=None, stride_block=None):
        g = geometry
        self.geometry = g
        self.handle = kvd_pool_create(
            base, g.num_layers, g.num_blocks, g.block_tokens, g.num_kv_heads, g.head_dim, g.elem_bytes,
            g.layout, g.stride_layer if stride_layer is None else stride_layer,
            g.stride_kv if stride_kv is None else stride_kv,
            g.stride_block if stride_block is None else stride_block)

    def close(self):
        kvd_free(self.handle)
        self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Plan:
    """Transaction queue from a source pool to a destination pool."""

    def __init__(self, src: Pool, dst: Pool, max_requests: int, max_total_blocks: int, flags: int = 0):
        self.handle = kvd_plan_create(src.handle, dst.handle, max_requests, max_total_blocks, flags)

    def build_descriptors(self, src_table, dst_table, seq_len, layer_begin, layer_end, stream=0):
        kvd_build_descriptors(self.handle, src_table, dst_table, seq_len, layer_begin, layer_end, stream)

    def build_descriptors_batch(self, src_tables, dst_tables, seq_lens, layer_begin, layer_end, stream=0):
        kvd_build_descriptors_batch(self.handle, src_tables, dst_tables, seq_lens, layer_begin, layer_end, stream)

    def pull(self, stream=0):
        kvd_pull(self.handle, stream)

    def pull_notify(self, words_ptr, value, stream=0):
        kvd_pull_notify(self.handle, words_ptr, value, stream)

    def set_completion_granularity(self, min_tokens):
        kvd_plan_set_completion_granularity(self.handle, min_tokens)

    def pull_layers(self, layer_begin, layer_end, stream=0):
        kvd_pull_layers(self.handle, layer_begin, layer_end, stream)

    def pull_blockwise_memcpy(self, stream=0):
        kvd_pull_blockwise_memcpy(self.handle, stream)

    def pull_staged(self, send_buffer, recv_buffer, buffer_bytes, stream=0):
        kvd_pull_staged(self.handle, send_buffer, recv_buffer, buffer_bytes, stream)

    def reset(self):
        kvd_plan_reset(self.handle)

    def stats(self, stream=0) -> dict:
        return kvd_plan_stats(self.handle, stream)

    def descriptors(self, stream=0) -> np.ndarray:
        return kvd_plan_get_descriptors(self.handle, stream)

    def close(self):
        kvd_free(self.handle)
        self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
