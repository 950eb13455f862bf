"""ctypes front end of the CPU oracle (``kvd_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by the tests, by the smoke check and by the
benchmark's CPU-baseline leg.  Nothing of the GPU library is imported here and
the GPU library never imports this module.

The tensor description mirrors the paper's metadata (section 4.1): Address,
Dims, Shape, Stride, with one tensor per model layer.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "kvd_oracle.c")
_LIB = os.path.join(_HERE, "libkvd_oracle.so")

# axis roles, section 4.1 item (ii)
B, KV, L, H, D = 0, 1, 2, 3, 4
ROLE_NAMES = {B: "B", KV: "KV", L: "L", H: "H", D: "D"}


class _Tensor(ctypes.Structure):
    _fields_ = [
        ("address", ctypes.c_void_p),
        ("dims", ctypes.c_int32 * 5),
        ("shape", ctypes.c_int64 * 5),
        ("stride", ctypes.c_int64 * 5),
        ("elem_bytes", ctypes.c_int64),
    ]


class _Txn(ctypes.Structure):
    _fields_ = [("remote", ctypes.c_int64), ("local", ctypes.c_int64), ("size", ctypes.c_int64)]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, no tuning flags)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-Wall", "-Wextra", "-shared", "-fPIC", "-o", _LIB, _SRC]
        )
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.kvdo_offset_bytes.restype = ctypes.c_int64
        _lib.kvdo_offset_bytes.argtypes = [ctypes.POINTER(_Tensor), ctypes.POINTER(ctypes.c_int64)]
        _lib.kvdo_block_span_bytes.restype = ctypes.c_int64
        _lib.kvdo_block_span_bytes.argtypes = [ctypes.POINTER(_Tensor)]
        _lib.kvdo_transfer_bytes.restype = ctypes.c_int64
        _lib.kvdo_transfer_bytes.argtypes = [ctypes.c_int64] * 5
        _lib.kvdo_pull.restype = ctypes.c_int
        _lib.kvdo_pull.argtypes = [
            ctypes.POINTER(_Tensor), ctypes.POINTER(_Tensor), ctypes.c_int64, ctypes.c_int64,
            ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32), ctypes.c_int64,
        ]
        _lib.kvdo_request_transactions.restype = ctypes.c_int64
        _lib.kvdo_request_transactions.argtypes = [
            ctypes.POINTER(_Tensor), ctypes.POINTER(_Tensor), ctypes.c_int64,
            ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32), ctypes.c_int64,
            ctypes.POINTER(_Txn), ctypes.c_int64,
        ]
        _lib.kvdo_coalesce.restype = ctypes.c_int64
        _lib.kvdo_coalesce.argtypes = [ctypes.POINTER(_Txn), ctypes.c_int64, ctypes.POINTER(_Txn)]
    return _lib


class Tensor:
    """One layer's KV cache tensor: Address / Dims / Shape / Stride (section 4.1).

    ``buffer`` is a numpy uint8 array that owns the memory; ``byte_offset`` is
    where this tensor starts inside it.  ``dims`` lists the role of each axis in
    axis order; ``shape`` and ``stride`` (elements) use that same order.
    """

    def __init__(self, buffer: np.ndarray | None, byte_offset: int, dims: Sequence[int],
                 shape: Sequence[int], stride: Sequence[int], elem_bytes: int):
        assert sorted(dims) == [0, 1, 2, 3, 4]
        self.buffer = buffer
        self.byte_offset = int(byte_offset)
        self.dims = [int(x) for x in dims]
        self.shape = [int(x) for x in shape]
        self.stride = [int(x) for x in stride]
        self.elem_bytes = int(elem_bytes)

    def c(self) -> _Tensor:
        t = _Tensor()
        if self.buffer is not None:
            assert self.buffer.dtype == np.uint8 and self.buffer.flags["C_CONTIGUOUS"]
            t.address = self.buffer.ctypes.data + self.byte_offset
        else:
            t.address = None
        t.dims = (ctypes.c_int32 * 5)(*self.dims)
        t.shape = (ctypes.c_int64 * 5)(*self.shape)
        t.stride = (ctypes.c_int64 * 5)(*self.stride)
        t.elem_bytes = self.elem_bytes
        return t


def offset_bytes(t: Tensor, index: Sequence[int]) -> int:
    """Byte offset of cache[index] (index in the tensor's axis order)."""
    ct = t.c()
    idx = (ctypes.c_int64 * 5)(*[int(i) for i in index])
    return int(lib().kvdo_offset_bytes(ctypes.byref(ct), idx))


def block_span_bytes(t: Tensor) -> int:
    ct = t.c()
    return int(lib().kvdo_block_span_bytes(ctypes.byref(ct)))


def transfer_bytes(tokens: int, layers: int, kv_heads: int, head_dim: int, elem_bytes: int) -> int:
    return int(lib().kvdo_transfer_bytes(tokens, layers, kv_heads, head_dim, elem_bytes))


def _table(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def pull(src: Sequence[Tensor], dst: Sequence[Tensor], layer_begin: int, layer_end: int,
         src_table, dst_table, seq_len: int) -> None:
    """Copy one request (all its tokens) from the source pool to the destination pool."""
    assert len(src) == len(dst) and 0 <= layer_begin <= layer_end <= len(src)
    cs = (_Tensor * len(src))(*[t.c() for t in src])
    cd = (_Tensor * len(dst))(*[t.c() for t in dst])
    st, dt = _table(src_table), _table(dst_table)
    ls = src[0].shape[src[0].dims.index(L)]
    ld = dst[0].shape[dst[0].dims.index(L)]
    assert len(st) * ls >= seq_len and len(dt) * ld >= seq_len
    rc = lib().kvdo_pull(cs, cd, layer_begin, layer_end,
                         st.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                         dt.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), seq_len)
    if rc != 0:
        raise ValueError("source and destination tensors describe different elements")


def request_transactions(s: Tensor, d: Tensor, kv: int, src_table, dst_table, seq_len: int) -> np.ndarray:
    """Read transactions (remote offset, local offset, size) of one request for one tensor:
    kv = 0 / 1 for its K / V half, kv = -1 for both in Transfer() order (K then V of every block)."""
    st, dt = _table(src_table), _table(dst_table)
    ls = s.shape[s.dims.index(L)]
    ld = d.shape[d.dims.index(L)]
    hh = s.shape[s.dims.index(H)]
    cap = 2 * (len(st) + len(dt) + 2) * max(1, hh) * max(ls, ld) + 8
    out = (_Txn * cap)()
    cs, cd = s.c(), d.c()
    n = lib().kvdo_request_transactions(
        ctypes.byref(cs), ctypes.byref(cd), kv,
        st.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
        dt.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), seq_len, out, cap)
    if n < 0:
        raise RuntimeError("transaction buffer too small")
    return np.array([(out[i].remote, out[i].local, out[i].size) for i in range(n)],
                    dtype=np.int64).reshape(n, 3)


def coalesce(txns: np.ndarray) -> np.ndarray:
    """Merge queued read transactions that continue each other on both sides (section 4.2)."""
    txns = np.asarray(txns, dtype=np.int64).reshape(-1, 3)
    n = len(txns)
    arr = (_Txn * max(n, 1))()
    for i in range(n):
        arr[i].remote, arr[i].local, arr[i].size = (int(x) for x in txns[i])
    out = (_Txn * max(n, 1))()
    m = lib().kvdo_coalesce(arr, n, out)
    return np.array([(out[i].remote, out[i].local, out[i].size) for i in range(m)],
                    dtype=np.int64).reshape(m, 3)
