"""GPU-side test plumbing: the device pools and workload driver of the package, plus the slab-wise
comparison of a device pool with the oracle."""
from __future__ import annotations

import numpy as np
import torch

import kvd_testlib as tl
from paper_2501_14743_amd import workloads as wl
from paper_2501_14743_amd.device import (DEV, GpuTransfer, device_pool_from_host, device_random_pool,  # noqa: F401
                                         device_sentinel_pool)


def oracle_expected(w: wl.Workload, src_host: np.ndarray) -> np.ndarray:
    dst = wl.host_pool_sentinel(w.dst)
    tl.oracle_pull_workload(w, src_host, dst)
    return dst


def assert_bytes_equal(got: np.ndarray, want: np.ndarray, what: str = ""):
    if not np.array_equal(got, want):
        bad = np.nonzero(got != want)[0]
        raise AssertionError(f"{what}: {bad.size} bytes differ, first at byte {int(bad[0])} "
                             f"(got {int(got[bad[0]])}, want {int(want[bad[0]])})")


def run_and_compare(w: wl.Workload, src_host: np.ndarray, flags: int = 0):
    """Whole-pool, element-by-element comparison of the GPU result with the oracle."""
    src = device_pool_from_host(src_host)
    dst = device_sentinel_pool(w.dst)
    x = GpuTransfer(w, src, dst, flags).run()
    want = oracle_expected(w, src_host)
    assert_bytes_equal(dst.cpu().numpy(), want, w.name)
    assert_bytes_equal(src.cpu().numpy(), src_host, w.name + " (source changed)")
    return x


def _layer_slabs(g: wl.PoolGeometry, pool: torch.Tensor, layer: int) -> np.ndarray:
    """One layer of a device pool on the host, as the bytes of a one-layer pool in [kv][block] order
    (a plain slice for layer-major pools; gathered through torch's strided view otherwise)."""
    if not g.block_major and not g.kv_adjacent:
        nbytes = g.stride_layer * g.elem_bytes
        return pool[layer * nbytes:(layer + 1) * nbytes].cpu().numpy()
    tile = g.tile_elems * g.elem_bytes
    if g.block_major:
        v = pool.view(g.num_blocks, g.num_layers, 2, tile)[:, layer]   # [block][kv][tile]
    else:
        v = pool.view(g.num_layers, g.num_blocks, 2, tile)[layer]      # [block][kv][tile]
    return v.permute(1, 0, 2).contiguous().view(-1).cpu().numpy()


def compare_layer_with_oracle(w: wl.Workload, src: torch.Tensor, dst: torch.Tensor, layer: int):
    """Oracle for one layer of a large workload: copies that layer's slabs to the host and hands
    them to the oracle as a one-layer pool in [kv][block] order, addressed with that pool's own strides."""
    g1s, g1d = (wl.PoolGeometry(1, g.num_blocks, g.block_tokens, g.num_kv_heads, g.head_dim, g.elem_bytes, g.layout)
                for g in (w.src, w.dst))
    src_host = _layer_slabs(w.src, src, layer)
    got = _layer_slabs(w.dst, dst, layer)
    want = np.full(got.size // 2, wl.SENTINEL16, dtype=np.uint16).view(np.uint8)
    if w.layer_begin <= layer < w.layer_end:
        s = tl.oracle_tensors(g1s, src_host)
        d = tl.oracle_tensors(g1d, want)
        from oracle import kvd_oracle as orc
        for r in w.requests:
            orc.pull(s, d, 0, 1, r.src_table, r.dst_table, r.seq_len)
    assert_bytes_equal(got, want, f"{w.name} layer {layer}")
