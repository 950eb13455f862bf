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


def compare_layer_with_oracle(w: wl.Workload, src: torch.Tensor, dst: torch.Tensor, layer: int):
    """Oracle for one layer of a large workload: copies that layer's slabs to the host."""
    gs, gd = w.src, w.dst
    sb, db = gs.stride_layer * gs.elem_bytes, gd.stride_layer * gd.elem_bytes
    src_host = src[layer * sb:(layer + 1) * sb].cpu().numpy()
    got = dst[layer * db:(layer + 1) * db].cpu().numpy()
    want = np.full(db // 2, wl.SENTINEL16, dtype=np.uint16).view(np.uint8)
    if w.layer_begin <= layer < w.layer_end:
        s = tl.oracle_tensors(gs, src_host, first_layer=layer, num_layers=1)
        d = tl.oracle_tensors(gd, want, first_layer=layer, num_layers=1)
        from oracle import kvd_oracle as orc
        for r in w.requests:
            orc.pull(s, d, layer, layer + 1, r.src_table, r.dst_table, r.seq_len)
    assert_bytes_equal(got, want, f"{w.name} layer {layer}")
