"""Device-side plumbing for the benchmark and the GPU tests: pools as torch byte tensors (torch is
the allocator and the stream provider, nothing more) and a small driver that runs a workload
through the C ABI.  No arithmetic of the transfer happens here."""
from __future__ import annotations

import numpy as np
import torch

from . import kvd
from . import workloads as wl

DEV = "cuda:0"


def device_pool_from_host(host_bytes: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(host_bytes).to(DEV)


def device_sentinel_pool(g: wl.PoolGeometry) -> torch.Tensor:
    t = torch.empty(g.total_bytes, dtype=torch.uint8, device=DEV)
    t.view(torch.int16).fill_(wl.SENTINEL16)
    return t


def device_random_pool(g: wl.PoolGeometry, dtype: str, seed: int) -> torch.Tensor:
    """N(0,1) in fp16 / bf16 everywhere, generated on the device layer by layer."""
    assert g.elem_bytes == 2
    t = torch.empty(g.total_bytes, dtype=torch.uint8, device=DEV)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(seed)
    td = torch.float16 if dtype == "fp16" else torch.bfloat16
    v = t.view(td).view(g.num_layers, -1)  # filled in num_layers equal parts
    for layer in range(g.num_layers):
        v[layer].normal_(generator=gen)
    return t


class GpuTransfer:
    """Pools + plan for one workload on the GPU."""

    def __init__(self, w: wl.Workload, src: torch.Tensor, dst: torch.Tensor, flags: int = 0,
                 stream: torch.cuda.Stream | None = None):
        self.w, self.src, self.dst = w, src, dst
        self.stream = stream or torch.cuda.Stream(device=DEV)
        self.src_pool = kvd.Pool(src.data_ptr(), w.src)
        self.dst_pool = kvd.Pool(dst.data_ptr(), w.dst)
        max_blocks = sum(max(len(r.src_table), len(r.dst_table)) for r in w.requests) + 1
        self.plan = kvd.Plan(self.src_pool, self.dst_pool, max(1, len(w.requests)), max_blocks, flags)
        self.after_torch()

    def after_torch(self):
        """Order this object's stream after what torch has queued on its current stream (pool fills)."""
        self.stream.wait_stream(torch.cuda.current_stream())

    def build(self, batch: bool = False):
        """Append every request of the workload: one call each, or one batched call."""
        w = self.w
        if batch:
            self.plan.build_descriptors_batch([r.src_table for r in w.requests], [r.dst_table for r in w.requests],
                                              [r.seq_len for r in w.requests], w.layer_begin, w.layer_end,
                                              self.stream.cuda_stream)
            return
        for r in w.requests:
            self.plan.build_descriptors(r.src_table, r.dst_table, r.seq_len, w.layer_begin, w.layer_end,
                                        self.stream.cuda_stream)

    def pull(self):
        self.plan.pull(self.stream.cuda_stream)

    def run(self, batch: bool = False):
        self.build(batch)
        self.pull()
        self.stream.synchronize()
        return self

    def close(self):
        self.plan.close()
        self.src_pool.close()
        self.dst_pool.close()
