"""Seeded synthetic inputs for the paged KV-cache transfer.

This module only *describes and generates inputs*: pool geometries, block
tables, prompt lengths and pool contents.  It holds none of the transfer's
arithmetic (no address translation, no coalescing, no copying) and imports
neither the GPU library nor the CPU oracle, so both can be fed from it.

The shapes follow the regime of the paper's workloads: 16-token blocks and
4 KB - 32 KB pieces per block (section 3), 8K - 64K token prompts (section
5.2.2), 8 KV heads with 128-wide heads (section 5.1), and one GPU's
tensor-parallel share of a 70B model (section 3).  Values are N(0,1) because
the transfer never interprets them.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List

import numpy as np

SENTINEL16 = 0x7FA5  # NaN in fp16 and in bf16: N(0,1) data can never equal it

BHTD = "BHTD"  # inside a block: [head][token][dim]
BTHD = "BTHD"  # inside a block: [token][head][dim]


@dataclass(frozen=True)
class PoolGeometry:
    """One paged pool, stored as a single dense allocation [layer][kv][block][inner],
    [layer][block][kv][inner] when kv_adjacent (K and V of a block next to each other), or
    [block][layer][kv][inner] when block_major (everything a block holds in one piece)."""
    num_layers: int
    num_blocks: int
    block_tokens: int
    num_kv_heads: int
    head_dim: int
    elem_bytes: int
    layout: str = BHTD
    kv_adjacent: bool = False
    block_major: bool = False

    @property
    def tile_elems(self) -> int:
        return self.block_tokens * self.num_kv_heads * self.head_dim

    @property
    def stride_block(self) -> int:
        if self.block_major:
            return 2 * self.num_layers * self.tile_elems
        return (2 if self.kv_adjacent else 1) * self.tile_elems

    @property
    def stride_kv(self) -> int:
        return self.tile_elems if (self.kv_adjacent or self.block_major) else self.num_blocks * self.tile_elems

    @property
    def stride_layer(self) -> int:
        return 2 * self.tile_elems if self.block_major else 2 * self.num_blocks * self.tile_elems

    @property
    def total_elems(self) -> int:
        return 2 * self.num_layers * self.num_blocks * self.tile_elems

    @property
    def total_bytes(self) -> int:
        return self.total_elems * self.elem_bytes


@dataclass
class Request:
    seq_len: int
    src_table: np.ndarray  # int32 physical block ids in the source pool
    dst_table: np.ndarray  # int32 physical block ids in the destination pool


@dataclass
class Workload:
    name: str
    src: PoolGeometry
    dst: PoolGeometry
    requests: List[Request]
    dtype: str  # "fp16" or "bf16": how the N(0,1) values are encoded
    seed: int
    layer_begin: int = 0
    layer_end: int = -1
    notes: str = ""
    extra: dict = field(default_factory=dict)

    def __post_init__(self):
        if self.layer_end < 0:
            self.layer_end = self.src.num_layers

    @property
    def total_tokens(self) -> int:
        return sum(r.seq_len for r in self.requests)


# ----------------------------------------------------------------- allocation recipes

def blocks_for(tokens: int, block_tokens: int) -> int:
    return -(-tokens // block_tokens)


def permutation_table(rng: np.random.Generator, pool_blocks: int, n: int) -> np.ndarray:
    """First n entries of a random permutation of the pool's block ids."""
    return rng.permutation(pool_blocks)[:n].astype(np.int32)


def fragmented_allocation(rng: np.random.Generator, free: np.ndarray, n: int,
                          max_run: int = 8) -> np.ndarray:
    """Allocate n blocks as runs of 1..max_run physically consecutive free ids.

    Each run's length is uniform in 1..max_run and its start is uniform over
    the positions where that many consecutive ids are still free.  ``free`` is
    updated in place, so later requests see the fragmentation left by earlier
    ones.
    """
    out: list[int] = []
    while len(out) < n:
        r = min(int(rng.integers(1, max_run + 1)), n - len(out))
        while True:
            c = np.concatenate(([0], np.cumsum(free, dtype=np.int64)))
            ok = np.nonzero(c[r:] - c[:-r] == r)[0]
            if ok.size:
                break
            if r == 1:
                raise RuntimeError("pool exhausted")
            r -= 1
        start = int(ok[int(rng.integers(ok.size))])
        free[start:start + r] = False
        out.extend(range(start, start + r))
    return np.asarray(out, dtype=np.int32)


def scattered_table(rng: np.random.Generator, pool_blocks: int, n: int) -> np.ndarray:
    """n distinct block ids with no two consecutive entries physically adjacent
    (entry i+1 is never entry i plus one): worst-case fragmentation."""
    tbl = rng.permutation(pool_blocks)[:n].astype(np.int64)
    for _ in range(1000):
        bad = np.nonzero(tbl[1:] == tbl[:-1] + 1)[0] + 1
        if bad.size == 0:
            return tbl.astype(np.int32)
        for i in bad:
            j = int(rng.integers(n))
            tbl[i], tbl[j] = tbl[j], tbl[i]
    raise RuntimeError("could not scatter the table")


def fixed_run_table(rng: np.random.Generator, pool_blocks: int, n: int, run: int) -> np.ndarray:
    """n block ids as runs of exactly ``run`` physically consecutive ids (the last one may be
    shorter); runs sit at random places and no run continues the one before it."""
    slots = rng.permutation(pool_blocks // (2 * run))  # slot s = ids [2*run*s, 2*run*s + run)
    runs = -(-n // run)
    if runs > slots.size:
        raise ValueError("pool too small for that many separate runs")
    ids = np.concatenate([np.arange(2 * run * s, 2 * run * s + run) for s in slots[:runs]])
    return ids[:n].astype(np.int32)


def lognormal_lengths(rng: np.random.Generator, count: int, median: float = 1024.0,
                      sigma: float = 1.0, lo: int = 16, hi: int = 16384) -> np.ndarray:
    x = np.exp(rng.normal(np.log(median), sigma, size=count))
    return np.clip(np.rint(x), lo, hi).astype(np.int64)


# ----------------------------------------------------------------- pool contents

def normal_bits(rng: np.random.Generator, n: int, dtype: str) -> np.ndarray:
    """n samples of N(0,1) encoded as 16-bit patterns (fp16 or bf16, round to nearest even)."""
    x = rng.standard_normal(n, dtype=np.float32)
    if dtype == "fp16":
        return x.astype(np.float16).view(np.uint16)
    if dtype == "bf16":
        u = x.view(np.uint32)
        return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)
    raise ValueError(dtype)


def host_pool_values(g: PoolGeometry, dtype: str, seed: int) -> np.ndarray:
    """Whole source pool as raw bytes (uint8), N(0,1) everywhere."""
    assert g.elem_bytes == 2
    rng = np.random.default_rng(seed)
    return normal_bits(rng, g.total_elems, dtype).view(np.uint8)


def host_pool_sentinel(g: PoolGeometry) -> np.ndarray:
    """Whole destination pool as raw bytes, every 16-bit word the sentinel."""
    assert g.total_bytes % 2 == 0
    return np.full(g.total_bytes // 2, SENTINEL16, dtype=np.uint16).view(np.uint8)


# ----------------------------------------------------------------- the five configurations

def _rngs(seed: int):
    return np.random.default_rng(seed), np.random.default_rng(seed + 50)


def config1() -> Workload:
    """Toy: 2 layers, 4 KV heads, head_dim 64, fp16, 128 tokens, 16-token blocks, 64-block pools."""
    seed = 1001
    rs, rd = _rngs(seed)
    g = PoolGeometry(2, 64, 16, 4, 64, 2, BHTD)
    n = blocks_for(128, 16)
    req = Request(128, permutation_table(rs, 64, n), permutation_table(rd, 64, n))
    return Workload("cfg1-toy", g, g, [req], "fp16", seed)


def config2(num_layers: int = 32, pool_blocks: int = 16384, tokens: int = 8192) -> Workload:
    """Llama-3-8B-shaped single request: 8 KV heads, head_dim 128, bf16, 16-token blocks,
    fragmented allocation in runs of 1-8 consecutive blocks on both sides."""
    seed = 1002
    rs, rd = _rngs(seed)
    g = PoolGeometry(num_layers, pool_blocks, 16, 8, 128, 2, BHTD)
    n = blocks_for(tokens, 16)
    req = Request(tokens,
                  fragmented_allocation(rs, np.ones(pool_blocks, bool), n),
                  fragmented_allocation(rd, np.ones(pool_blocks, bool), n))
    return Workload("cfg2-llama3-8b-8k", g, g, [req], "bf16", seed)


def config3(num_layers: int = 32, num_requests: int = 64, median: float = 1024.0,
            hi: int = 16384) -> Workload:
    """Batch of concurrent requests with lognormal prompt lengths in shared fragmented pools
    sized 1.25x the total demand."""
    seed = 1003
    rs, rd = _rngs(seed)
    lens = lognormal_lengths(np.random.default_rng(seed + 7), num_requests, median, 1.0, 16, hi)
    demand = int(sum(blocks_for(int(t), 16) for t in lens))
    pool_blocks = int(np.ceil(1.25 * demand))
    g = PoolGeometry(num_layers, pool_blocks, 16, 8, 128, 2, BHTD)
    free_s, free_d = np.ones(pool_blocks, bool), np.ones(pool_blocks, bool)
    reqs = []
    for t in lens:
        n = blocks_for(int(t), 16)
        reqs.append(Request(int(t), fragmented_allocation(rs, free_s, n),
                            fragmented_allocation(rd, free_d, n)))
    return Workload("cfg3-batch", g, g, reqs, "bf16", seed,
                    extra={"lengths": [int(t) for t in lens]})


def config4(num_layers: int = 80, pool_blocks: int = 8192, tokens: int = 32768) -> Workload:
    """Llama-3-70B, one GPU's tensor-parallel share: 1 KV head, head_dim 128, bf16,
    every block alone (no two consecutive entries adjacent on either side)."""
    seed = 1004
    rs, rd = _rngs(seed)
    g = PoolGeometry(num_layers, pool_blocks, 16, 1, 128, 2, BHTD)
    n = blocks_for(tokens, 16)
    req = Request(tokens, scattered_table(rs, pool_blocks, n), scattered_table(rd, pool_blocks, n))
    return Workload("cfg4-llama3-70b-tp8", g, g, [req], "bf16", seed)


def config5(num_layers: int = 32, src_pool_blocks: int = 2048, tokens: int = 4096) -> Workload:
    """Re-layout: source 16-token blocks [head][token][dim], destination 32-token blocks
    [token][head][dim]; random-permutation tables on both sides."""
    seed = 1005
    rs, rd = _rngs(seed)
    gs = PoolGeometry(num_layers, src_pool_blocks, 16, 8, 128, 2, BHTD)
    gd = PoolGeometry(num_layers, src_pool_blocks // 2, 32, 8, 128, 2, BTHD)
    req = Request(tokens,
                  permutation_table(rs, gs.num_blocks, blocks_for(tokens, 16)),
                  permutation_table(rd, gd.num_blocks, blocks_for(tokens, 32)))
    return Workload("cfg5-relayout", gs, gd, [req], "bf16", seed)


CONFIGS = {1: config1, 2: config2, 3: config3, 4: config4, 5: config5}
