"""Test-side glue: turns a workload's pool geometry into the oracle's tensor metadata,
runs the oracle over a workload, and holds the tiny element-by-element brute force that
pins the oracle."""
from __future__ import annotations

import numpy as np

from oracle import kvd_oracle as orc
from paper_2501_14743_amd import workloads as wl


def oracle_tensors(g: wl.PoolGeometry, buffer: np.ndarray | None, first_layer: int = 0,
                   num_layers: int | None = None) -> list:
    """One oracle tensor per layer.  ``buffer`` holds layers [first_layer, first_layer+num_layers)
    of the pool back to back (or the whole pool by default); tensors for layers outside that
    window get no address and must not be used."""
    if num_layers is None:
        num_layers = g.num_layers - first_layer
    stride_layer, stride_kv, stride_block = outer_strides(g)
    if g.layout == wl.BHTD:
        dims = [orc.KV, orc.B, orc.H, orc.L, orc.D]
        shape = [2, g.num_blocks, g.num_kv_heads, g.block_tokens, g.head_dim]
        stride = [stride_kv, stride_block, g.block_tokens * g.head_dim, g.head_dim, 1]
    else:
        dims = [orc.KV, orc.B, orc.L, orc.H, orc.D]
        shape = [2, g.num_blocks, g.block_tokens, g.num_kv_heads, g.head_dim]
        stride = [stride_kv, stride_block, g.num_kv_heads * g.head_dim, g.head_dim, 1]
    out = []
    for layer in range(g.num_layers):
        inside = first_layer <= layer < first_layer + num_layers
        out.append(orc.Tensor(buffer if inside else None,
                              (layer - first_layer) * stride_layer * g.elem_bytes if inside else 0,
                              dims, shape, stride, g.elem_bytes))
    return out


def outer_strides(g: wl.PoolGeometry) -> tuple:
    """(layer, K/V, block) strides in elements of the dense allocation the geometry names, worked out here
    from the order of its axes - outermost first, each stride the product of the extents inside it - and not
    taken from the geometry's own stride properties, which are what the library under test is given."""
    extent = {"layer": g.num_layers, "kv": 2, "block": g.num_blocks}
    if g.block_major:
        order = ["block", "layer", "kv"]
    elif g.kv_adjacent:
        order = ["layer", "block", "kv"]
    else:
        order = ["layer", "kv", "block"]
    stride, inside = {}, g.block_tokens * g.num_kv_heads * g.head_dim
    for axis in reversed(order):
        stride[axis] = inside
        inside *= extent[axis]
    return stride["layer"], stride["kv"], stride["block"]


def oracle_pull_workload(w: wl.Workload, src_bytes: np.ndarray, dst_bytes: np.ndarray,
                         layer_begin: int | None = None, layer_end: int | None = None) -> None:
    """Run the oracle for every request of the workload (whole pools resident on the host)."""
    lb = w.layer_begin if layer_begin is None else layer_begin
    le = w.layer_end if layer_end is None else layer_end
    s = oracle_tensors(w.src, src_bytes)
    d = oracle_tensors(w.dst, dst_bytes)
    for r in w.requests:
        orc.pull(s, d, lb, le, r.src_table, r.dst_table, r.seq_len)


def oracle_plan_descriptors(w: wl.Workload, layer: int, kv: int) -> np.ndarray:
    """Coalesced read transactions of the whole batch for one (layer, K/V) tensor, or with
    kv = -1 for the layer's whole tensor (K then V of every block):
    every request's transactions queued in order, then merged (section 4.2)."""
    s = oracle_tensors(w.src, None)[layer]
    d = oracle_tensors(w.dst, None)[layer]
    q = [orc.request_transactions(s, d, kv, r.src_table, r.dst_table, r.seq_len)
         for r in w.requests]
    q = np.concatenate(q) if q else np.zeros((0, 3), np.int64)
    merged = orc.coalesce(q)
    # the tensors carry no address here, so offsets are relative to the layer's tensor;
    # make them relative to the pool instead
    merged[:, 0] += layer * outer_strides(w.src)[0] * w.src.elem_bytes
    merged[:, 1] += layer * outer_strides(w.dst)[0] * w.dst.elem_bytes
    return merged


def oracle_plan_descriptors_block_major(w: wl.Workload) -> np.ndarray:
    """Coalesced read transactions of the whole batch when the layer tensors are queued block by
    block: for every piece of a request (tokens that share one block on both sides), the
    transactions of layer_begin, layer_begin+1, ... in turn.  In pools that keep all layers of a
    block together that is the order in which consecutive ranges continue each other, so section
    4.2 merges a block's layers.  Offsets are relative to the pool.

    A piece's transactions in one layer's tensor are what the oracle's list for that tensor gains
    when the request is cut one piece later: the list of the shorter request is a prefix of the
    longer one's (asserted).  To keep this linear, the cuts are taken inside one block of the side
    with the larger blocks at a time, on tables that start at that block."""
    ls, ld = w.src.block_tokens, w.dst.block_tokens
    tmin, tmax = min(ls, ld), max(ls, ld)
    s_all, d_all = oracle_tensors(w.src, None), oracle_tensors(w.dst, None)
    layers = range(w.layer_begin, w.layer_end)
    queue = []
    for r in w.requests:
        for big in range(0, r.seq_len, tmax):
            st, dt = r.src_table[big // ls:], r.dst_table[big // ld:]
            have = {layer: np.zeros((0, 3), np.int64) for layer in layers}
            for end in range(tmin, tmax + tmin, tmin):
                end = min(end, r.seq_len - big)
                for layer in layers:
                    t = orc.request_transactions(s_all[layer], d_all[layer], -1, st, dt, end)
                    t[:, 0] += layer * outer_strides(w.src)[0] * w.src.elem_bytes
                    t[:, 1] += layer * outer_strides(w.dst)[0] * w.dst.elem_bytes
                    n = len(have[layer])
                    assert np.array_equal(t[:n], have[layer]) and len(t) > n
                    queue.append(t[n:])
                    have[layer] = t
                if end == r.seq_len - big:
                    break
    q = np.concatenate(queue) if queue else np.zeros((0, 3), np.int64)
    return orc.coalesce(q)


# ------------------------------------------------------------------ brute force (tiny inputs)

def _inner_index(layout: str, tb: int, hk: int, tok: int, head: int) -> int:
    if layout == wl.BHTD:
        return head * tb + tok
    return tok * hk + head


def brute_force_pull(w: wl.Workload, src_elems: np.ndarray, dst_elems: np.ndarray):
    """Element-by-element definition in pure Python on arrays of whole elements
    (dtype of elem_bytes width).  Returns the per-element write count of the destination."""
    gs, gd = w.src, w.dst
    count = np.zeros(dst_elems.shape, dtype=np.int32)
    for r in w.requests:
        for layer in range(w.layer_begin, w.layer_end):
            for kv in range(2):
                for t in range(r.seq_len):
                    sb = int(r.src_table[t // gs.block_tokens])
                    db = int(r.dst_table[t // gd.block_tokens])
                    for h in range(gs.num_kv_heads):
                        si = (layer * gs.stride_layer + kv * gs.stride_kv + sb * gs.stride_block
                              + _inner_index(gs.layout, gs.block_tokens, gs.num_kv_heads,
                                             t % gs.block_tokens, h) * gs.head_dim)
                        di = (layer * gd.stride_layer + kv * gd.stride_kv + db * gd.stride_block
                              + _inner_index(gd.layout, gd.block_tokens, gd.num_kv_heads,
                                             t % gd.block_tokens, h) * gd.head_dim)
                        for x in range(gs.head_dim):
                            dst_elems[di + x] = src_elems[si + x]
                            count[di + x] += 1
    return count


def read_golden(path: str) -> dict:
    out = {}
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, v = line.split("=", 1)
            out[k.strip()] = v.strip()
    return out
