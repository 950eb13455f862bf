"""Pins the CPU oracle to things other than itself: the values the paper prints for its
worked examples (tests/golden/paper_worked_example.txt), closed forms, an independent
element-by-element brute force, numpy's own reshape addressing, and invariants of a copy."""
import os

import dataclasses

import numpy as np
import pytest

import kvd_testlib as tl
from oracle import kvd_oracle as orc
from paper_2501_14743_amd import workloads as wl

GOLD = tl.read_golden(os.path.join(os.path.dirname(__file__), "golden", "paper_worked_example.txt"))
ROLE = {"B": orc.B, "KV": orc.KV, "L": orc.L, "H": orc.H, "D": orc.D}


def paper_tensor():
    dims = [ROLE[x] for x in GOLD["dims"].split()]
    shape = [int(x) for x in GOLD["shape"].split()]
    stride = [int(x) for x in GOLD["stride"].split()]
    return orc.Tensor(None, 0, dims, shape, stride, int(GOLD["elem_bytes"]))


# ---------------------------------------------------------------- section 4.1 worked example

def test_block8_offsets_match_paper():
    t = paper_tensor()
    assert orc.offset_bytes(t, [8, 0, 0, 0, 0]) == int(GOLD["block8_K_offset"]) == 65536
    assert orc.offset_bytes(t, [8, 1, 0, 0, 0]) == int(GOLD["block8_V_offset"]) == 147456
    assert orc.offset_bytes(t, [0, 0, 0, 0, 0]) == int(GOLD["block0_K_offset"])
    assert orc.offset_bytes(t, [1, 0, 0, 0, 0]) == int(GOLD["block1_K_offset"])


def test_offset_uses_every_axis():
    t = paper_tensor()
    # one step along each axis moves by that axis' stride times the element size
    for axis, stride in enumerate(t.stride):
        idx = [0] * 5
        idx[axis] = 1
        assert orc.offset_bytes(t, idx) == stride * 2
    assert orc.offset_bytes(t, [3, 1, 5, 1, 7]) == (3 * 4096 + 40960 + 5 * 256 + 128 + 7) * 2


def test_span_size_matches_paper():
    assert orc.block_span_bytes(paper_tensor()) == int(GOLD["block_span_bytes"]) == 8192


def test_span_size_follows_largest_stride_axis():
    # heads outermost inside a block: H has the largest stride among L, H, D
    t = orc.Tensor(None, 0, [orc.KV, orc.B, orc.H, orc.L, orc.D], [2, 10, 4, 16, 64],
                   [10 * 4096, 4096, 16 * 64, 64, 1], 2)
    assert orc.block_span_bytes(t) == 4 * 16 * 64 * 2
    # padded blocks: span is what the strides say, not the product of the extents
    t = orc.Tensor(None, 0, [orc.KV, orc.B, orc.L, orc.H, orc.D], [2, 10, 16, 2, 128],
                   [10 * 8192, 8192, 320, 128, 1], 2)
    assert orc.block_span_bytes(t) == 16 * 320 * 2


def test_block8_is_two_transactions_and_blocks01_merge():
    t = paper_tensor()
    # block 8 -> block 8: K and V spans, 8192 B each, disjoint
    k = orc.request_transactions(t, t, 0, [8], [8], 16)
    v = orc.request_transactions(t, t, 1, [8], [8], 16)
    both = np.concatenate([k, v])
    assert len(both) == int(GOLD["block8_transactions"])
    assert both[:, 2].tolist() == [8192, 8192]
    assert both[0, 0] == 65536 and both[1, 0] == 147456
    assert len(orc.coalesce(both)) == 2  # disjoint: they stay two
    # blocks 0 and 1: K tensors at 0 and 8192 -> one 16384 B transaction
    q = orc.request_transactions(t, t, 0, [0, 1], [0, 1], 32)
    assert q[:, 0].tolist() == [0, 8192]
    m = orc.coalesce(q)
    assert m.tolist() == [[0, 0, int(GOLD["blocks01_merged_bytes"])]]


def test_partial_last_block_moves_only_the_request_tokens():
    """Tokens beyond seq_len never appear in a transaction (closed forms for both inner orders)."""
    t = paper_tensor()  # [token][head][dim] inside a block: a token range is one byte range
    q = orc.request_transactions(t, t, 0, [3, 7], [2, 9], 16 + 5)
    assert q.tolist() == [[3 * 8192, 2 * 8192, 8192], [7 * 8192, 9 * 8192, 5 * 2 * 128 * 2]]
    assert q[:, 2].sum() == orc.transfer_bytes(21, 1, 2, 128, 2) // 2
    # [head][token][dim]: the 5 tokens are 5*128 elements in each of the two head planes
    hm = orc.Tensor(None, 0, [orc.B, orc.KV, orc.H, orc.L, orc.D], [10, 2, 2, 16, 128],
                    [4096, 40960, 2048, 128, 1], 2)
    q = orc.request_transactions(hm, hm, 1, [3, 7], [2, 9], 16 + 5)
    v = 40960 * 2
    assert q.tolist() == [[v + 3 * 8192, v + 2 * 8192, 8192],
                          [v + 7 * 8192, v + 9 * 8192, 5 * 128 * 2],
                          [v + 7 * 8192 + 4096, v + 9 * 8192 + 4096, 5 * 128 * 2]]
    # a single token, and an exact multiple (no tail at all)
    assert orc.request_transactions(t, t, 0, [4], [5], 1).tolist() == [[4 * 8192, 5 * 8192, 512]]
    assert len(orc.request_transactions(hm, hm, 0, [1, 2], [3, 4], 32)) == 2


def test_adjacent_k_and_v_are_queued_k_first_and_merge():
    # the paper's tensor keeps K and V 10 sub-tensors apart: K then V, two transactions that stay two
    t = paper_tensor()
    q = orc.request_transactions(t, t, -1, [8], [8], 16)
    assert q.tolist() == [[65536, 65536, 8192], [147456, 147456, 8192]]
    assert len(orc.coalesce(q)) == 2
    # same shapes, but V of a block right behind its K (stride of KV = one sub-tensor)
    adj = orc.Tensor(None, 0, [orc.B, orc.KV, orc.L, orc.H, orc.D], [10, 2, 16, 2, 128],
                     [8192, 4096, 256, 128, 1], 2)
    q = orc.request_transactions(adj, adj, -1, [3, 4], [6, 7], 32)
    assert q.tolist() == [[3 * 16384, 6 * 16384, 8192], [3 * 16384 + 8192, 6 * 16384 + 8192, 8192],
                          [4 * 16384, 7 * 16384, 8192], [4 * 16384 + 8192, 7 * 16384 + 8192, 8192]]
    assert orc.coalesce(q).tolist() == [[3 * 16384, 6 * 16384, 4 * 8192]]
    # a partial block: the K part and the V part are apart again
    q = orc.request_transactions(adj, adj, -1, [3], [6], 5)
    assert q.tolist() == [[3 * 16384, 6 * 16384, 2560], [3 * 16384 + 8192, 6 * 16384 + 8192, 2560]]
    assert len(orc.coalesce(q)) == 2


# ---------------------------------------------------------------- section 4.2 queue example

def test_queue_example_merges_across_requests():
    t = paper_tensor()
    r1s, r1d = (int(x) for x in GOLD["queue_R1"].split())
    r2s, r2d = (int(x) for x in GOLD["queue_R2_first"].split())
    q = np.concatenate([
        orc.request_transactions(t, t, 0, [r1s], [r1d], 16),
        # R2's second read is not given in the text; 3 -> 9 is this test's choice (not adjacent)
        orc.request_transactions(t, t, 0, [r2s, 3], [r2d, 9], 32),
    ])
    m = orc.coalesce(q)
    assert len(m) == int(GOLD["queue_merged_transactions_per_tensor"]) + 1
    assert m[0].tolist() == [0, 5 * 8192, 2 * 8192]
    assert m[1].tolist() == [3 * 8192, 9 * 8192, 8192]


def test_merging_stops_at_a_completion_in_the_queue():
    """Section 4.2 pops the reads "until the first completion" and merges among those.  The same two reads of the
    queue example merge when both are queued before any completion, and stay two transactions when R1's completion
    sits between them (each request's reads merged by themselves, the lists put one behind the other)."""
    t = paper_tensor()
    r1s, r1d = (int(x) for x in GOLD["queue_R1"].split())
    r2s, r2d = (int(x) for x in GOLD["queue_R2_first"].split())
    r1 = orc.request_transactions(t, t, 0, [r1s], [r1d], 16)
    r2 = orc.request_transactions(t, t, 0, [r2s], [r2d], 16)
    assert orc.coalesce(np.concatenate([r1, r2])).tolist() == [[0, 5 * 8192, 2 * 8192]]
    stopped = np.concatenate([orc.coalesce(r1), orc.coalesce(r2)])
    assert stopped.tolist() == [[0, 5 * 8192, 8192], [8192, 6 * 8192, 8192]]


def test_merge_needs_both_sides_contiguous():
    # remote contiguous, local not -> no merge; and the other way round
    assert len(orc.coalesce([[0, 0, 100], [100, 300, 100]])) == 2
    assert len(orc.coalesce([[0, 0, 100], [300, 100, 100]])) == 2
    assert orc.coalesce([[0, 0, 100], [100, 100, 50], [150, 150, 10]]).tolist() == [[0, 0, 160]]
    # order matters: a later transaction that would continue an earlier, non-neighbouring one stays
    assert len(orc.coalesce([[0, 0, 100], [500, 500, 100], [100, 100, 100]])) == 3
    assert len(orc.coalesce(np.zeros((0, 3)))) == 0


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_run_count_closed_form(seed):
    # full blocks of equal size: merged count = 1 + number of positions where either side breaks
    rng = np.random.default_rng(seed)
    g = wl.PoolGeometry(1, 256, 16, 2, 32, 2, wl.BHTD)
    free_s, free_d = np.ones(256, bool), np.ones(256, bool)
    n = 100
    st = wl.fragmented_allocation(rng, free_s, n, 6)
    dt = wl.fragmented_allocation(rng, free_d, n, 6)
    w = wl.Workload("t", g, g, [wl.Request(n * 16, st, dt)], "bf16", seed)
    got = tl.oracle_plan_descriptors(w, 0, 1)
    breaks = np.count_nonzero((st[1:] != st[:-1] + 1) | (dt[1:] != dt[:-1] + 1))
    assert len(got) == 1 + breaks
    assert got[:, 2].sum() == n * g.tile_elems * 2
    # V tensor: offsets sit stride_kv above the K tensor's
    k = tl.oracle_plan_descriptors(w, 0, 0)
    assert np.array_equal(got[:, 0] - k[:, 0], np.full(len(k), g.stride_kv * 2))


# ---------------------------------------------------------------- sizes the paper quotes

def test_sizes_quoted_in_paper():
    per_token = orc.transfer_bytes(1, int(GOLD["mistral_large_layers"]), int(GOLD["mistral_large_kv_heads"]),
                                   int(GOLD["mistral_large_head_dim"]), 2)
    assert per_token == int(GOLD["mistral_large_bytes_per_token_KB"]) * 1024
    share = orc.transfer_bytes(int(GOLD["l70b_tokens"]), int(GOLD["l70b_layers"]),
                               int(GOLD["l70b_kv_heads_per_gpu"]), int(GOLD["l70b_head_dim"]), 2)
    assert share == int(GOLD["l70b_share_MB"]) * 2 ** 20
    # 2048 disjoint 4 KB pieces per layer = 1024 blocks x {K, V}
    g = wl.PoolGeometry(1, 2048, 16, 1, 128, 2, wl.BHTD)
    tbl = wl.scattered_table(np.random.default_rng(0), 2048, 1024)
    w = wl.Workload("t", g, g, [wl.Request(16384, tbl, tbl)], "bf16", 0)
    pieces = np.concatenate([tl.oracle_plan_descriptors(w, 0, 0), tl.oracle_plan_descriptors(w, 0, 1)])
    assert len(pieces) == int(GOLD["l70b_pieces_per_layer"])
    assert set(pieces[:, 2].tolist()) == {int(GOLD["l70b_piece_bytes"])}
    # 8K tokens <-> 1024 pieces of 4 KB
    w8 = wl.Workload("t", g, g, [wl.Request(8192, tbl[:512], tbl[:512])], "bf16", 0)
    n8 = len(tl.oracle_plan_descriptors(w8, 0, 0)) + len(tl.oracle_plan_descriptors(w8, 0, 1))
    assert n8 == int(GOLD["pieces_for_8k_tokens"])


def test_runs_of_fixed_length_coalesce_to_one_transaction_per_run():
    """Tables built from runs of exactly k adjacent blocks on both sides: the merged queue has one
    transaction per run, each of k whole blocks (the last one what is left), in request order."""
    g = wl.PoolGeometry(1, 512, 16, 2, 32, 2, wl.BHTD)
    block = 16 * 2 * 32 * 2
    for run in (1, 2, 3, 8):
        rng = np.random.default_rng(run)
        n = 50
        st, dt = wl.fixed_run_table(rng, 512, n, run), wl.fixed_run_table(rng, 512, n, run)
        assert len(set(st.tolist())) == n and len(set(dt.tolist())) == n
        w = wl.Workload("t", g, g, [wl.Request(n * 16, st, dt)], "bf16", 0)
        d = tl.oracle_plan_descriptors(w, 0, 0)
        want = [min(run, n - i) * block for i in range(0, n, run)]
        assert d[:, 2].tolist() == want
        assert d[:, 0].tolist() == [int(st[i]) * block for i in range(0, n, run)]
        assert d[:, 1].tolist() == [int(dt[i]) * block for i in range(0, n, run)]
        # a straight table on one side does not merge what the other side breaks
        w1 = wl.Workload("t", g, g, [wl.Request(n * 16, st, np.arange(n, dtype=np.int32))], "bf16", 0)
        assert tl.oracle_plan_descriptors(w1, 0, 0)[:, 2].tolist() == want


def test_block_major_pools_coalesce_a_block_over_all_its_layers():
    """Pools that keep every layer of a block together, layer tensors queued block by block: a run
    of r adjacent whole blocks is ONE transaction of r * layers * (K + V) tiles; a ragged last
    block adds one range per (layer, K/V, head)."""
    layers, hk = 3, 2
    g = wl.PoolGeometry(layers, 64, 4, hk, 8, 2, wl.BHTD, block_major=True)
    tile = 4 * hk * 8 * 2
    block_bytes = layers * 2 * tile
    st = np.array([10, 11, 12, 40, 41, 7], np.int32)
    dt = np.array([20, 21, 22, 50, 51, 9], np.int32)
    w = wl.Workload("t", g, g, [wl.Request(24, st, dt)], "bf16", 0)
    d = tl.oracle_plan_descriptors_block_major(w)
    assert d.tolist() == [[10 * block_bytes, 20 * block_bytes, 3 * block_bytes],
                          [40 * block_bytes, 50 * block_bytes, 2 * block_bytes],
                          [7 * block_bytes, 9 * block_bytes, block_bytes]]
    # layers 1..2 only: the range starts one layer into the block and two blocks no longer touch
    w12 = wl.Workload("t", g, g, [wl.Request(24, st, dt)], "bf16", 0, layer_begin=1, layer_end=3)
    d = tl.oracle_plan_descriptors_block_major(w12)
    assert len(d) == 6 and set(d[:, 2].tolist()) == {2 * 2 * tile}
    assert d[0].tolist() == [10 * block_bytes + 2 * tile, 20 * block_bytes + 2 * tile, 4 * tile]
    # ragged tail (22 tokens: the last block holds 2 of 4 slots): per (layer, K/V, head) ranges of 2 rows
    wr = wl.Workload("t", g, g, [wl.Request(22, st, dt)], "bf16", 0)
    d = tl.oracle_plan_descriptors_block_major(wr)
    assert len(d) == 2 + layers * 2 * hk
    assert set(d[2:, 2].tolist()) == {2 * 8 * 2}
    assert d[:, 2].sum() == 22 * layers * 2 * hk * 8 * 2
    # the same queue order in layer-major pools merges nothing at all (consecutive entries belong to
    # different layers, far apart), while the layer-by-layer order merges the runs of each tensor
    gl = wl.PoolGeometry(layers, 64, 4, hk, 8, 2, wl.BHTD)
    wlm = wl.Workload("t", gl, gl, [wl.Request(24, st, dt)], "bf16", 0)
    assert len(tl.oracle_plan_descriptors_block_major(wlm)) == 6 * layers * 2
    assert len(tl.oracle_plan_descriptors(wlm, 0, 0)) == 3


# ---------------------------------------------------------------- the copy itself

def tiny_workloads():
    rng = np.random.default_rng(7)
    out = []
    # same layout, ragged tail, two requests
    g = wl.PoolGeometry(2, 8, 4, 2, 8, 2, wl.BHTD)
    perm_s, perm_d = rng.permutation(8), rng.permutation(8)
    out.append(wl.Workload("tiny-bhtd", g, g, [
        wl.Request(10, perm_s[:3].astype(np.int32), perm_d[:3].astype(np.int32)),
        wl.Request(5, perm_s[3:5].astype(np.int32), perm_d[3:5].astype(np.int32)),
    ], "bf16", 7))
    # token-major both sides
    g2 = wl.PoolGeometry(2, 8, 4, 3, 8, 2, wl.BTHD)
    out.append(wl.Workload("tiny-bthd", g2, g2, [
        wl.Request(13, perm_s[:4].astype(np.int32), perm_d[:4].astype(np.int32))], "bf16", 7))
    # re-layout with different block sizes, both directions
    gs = wl.PoolGeometry(2, 8, 4, 2, 8, 2, wl.BHTD)
    gd = wl.PoolGeometry(2, 4, 8, 2, 8, 2, wl.BTHD)
    out.append(wl.Workload("tiny-relayout", gs, gd, [
        wl.Request(19, perm_s[:5].astype(np.int32), rng.permutation(4)[:3].astype(np.int32))], "bf16", 7))
    out.append(wl.Workload("tiny-relayout-back", gd, gs, [
        wl.Request(19, rng.permutation(4)[:3].astype(np.int32), perm_s[:5].astype(np.int32))], "bf16", 7))
    # a layer sub-range
    out.append(wl.Workload("tiny-layers", g, g, [
        wl.Request(7, perm_s[:2].astype(np.int32), perm_d[:2].astype(np.int32))], "bf16", 7,
        layer_begin=1, layer_end=2))
    # pools that keep all layers of a block together, on both sides and on one side only
    gb = wl.PoolGeometry(3, 8, 4, 2, 8, 2, wl.BHTD, block_major=True)
    out.append(wl.Workload("tiny-block-major", gb, gb, [
        wl.Request(10, perm_s[:3].astype(np.int32), perm_d[:3].astype(np.int32))], "bf16", 7,
        layer_begin=1, layer_end=3))
    gb2 = wl.PoolGeometry(2, 8, 4, 2, 8, 2, wl.BHTD, block_major=True)
    out.append(wl.Workload("tiny-block-major-src", gb2, g, [
        wl.Request(10, perm_s[:3].astype(np.int32), perm_d[:3].astype(np.int32))], "bf16", 7))
    # four-byte elements
    g4 = wl.PoolGeometry(1, 6, 4, 2, 4, 4, wl.BHTD)
    out.append(wl.Workload("tiny-e4", g4, g4, [
        wl.Request(9, np.array([4, 0, 2], np.int32), np.array([1, 5, 3], np.int32))], "bf16", 7))
    return out


def _random_pool(g, seed, sentinel=False):
    dt = {1: np.uint8, 2: np.uint16, 4: np.uint32}[g.elem_bytes]
    if sentinel:
        return np.full(g.total_elems, 0x7FA5 if g.elem_bytes >= 2 else 0xA5, dtype=dt)
    rng = np.random.default_rng(seed)
    x = rng.integers(0, np.iinfo(dt).max, size=g.total_elems, dtype=dt, endpoint=False)
    x[x == 0x7FA5] = 1
    return x


@pytest.mark.parametrize("w", tiny_workloads(), ids=lambda w: w.name)
def test_oracle_equals_brute_force_and_writes_each_element_once(w):
    src = _random_pool(w.src, 11)
    src_before = src.copy()
    dst_oracle = _random_pool(w.dst, 0, sentinel=True)
    dst_brute = dst_oracle.copy()
    tl.oracle_pull_workload(w, src.view(np.uint8), dst_oracle.view(np.uint8))
    count = tl.brute_force_pull(w, src, dst_brute)
    assert np.array_equal(dst_oracle, dst_brute)
    assert count.max() == 1  # exactly once
    moved = w.total_tokens * (w.layer_end - w.layer_begin) * 2 * w.src.num_kv_heads * w.src.head_dim
    assert int(count.sum()) == moved
    assert moved * w.src.elem_bytes == sum(
        orc.transfer_bytes(r.seq_len, w.layer_end - w.layer_begin, w.src.num_kv_heads,
                           w.src.head_dim, w.src.elem_bytes) for r in w.requests)
    # everything that was not a target keeps the sentinel; the source is untouched
    assert np.all(dst_oracle[count == 0] == dst_oracle.dtype.type(0x7FA5))
    assert np.count_nonzero(dst_oracle != dst_oracle.dtype.type(0x7FA5)) == moved
    assert np.array_equal(src, src_before)


def _view(g, flat):
    """numpy's own addressing of the pool: reshape, no stride arithmetic of ours."""
    if g.block_major:
        if g.layout == wl.BHTD:
            v = flat.reshape(g.num_blocks, g.num_layers, 2, g.num_kv_heads, g.block_tokens, g.head_dim)
        else:
            v = flat.reshape(g.num_blocks, g.num_layers, 2, g.block_tokens, g.num_kv_heads,
                             g.head_dim).transpose(0, 1, 2, 4, 3, 5)
        return v.transpose(1, 2, 0, 3, 4, 5)  # -> [layer, kv, block, head, token, dim]
    if g.layout == wl.BHTD:
        return flat.reshape(g.num_layers, 2, g.num_blocks, g.num_kv_heads, g.block_tokens, g.head_dim)
    return flat.reshape(g.num_layers, 2, g.num_blocks, g.block_tokens, g.num_kv_heads,
                        g.head_dim).transpose(0, 1, 2, 4, 3, 5)  # -> [..., head, token, dim]


@pytest.mark.parametrize("block_major", [(False, False), (True, True), (False, True)])
@pytest.mark.parametrize("src_layout,dst_layout,tbs,tbd", [
    (wl.BHTD, wl.BHTD, 16, 16), (wl.BTHD, wl.BTHD, 8, 8), (wl.BHTD, wl.BTHD, 16, 32),
    (wl.BTHD, wl.BHTD, 32, 16), (wl.BHTD, wl.BHTD, 8, 16)])
def test_unique_ids_arrive_where_reshape_says(src_layout, dst_layout, tbs, tbd, block_major):
    """Fill the source so that logical element (layer, kv, token, head, dim) holds its own id;
    after the pull, the destination read through numpy's reshape view must hold the same ids."""
    rng = np.random.default_rng(3)
    layers, hk, dd, tokens = 3, 3, 8, 75
    gs = wl.PoolGeometry(layers, 16, tbs, hk, dd, 4, src_layout, block_major=block_major[0])
    gd = wl.PoolGeometry(layers, 16 * tbs // tbd + 2, tbd, hk, dd, 4, dst_layout, block_major=block_major[1])
    st = wl.permutation_table(rng, gs.num_blocks, wl.blocks_for(tokens, tbs))
    dt = wl.permutation_table(rng, gd.num_blocks, wl.blocks_for(tokens, tbd))
    src = np.zeros(gs.total_elems, np.uint32)
    sv = _view(gs, src)
    ids = np.arange(layers * 2 * tokens * hk * dd, dtype=np.uint32).reshape(layers, 2, tokens, hk, dd) + 1
    for t in range(tokens):
        sv[:, :, st[t // tbs], :, t % tbs, :] = ids[:, :, t]
    dst = np.full(gd.total_elems, 0x7FA5, np.uint32)
    w = wl.Workload("ids", gs, gd, [wl.Request(tokens, st, dt)], "bf16", 3)
    tl.oracle_pull_workload(w, src.view(np.uint8), dst.view(np.uint8))
    dv = _view(gd, dst)
    for t in range(tokens):
        assert np.array_equal(dv[:, :, dt[t // tbd], :, t % tbd, :], ids[:, :, t]), t
    assert np.count_nonzero(dst != 0x7FA5) == ids.size


def test_round_trip_is_identity_on_valid_tokens():
    w = tiny_workloads()[2]  # re-layout
    src = _random_pool(w.src, 5)
    mid = _random_pool(w.dst, 0, sentinel=True)
    back = _random_pool(w.src, 0, sentinel=True)
    tl.oracle_pull_workload(w, src.view(np.uint8), mid.view(np.uint8))
    r = w.requests[0]
    wb = wl.Workload("back", w.dst, w.src, [wl.Request(r.seq_len, r.dst_table, r.src_table)], "bf16", 0)
    tl.oracle_pull_workload(wb, mid.view(np.uint8), back.view(np.uint8))
    touched = back != 0x7FA5
    assert np.array_equal(back[touched], src[touched])
    assert np.count_nonzero(touched) == r.seq_len * 2 * 2 * w.src.num_kv_heads * w.src.head_dim


def test_identity_tables_reduce_to_memcpy():
    g = wl.PoolGeometry(2, 8, 4, 2, 8, 2, wl.BHTD)
    n = 5
    tbl = np.arange(n, dtype=np.int32)
    w = wl.Workload("ident", g, g, [wl.Request(n * 4, tbl, tbl)], "bf16", 0)
    src = _random_pool(g, 9)
    dst = _random_pool(g, 0, sentinel=True)
    tl.oracle_pull_workload(w, src.view(np.uint8), dst.view(np.uint8))
    expect = np.full_like(dst, 0x7FA5)
    for layer in range(2):
        for kv in range(2):
            o = layer * g.stride_layer + kv * g.stride_kv
            expect[o:o + n * g.tile_elems] = src[o:o + n * g.tile_elems]  # one memcpy per slab
    assert np.array_equal(dst, expect)


def test_config1_shapes():
    w = wl.config1()
    assert w.src.tile_elems * 2 == 8192 and len(w.requests[0].src_table) == 8
    assert orc.transfer_bytes(128, 2, 4, 64, 2) == 256 * 1024


@pytest.mark.parametrize("seed", range(40))
def test_oracle_equals_brute_force_on_random_tiny_geometries(seed):
    """Random small shapes: inner orders, block-size ratios, K/V placement, element widths, layer ranges."""
    rng = np.random.default_rng(900 + seed)
    elem = int(rng.choice([1, 2, 4]))
    hk, dd, layers = int(rng.integers(1, 4)), int(rng.choice([2, 4, 8])), int(rng.integers(1, 4))
    tbs = int(rng.choice([1, 2, 4, 8]))
    tbd = tbs * int(rng.choice([1, 2, 4])) if rng.random() < 0.5 else max(1, tbs // int(rng.choice([1, 2, 4])))
    tokens = int(rng.integers(1, 40))
    gs = wl.PoolGeometry(layers, wl.blocks_for(tokens, tbs) + 3, tbs, hk, dd, elem,
                         str(rng.choice([wl.BHTD, wl.BTHD])), bool(rng.random() < 0.4))
    gd = wl.PoolGeometry(layers, wl.blocks_for(tokens, tbd) + 3, tbd, hk, dd, elem,
                         str(rng.choice([wl.BHTD, wl.BTHD])), bool(rng.random() < 0.4))
    l0 = int(rng.integers(0, layers))
    l1 = int(rng.integers(l0 + 1, layers + 1))
    if seed >= 15:  # the later seeds also draw pools that keep all layers of a block together
        gs = dataclasses.replace(gs, block_major=bool(rng.random() < 0.5))
        gd = dataclasses.replace(gd, block_major=bool(rng.random() < 0.5))
    w = wl.Workload("rand", gs, gd, [wl.Request(tokens, wl.permutation_table(rng, gs.num_blocks, wl.blocks_for(tokens, tbs)),
                                                wl.permutation_table(rng, gd.num_blocks, wl.blocks_for(tokens, tbd)))],
                    "bf16", seed, l0, l1)
    dt = {1: np.uint8, 2: np.uint16, 4: np.uint32}[elem]
    src = rng.integers(0, 200, size=gs.total_elems).astype(dt)
    dst_o = np.full(gd.total_elems, 0xA5, dtype=dt)
    dst_b = dst_o.copy()
    tl.oracle_pull_workload(w, src.view(np.uint8), dst_o.view(np.uint8))
    count = tl.brute_force_pull(w, src, dst_b)
    assert np.array_equal(dst_o, dst_b)
    assert count.max() == 1 and int(count.sum()) == tokens * (l1 - l0) * 2 * hk * dd
    # the transactions of every layer tensor tile the moved bytes exactly once on both sides
    s_t, d_t = tl.oracle_tensors(gs, None)[l0], tl.oracle_tensors(gd, None)[l0]
    q = orc.request_transactions(s_t, d_t, -1, w.requests[0].src_table, w.requests[0].dst_table, tokens)
    assert q[:, 2].sum() == tokens * 2 * hk * dd * elem
    for col in (0, 1):
        o = np.argsort(q[:, col])
        assert np.all(q[o, col][1:] >= (q[o, col] + q[o, 2])[:-1])  # no two ranges overlap
    m = orc.coalesce(q)
    assert m[:, 2].sum() == q[:, 2].sum() and len(m) <= len(q)


@pytest.mark.parametrize("kw", [{}, {"kv_adjacent": True}, {"block_major": True}])
def test_input_generator_strides_equal_the_test_glue_own_derivation(kw):
    """The oracle is given strides that the test glue works out from the order of the pool's axes; the library is
    given the strides the input generators carry.  Both describe the same dense allocation."""
    for layout in (wl.BHTD, wl.BTHD):
        g = wl.PoolGeometry(3, 7, 16, 2, 64, 2, layout, **kw)
        assert tl.outer_strides(g) == (g.stride_layer, g.stride_kv, g.stride_block)
        assert g.total_bytes == 3 * 2 * 7 * 16 * 2 * 64 * 2
