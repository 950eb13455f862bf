"""Parity of the HIP path with the CPU oracle, through the C ABI, bit for bit.

Small cases compare whole pools element by element; the full-size configurations compare every
layer with the oracle, slab by slab (the batch of 64 requests: eight layers spread over the pool),
and check size-independent properties on every layer."""
import dataclasses

import numpy as np
import pytest
import torch

import kvd_testlib as tl
from oracle import kvd_oracle as orc
from paper_2501_14743_amd import kvd
from paper_2501_14743_amd import workloads as wl

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import kvd_gpu as G


def say(msg):
    print(f"[kvd-test] {msg}", flush=True)


def host_src(w, seed=None):
    return wl.host_pool_values(w.src, w.dtype, w.seed if seed is None else seed)


# ------------------------------------------------------------------ the five configurations, reduced

def reduced_configs():
    return [
        wl.config1(),
        wl.config2(num_layers=2, pool_blocks=2048, tokens=8192),
        wl.config3(num_layers=2, num_requests=16, median=256.0, hi=2048),
        wl.config4(num_layers=4, pool_blocks=2048, tokens=8192),
        wl.config5(num_layers=2, src_pool_blocks=512, tokens=2000),
    ]


@pytest.mark.parametrize("w", reduced_configs(), ids=lambda w: w.name)
def test_reduced_configs_match_oracle(w):
    say(f"{w.name}: {len(w.requests)} requests, {w.total_tokens} tokens")
    x = G.run_and_compare(w, host_src(w))
    st = x.plan.stats(x.stream.cuda_stream)
    assert st["num_requests"] == len(w.requests)
    assert st["payload_bytes"] == w.total_tokens * (w.layer_end - w.layer_begin) * 2 * \
        w.src.num_kv_heads * w.src.head_dim * w.src.elem_bytes
    x.close()


@pytest.mark.parametrize("w", reduced_configs()[:4], ids=lambda w: w.name)
def test_descriptors_equal_oracle_coalescing(w):
    """Byte-copy plans: the compacted descriptor list is exactly the oracle's merged queue."""
    src = G.device_sentinel_pool(w.src)
    dst = G.device_sentinel_pool(w.dst)
    x = G.GpuTransfer(w, src, dst)
    x.build()
    got = x.plan.descriptors(x.stream.cuda_stream)
    st = x.plan.stats(x.stream.cuda_stream)
    assert st["relayout"] == 0
    want = tl.oracle_plan_descriptors(w, 0, 0)
    assert np.array_equal(got, want)
    assert st["num_descriptors"] == len(want) <= st["num_transactions"]
    # and for another (layer, K/V) tensor the same list shifted by the slab strides
    want_v = tl.oracle_plan_descriptors(w, 1, 1)
    shift_s = (w.src.stride_layer + w.src.stride_kv) * w.src.elem_bytes
    shift_d = (w.dst.stride_layer + w.dst.stride_kv) * w.dst.elem_bytes
    assert np.array_equal(got + np.array([shift_s, shift_d, 0]), want_v)
    x.close()


def test_batched_build_equals_one_call_per_request():
    w = wl.config3(num_layers=2, num_requests=40, median=200.0, hi=3000)
    src_host = host_src(w)
    src, dst = G.device_pool_from_host(src_host), G.device_sentinel_pool(w.dst)
    one = G.GpuTransfer(w, src, dst)
    one.build(batch=False)
    d_one = one.plan.descriptors(one.stream.cuda_stream)
    st_one = one.plan.stats(one.stream.cuda_stream)
    one.close()
    x = G.GpuTransfer(w, src, dst)
    x.run(batch=True)
    assert np.array_equal(x.plan.descriptors(x.stream.cuda_stream), d_one)
    assert x.plan.stats(x.stream.cuda_stream) == st_one
    assert np.array_equal(d_one, tl.oracle_plan_descriptors(w, 0, 0))
    G.assert_bytes_equal(dst.cpu().numpy(), G.oracle_expected(w, src_host), "batched build")
    x.close()


def test_batch_larger_than_one_launch_takes():
    # 700 short requests: more than one build launch holds; mixed with an earlier single request
    g = wl.PoolGeometry(1, 4096, 16, 2, 64, 2, wl.BHTD)
    rng = np.random.default_rng(12)
    free_s, free_d = np.ones(4096, bool), np.ones(4096, bool)
    reqs = []
    for _ in range(701):
        t = int(rng.integers(1, 70))
        n = wl.blocks_for(t, 16)
        reqs.append(wl.Request(t, wl.fragmented_allocation(rng, free_s, n, 4), wl.fragmented_allocation(rng, free_d, n, 4)))
    w = wl.Workload("many", g, g, reqs, "bf16", 12)
    src_host = host_src(w)
    src, dst = G.device_pool_from_host(src_host), G.device_sentinel_pool(g)
    x = G.GpuTransfer(w, src, dst)
    r0 = reqs[0]
    x.plan.build_descriptors(r0.src_table, r0.dst_table, r0.seq_len, 0, 1, x.stream.cuda_stream)
    x.plan.build_descriptors_batch([r.src_table for r in reqs[1:]], [r.dst_table for r in reqs[1:]],
                                   [r.seq_len for r in reqs[1:]], 0, 1, x.stream.cuda_stream)
    x.pull()
    x.stream.synchronize()
    assert x.plan.stats(x.stream.cuda_stream)["num_requests"] == 701
    assert np.array_equal(x.plan.descriptors(x.stream.cuda_stream), tl.oracle_plan_descriptors(w, 0, 0))
    G.assert_bytes_equal(dst.cpu().numpy(), G.oracle_expected(w, src_host), "701 requests")
    x.close()


@pytest.mark.parametrize("n_req,appended", [(250, False), (250, True), (500, False), (500, True)])
def test_one_build_launch_below_and_above_its_descriptor_cache(n_req, appended):
    """One build launch keeps up to 1024 new descriptors in LDS and falls back to global memory beyond that:
    250 requests stay below (about 860 descriptors), 500 go above (about 1700).  `appended`: a request built
    before the batch leaves a descriptor that the batch's first transaction continues."""
    g = wl.PoolGeometry(2, 4096, 16, 2, 64, 2, wl.BTHD)
    rng = np.random.default_rng(1000 + n_req)
    free_s, free_d = np.ones(4096, bool), np.ones(4096, bool)
    free_s[:8] = free_d[:8] = False
    first = wl.Request(64, np.arange(0, 4, dtype=np.int32), np.arange(0, 4, dtype=np.int32))
    reqs = [first, wl.Request(40, np.arange(4, 7, dtype=np.int32), np.arange(4, 7, dtype=np.int32))]
    for _ in range(n_req - 2):
        t = int(rng.integers(33, 64))
        n = wl.blocks_for(t, 16)
        reqs.append(wl.Request(t, wl.fragmented_allocation(rng, free_s, n, 1), wl.fragmented_allocation(rng, free_d, n, 1)))
    w = wl.Workload("cache", g, g, reqs, "bf16", 13)
    src_host = host_src(w)
    src, dst = G.device_pool_from_host(src_host), G.device_sentinel_pool(g)
    x = G.GpuTransfer(w, src, dst)
    rest = reqs
    if appended:
        x.plan.build_descriptors(first.src_table, first.dst_table, first.seq_len, 0, 2, x.stream.cuda_stream)
        rest = reqs[1:]
    x.plan.build_descriptors_batch([r.src_table for r in rest], [r.dst_table for r in rest],
                                   [r.seq_len for r in rest], 0, 2, x.stream.cuda_stream)
    x.pull()
    x.stream.synchronize()
    want = tl.oracle_plan_descriptors(w, 0, 0)
    assert (len(want) < 1024) == (n_req == 250), len(want)
    assert np.array_equal(x.plan.descriptors(x.stream.cuda_stream), want)
    G.assert_bytes_equal(dst.cpu().numpy(), G.oracle_expected(w, src_host), "descriptor cache")
    x.close()


def test_wide_expansion_continues_an_open_descriptor():
    """A long request (its work items are written by the separate wide launch) that continues the
    previous request's last descriptor, whose last work item was a short one; then another long
    request that may not merge (other layers)."""
    g = wl.PoolGeometry(2, 40000, 16, 1, 80, 2, wl.BHTD)  # 2560-byte blocks: 1.6 blocks per work item
    n_b = 14000
    a = wl.Request(3 * 16, np.arange(100, 103, dtype=np.int32), np.arange(200, 203, dtype=np.int32))
    tail_s = np.array([30000, 30001, 5, 39999], np.int32)
    tail_d = np.array([31000, 31001, 39999, 7], np.int32)
    b = wl.Request((n_b + 4) * 16 - 3, np.concatenate([np.arange(103, 103 + n_b, dtype=np.int32), tail_s]),
                   np.concatenate([np.arange(203, 203 + n_b, dtype=np.int32), tail_d]))
    c = wl.Request(n_b * 16, np.arange(15000, 15000 + n_b, dtype=np.int32), np.arange(16000, 16000 + n_b, dtype=np.int32))
    src_host = host_src(wl.Workload("wide", g, g, [], "bf16", 51))
    src, dst = G.device_pool_from_host(src_host), G.device_sentinel_pool(g)
    plan = kvd.Plan(kvd.Pool(src.data_ptr(), g), kvd.Pool(dst.data_ptr(), g), 3, 2 * n_b + 16)
    plan.build_descriptors(a.src_table, a.dst_table, a.seq_len, 0, 2)
    assert plan.stats()["num_work_items"] == 2                      # 7680 bytes: one whole item and a short one
    plan.build_descriptors(b.src_table, b.dst_table, b.seq_len, 0, 2)
    st = plan.stats()
    assert st["num_descriptors"] == 4 and st["num_work_items"] > 8192
    want_ab = tl.oracle_plan_descriptors(wl.Workload("ab", g, g, [a, b], "bf16", 51), 0, 0)
    assert np.array_equal(plan.descriptors(), want_ab) and want_ab[0, 2] == (3 + n_b) * 2560
    plan.build_descriptors(c.src_table, c.dst_table, c.seq_len, 1, 2)
    assert plan.stats()["num_descriptors"] == 5
    plan.pull()
    torch.cuda.synchronize()
    want = wl.host_pool_sentinel(g)
    tl.oracle_pull_workload(wl.Workload("ab", g, g, [a, b], "bf16", 51), src_host, want)
    tl.oracle_pull_workload(wl.Workload("c", g, g, [c], "bf16", 51, 1, 2), src_host, want)
    G.assert_bytes_equal(dst.cpu().numpy(), want, "wide expansion")
    plan.close()


def test_no_coalesce_flag_keeps_every_transaction_and_same_bytes():
    w = wl.config2(num_layers=2, pool_blocks=1024, tokens=3000)
    x = G.run_and_compare(w, host_src(w), flags=kvd.KVD_PLAN_NO_COALESCE)
    st = x.plan.stats(x.stream.cuda_stream)
    assert st["num_descriptors"] == st["num_transactions"] == 187 + 8  # 187 whole blocks + 8 head rows
    x.close()


def test_relayout_pieces():
    w = wl.config5(num_layers=1, src_pool_blocks=64, tokens=100)
    x = G.GpuTransfer(w, G.device_sentinel_pool(w.src), G.device_sentinel_pool(w.dst))
    x.build()
    got = x.plan.descriptors(x.stream.cuda_stream)
    r = w.requests[0]
    want = [(r.src_table[p], 0, r.dst_table[p // 2], (p % 2) * 16, min(16, 100 - 16 * p)) for p in range(7)]
    assert got.tolist() == [list(map(int, t)) for t in want]
    x.close()


# ------------------------------------------------------------------ edge cases

def small_geom(**kw):
    base = dict(num_layers=3, num_blocks=96, block_tokens=16, num_kv_heads=4, head_dim=64, elem_bytes=2,
                layout=wl.BHTD)
    base.update(kw)
    return wl.PoolGeometry(**base)


def one_request(gs, gd, tokens, seed=5, **kw):
    rng = np.random.default_rng(seed)
    return wl.Workload(f"edge-{tokens}", gs, gd, [wl.Request(
        tokens, wl.permutation_table(rng, gs.num_blocks, wl.blocks_for(tokens, gs.block_tokens)),
        wl.permutation_table(rng, gd.num_blocks, wl.blocks_for(tokens, gd.block_tokens)))], "bf16", seed, **kw)


@pytest.mark.parametrize("tokens", [1, 15, 16, 17, 255, 1000])
@pytest.mark.parametrize("layout", [wl.BHTD, wl.BTHD])
def test_ragged_lengths(tokens, layout):
    g = small_geom(layout=layout)
    w = one_request(g, g, tokens)
    say(f"ragged {layout} {tokens}")
    G.run_and_compare(w, host_src(w)).close()


@pytest.mark.parametrize("gs,gd", [
    (small_geom(block_tokens=8, num_blocks=192), small_geom(block_tokens=16)),                       # head-major, 8 -> 16
    (small_geom(block_tokens=32, num_blocks=48), small_geom(block_tokens=8, num_blocks=192)),                       # head-major, 32 -> 8
    (small_geom(layout=wl.BTHD), small_geom(layout=wl.BTHD, block_tokens=32, num_blocks=48)),       # token-major 16 -> 32
    (small_geom(), small_geom(layout=wl.BTHD)),                                                     # re-layout, equal block size
    (small_geom(layout=wl.BTHD, block_tokens=32, num_blocks=48), small_geom()),                     # re-layout back, 32 -> 16
    (small_geom(num_kv_heads=3, head_dim=96), small_geom(num_kv_heads=3, head_dim=96, layout=wl.BTHD, block_tokens=64, num_blocks=24)),
    (small_geom(num_kv_heads=3, head_dim=96, layout=wl.BTHD), small_geom(num_kv_heads=3, head_dim=96, block_tokens=4, num_blocks=384)),
    (small_geom(num_kv_heads=1), small_geom(num_kv_heads=1, layout=wl.BTHD, block_tokens=32, num_blocks=48)),  # one head: layouts coincide
], ids=["hm8-16", "hm32-8", "tm16-32", "relayout-eq", "relayout-back", "relayout-odd", "relayout-odd-back", "one-head"])
@pytest.mark.parametrize("tokens", [333, 1024])
def test_mixed_block_sizes_and_layouts(gs, gd, tokens):
    w = one_request(gs, gd, tokens)
    say(f"mixed {gs.layout}{gs.block_tokens}->{gd.layout}{gd.block_tokens} {tokens}")
    G.run_and_compare(w, host_src(w)).close()


@pytest.mark.parametrize("elem_bytes,head_dim", [(1, 128), (4, 32), (8, 16)])
def test_element_sizes(elem_bytes, head_dim):
    g = small_geom(elem_bytes=elem_bytes, head_dim=head_dim)
    w = one_request(g, g, 200)
    rng = np.random.default_rng(1)
    src = rng.integers(0, 255, size=g.total_bytes, dtype=np.uint8)
    G.run_and_compare(w, src).close()


def test_layer_sub_range_and_mixed_ranges_in_one_plan():
    g = small_geom(num_layers=4)
    rng = np.random.default_rng(2)
    perm_s, perm_d = rng.permutation(96).astype(np.int32), rng.permutation(96).astype(np.int32)
    src_host = wl.host_pool_values(g, "bf16", 3)
    src, dst = G.device_pool_from_host(src_host), G.device_sentinel_pool(g)
    sp, dp = kvd.Pool(src.data_ptr(), g), kvd.Pool(dst.data_ptr(), g)
    plan = kvd.Plan(sp, dp, 4, 96)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())  # the pools were filled on torch's stream
    reqs = [(100, 0, 10, 1, 3), (50, 10, 14, 1, 3), (77, 14, 19, 0, 4), (16, 19, 20, 3, 4)]
    want = wl.host_pool_sentinel(g)
    for tokens, a, b, l0, l1 in reqs:
        plan.build_descriptors(perm_s[a:b], perm_d[a:b], tokens, l0, l1, s.cuda_stream)
        w = wl.Workload("r", g, g, [wl.Request(tokens, perm_s[a:b], perm_d[a:b])], "bf16", 0, l0, l1)
        tl.oracle_pull_workload(w, src_host, want)
    st = plan.stats(s.cuda_stream)
    assert st["num_requests"] == 4 and st["num_transactions"] == (6 + 4) + (3 + 4) + (4 + 4) + 1
    plan.pull(s.cuda_stream)
    s.synchronize()
    G.assert_bytes_equal(dst.cpu().numpy(), want, "mixed layer ranges")
    plan.close()


@pytest.mark.parametrize("gs,gd", [(small_geom(num_layers=5), small_geom(num_layers=5)),
                                   (small_geom(num_layers=5, kv_adjacent=True), small_geom(num_layers=5, kv_adjacent=True)),
                                   (small_geom(num_layers=5), small_geom(num_layers=5, layout=wl.BTHD, block_tokens=32, num_blocks=48))],
                         ids=["same", "kv-adjacent", "relayout"])
def test_pull_layer_by_layer_from_one_plan(gs, gd):
    """One plan, built once; its layers moved by separate kvd_pull_layers calls: after each call the
    destination holds exactly the layers moved so far; requests built for other layers sit out."""
    rng = np.random.default_rng(71)
    free_s, free_d = np.ones(gs.num_blocks, bool), np.ones(gd.num_blocks, bool)
    lens, ranges = [300, 77, 160], [(0, 5), (1, 3), (4, 5)]
    reqs = [wl.Request(t, wl.fragmented_allocation(rng, free_s, wl.blocks_for(t, gs.block_tokens), 4),
                       wl.fragmented_allocation(rng, free_d, wl.blocks_for(t, gd.block_tokens), 4)) for t in lens]
    src_host = rng.integers(0, 256, size=gs.total_bytes, dtype=np.uint8)
    src, dst = G.device_pool_from_host(src_host), G.device_sentinel_pool(gd)
    plan = kvd.Plan(kvd.Pool(src.data_ptr(), gs), kvd.Pool(dst.data_ptr(), gd), 3, 64)
    for r, (l0, l1) in zip(reqs, ranges):
        plan.build_descriptors(r.src_table, r.dst_table, r.seq_len, l0, l1)
    want = wl.host_pool_sentinel(gd)
    for (p0, p1) in [(2, 3), (0, 2), (3, 5)]:                           # out of order, two layers at a time too
        plan.pull_layers(p0, p1)
        torch.cuda.synchronize()
        for r, (l0, l1) in zip(reqs, ranges):
            a, b = max(l0, p0), min(l1, p1)
            if a < b:
                tl.oracle_pull_workload(wl.Workload("part", gs, gd, [r], "bf16", 0, a, b), src_host, want)
        G.assert_bytes_equal(dst.cpu().numpy(), want, f"after layers [{p0}, {p1})")
    with pytest.raises(kvd.KvdError):
        plan.pull_layers(3, 6)
    with pytest.raises(kvd.KvdError):
        plan.pull_layers(2, 2)
    plan.close()
    g_bm = small_geom(block_major=True)
    sp, dp = kvd.Pool(src.data_ptr(), g_bm), kvd.Pool(dst.data_ptr(), g_bm)
    with pytest.raises(kvd.KvdError):
        kvd.Plan(sp, dp, 1, 8).pull_layers(0, 1)


def test_layer_by_layer_pulls_recorded_into_one_hip_graph():
    """The launch-bound form of the transfer, one pull per layer, as one graph: each replay moves everything."""
    w = wl.config2(num_layers=8, pool_blocks=1024, tokens=3000)
    src_host = host_src(w)
    want = G.oracle_expected(w, src_host)
    src, dst = G.device_pool_from_host(src_host), G.device_sentinel_pool(w.dst)
    x = G.GpuTransfer(w, src, dst)
    x.build()
    x.stream.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=x.stream):
        for layer in range(8):
            x.plan.pull_layers(layer, layer + 1, x.stream.cuda_stream)
    for replay in range(3):
        dst.view(torch.int16).fill_(wl.SENTINEL16)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        G.assert_bytes_equal(dst.cpu().numpy(), want, f"replay {replay}")
    del graph
    x.close()


def test_completion_word():
    """kvd_complete behind a pull: once the word shows the request id, the pulled bytes are there -
    read by the host from pinned memory without synchronising the stream, and from device memory."""
    w = wl.config2(num_layers=4, pool_blocks=2048, tokens=8192)
    src_host = host_src(w)
    want = G.oracle_expected(w, src_host)
    src, dst = G.device_pool_from_host(src_host), G.device_sentinel_pool(w.dst)
    pinned = torch.zeros(2, dtype=torch.int64).pin_memory()
    on_device = torch.zeros(1, dtype=torch.int64, device="cuda")
    torch.cuda.synchronize()
    x = G.GpuTransfer(w, src, dst)
    sh = x.stream.cuda_stream
    for request_id in (41, 42):
        dst.view(torch.int16).fill_(wl.SENTINEL16)
        x.after_torch()
        x.plan.reset()
        x.build()
        x.pull()
        kvd.kvd_complete(pinned.data_ptr(), request_id, sh)
        kvd.kvd_complete(on_device.data_ptr(), request_id + 100, sh)
        peer = torch.cuda.Stream()              # a reader that synchronises with nothing but the word
        import time
        t0 = time.time()
        while int(pinned[0]) != request_id:
            assert time.time() - t0 < 20, "the completion word never arrived"
        with torch.cuda.stream(peer):
            got = dst.clone()
        peer.synchronize()
        G.assert_bytes_equal(got.cpu().numpy(), want, f"after completion word {request_id}")
        x.stream.synchronize()
        assert int(on_device[0]) == request_id + 100
    host_only = np.zeros(1, np.int64)
    for bad in (0, pinned.data_ptr() + 4, host_only.ctypes.data):
        with pytest.raises(kvd.KvdError):
            kvd.kvd_complete(bad, 1, sh)
    x.close()


def _request_words(w, request, g):
    """Indices of the 16-bit words of the destination pool (as [layer][kv][block][words of a block]) that
    one request's blocks cover, as a boolean mask over blocks."""
    mask = np.zeros(g.num_blocks, bool)
    mask[request.dst_table[:wl.blocks_for(request.seq_len, g.block_tokens)]] = True
    return mask


@pytest.mark.parametrize("min_tokens", [0, 1500, 1 << 30])
def test_per_request_completion_inside_one_batched_pull(min_tokens):
    """kvd_pull_notify: every request of a batch gets its own completion word (section 4.2).  The descriptor
    list is the oracle's merge of each request's reads by itself (merging stops at a completion); a reader
    that waits for word k only, without synchronising any stream, finds request k's bytes equal to the
    oracle's; at the end the whole pool equals the oracle's.  min_tokens: requests announced one by one, in
    launches of at least 1500 tokens, or all together (kvd_plan_set_completion_granularity)."""
    import time
    w = wl.config3(num_layers=4, num_requests=24, median=700.0, hi=4096)
    g = w.dst
    src_host = host_src(w)
    want = G.oracle_expected(w, src_host)
    src, dst = G.device_pool_from_host(src_host), G.device_sentinel_pool(g)
    x = G.GpuTransfer(w, src, dst, kvd.KVD_PLAN_COMPLETE_PER_REQUEST)
    x.plan.set_completion_granularity(min_tokens)
    sh = x.stream.cuda_stream
    x.build(batch=True)
    got_desc = x.plan.descriptors(sh)
    s_t, d_t = tl.oracle_tensors(w.src, None)[0], tl.oracle_tensors(w.dst, None)[0]
    per_request = [orc.coalesce(orc.request_transactions(s_t, d_t, 0, r.src_table, r.dst_table, r.seq_len)) for r in w.requests]
    assert np.array_equal(got_desc, np.concatenate(per_request))
    n = len(w.requests)
    words = torch.zeros(n, dtype=torch.int64).pin_memory()
    want5 = torch.from_numpy(want).view(torch.int16).view(g.num_layers, 2, g.num_blocks, -1)
    dst5 = dst.view(torch.int16).view(g.num_layers, 2, g.num_blocks, -1)
    peer = torch.cuda.Stream()  # the reader's stream: ordered behind nothing but what the reader has seen in the words
    for value in (7, 8):       # twice: the second time with the words holding the first value
        dst.view(torch.int16).fill_(wl.SENTINEL16)
        x.after_torch()
        x.plan.pull_notify(words.data_ptr(), value, sh)
        seen_at = {}
        t0 = time.time()
        pending = set(range(n))
        while pending:
            assert time.time() - t0 < 30, f"completion words of requests {sorted(pending)} never arrived"
            for k in sorted(pending):
                if int(words[k]) == value:
                    seen_at[k] = time.time() - t0
                    pending.discard(k)
                    idx = torch.from_numpy(np.nonzero(_request_words(w, w.requests[k], g))[0]).cuda()
                    with torch.cuda.stream(peer):
                        got = dst5[:, :, idx].clone()
                    peer.synchronize()
                    assert torch.equal(got.cpu(), want5[:, :, idx.cpu()]), f"request {k} after its completion word"
        x.stream.synchronize()
        G.assert_bytes_equal(dst.cpu().numpy(), want, f"whole pool after pull_notify (value {value})")
        say(f"pull_notify value {value}: first word after {min(seen_at.values()) * 1e3:.2f} ms, last after {max(seen_at.values()) * 1e3:.2f} ms")
    # the plain pull of such a plan moves the same bytes
    dst.view(torch.int16).fill_(wl.SENTINEL16)
    x.after_torch()
    x.pull()
    x.stream.synchronize()
    G.assert_bytes_equal(dst.cpu().numpy(), want, "kvd_pull of a plan with per-request completion")
    # refusals
    y = G.GpuTransfer(w, src, dst)
    y.build(batch=True)
    with pytest.raises(kvd.KvdError) as e:
        y.plan.pull_notify(words.data_ptr(), 1, sh)
    assert e.value.code == kvd.KVD_ERR_MISMATCH
    y.close()
    host_only = np.zeros(n, np.int64)
    for bad in (0, words.data_ptr() + 4, host_only.ctypes.data):
        with pytest.raises(kvd.KvdError):
            x.plan.pull_notify(bad, 1, sh)
    x.close()


def test_per_request_completion_recorded_into_a_hip_graph():
    """kvd_pull_notify forks to its side streams and joins again, so a recording stream records all of it: three
    replays with eager fills between them, each checked against the oracle and for its words."""
    w = wl.config3(num_layers=2, num_requests=9, median=300.0, hi=2048)
    src_host = host_src(w)
    want = G.oracle_expected(w, src_host)
    src, dst = G.device_pool_from_host(src_host), G.device_sentinel_pool(w.dst)
    x = G.GpuTransfer(w, src, dst, kvd.KVD_PLAN_COMPLETE_PER_REQUEST)
    x.build(batch=True)
    words = torch.zeros(len(w.requests), dtype=torch.int64, device="cuda")
    x.plan.pull_notify(words.data_ptr(), 5, x.stream.cuda_stream)  # eager first: the side streams exist before the recording
    x.stream.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=x.stream):
        x.plan.pull_notify(words.data_ptr(), 6, x.stream.cuda_stream)
    for replay in range(3):
        dst.view(torch.int16).fill_(wl.SENTINEL16)
        words.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert words.tolist() == [6] * len(w.requests), f"replay {replay}"
        G.assert_bytes_equal(dst.cpu().numpy(), want, f"replay {replay}")
    del graph
    x.close()


@pytest.mark.parametrize("min_tokens", [0, 100, 3000])
def test_per_request_completion_with_more_requests_than_one_build_launch_takes(min_tokens):
    """701 short requests: two launches of the build kernel, whose per-request tables continue each other; after a
    reset the same plan takes a smaller batch.  With min_tokens = 3000 a launch announces about 85 requests, more than
    a wave has lanes."""
    g = wl.PoolGeometry(2, 4096, 16, 2, 64, 2, wl.BHTD)
    rng = np.random.default_rng(13)
    free_s, free_d = np.ones(4096, bool), np.ones(4096, bool)
    reqs = []
    for _ in range(701):
        t = int(rng.integers(1, 70))
        n = wl.blocks_for(t, 16)
        reqs.append(wl.Request(t, wl.fragmented_allocation(rng, free_s, n, 4), wl.fragmented_allocation(rng, free_d, n, 4)))
    w = wl.Workload("many-notify", g, g, reqs, "bf16", 13)
    src_host = host_src(w)
    src, dst = G.device_pool_from_host(src_host), G.device_sentinel_pool(g)
    x = G.GpuTransfer(w, src, dst, kvd.KVD_PLAN_COMPLETE_PER_REQUEST)
    x.plan.set_completion_granularity(min_tokens)
    sh = x.stream.cuda_stream
    x.build(batch=True)
    s_t, d_t = tl.oracle_tensors(g, None)[0], tl.oracle_tensors(g, None)[0]
    per_request = [orc.coalesce(orc.request_transactions(s_t, d_t, 0, r.src_table, r.dst_table, r.seq_len)) for r in reqs]
    assert np.array_equal(x.plan.descriptors(sh), np.concatenate(per_request))
    words = torch.zeros(701, dtype=torch.int64, device="cuda")
    torch.cuda.synchronize()
    x.plan.pull_notify(words.data_ptr(), 3, sh)
    x.stream.synchronize()
    assert int((words != 3).sum()) == 0
    G.assert_bytes_equal(dst.cpu().numpy(), G.oracle_expected(w, src_host), "701 requests, per-request completion")
    # the same plan again with the first 40 requests only
    w2 = wl.Workload("fewer", g, g, reqs[:40], "bf16", 13)
    dst.view(torch.int16).fill_(wl.SENTINEL16)
    words.zero_()
    x.after_torch()
    x.plan.reset()
    x.plan.build_descriptors_batch([r.src_table for r in reqs[:40]], [r.dst_table for r in reqs[:40]], [r.seq_len for r in reqs[:40]], 0, 2, sh)
    x.plan.pull_notify(words.data_ptr(), 4, sh)
    x.stream.synchronize()
    assert words.tolist() == [4] * 40 + [0] * 661
    G.assert_bytes_equal(dst.cpu().numpy(), G.oracle_expected(w2, src_host), "40 requests after a reset")
    x.close()


@pytest.mark.parametrize("min_tokens", [0, 400])
@pytest.mark.parametrize("kind", ["mixed-layers", "block-major", "ragged-relayout"])
def test_per_request_completion_other_plan_kinds(kind, min_tokens):
    """Requests built one call at a time with different layer ranges, block-major pools (layers folded, wide
    expansion) and a re-layout plan: device-memory words, whole pool against the oracle.  With min_tokens = 400
    neighbouring requests share a launch where they move the same layers."""
    rng = np.random.default_rng(17)
    if kind == "block-major":
        gs = gd = small_geom(block_major=True, num_blocks=256, num_layers=4)
    elif kind == "ragged-relayout":
        gs, gd = small_geom(num_blocks=256), small_geom(num_blocks=128, block_tokens=32, layout=wl.BTHD)
    else:
        gs = gd = small_geom(num_blocks=256, num_layers=5)
    free_s, free_d = np.ones(gs.num_blocks, bool), np.ones(gd.num_blocks, bool)
    lens = [333, 16, 1, 700, 64]
    ranges = [(0, gs.num_layers)] * 5 if kind != "mixed-layers" else [(0, 5), (1, 3), (1, 3), (4, 5), (0, 5)]
    reqs = [wl.Request(t, wl.fragmented_allocation(rng, free_s, wl.blocks_for(t, gs.block_tokens), 4),
                       wl.fragmented_allocation(rng, free_d, wl.blocks_for(t, gd.block_tokens), 4)) for t in lens]
    src_host = rng.integers(0, 256, size=gs.total_bytes, dtype=np.uint8)
    want = wl.host_pool_sentinel(gd)
    for r, (l0, l1) in zip(reqs, ranges):
        tl.oracle_pull_workload(wl.Workload("one", gs, gd, [r], "bf16", 0, l0, l1), src_host, want)
    src, dst = G.device_pool_from_host(src_host), G.device_sentinel_pool(gd)
    plan = kvd.Plan(kvd.Pool(src.data_ptr(), gs), kvd.Pool(dst.data_ptr(), gd), 5, 512, kvd.KVD_PLAN_COMPLETE_PER_REQUEST)
    plan.set_completion_granularity(min_tokens)
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    for r, (l0, l1) in zip(reqs, ranges):
        plan.build_descriptors(r.src_table, r.dst_table, r.seq_len, l0, l1, stream.cuda_stream)
    words = torch.zeros(5, dtype=torch.int64, device="cuda")
    torch.cuda.synchronize()
    plan.pull_notify(words.data_ptr(), 99, stream.cuda_stream)
    stream.synchronize()
    assert words.tolist() == [99] * 5
    G.assert_bytes_equal(dst.cpu().numpy(), want, kind)
    G.assert_bytes_equal(src.cpu().numpy(), src_host, kind + ": source changed")
    plan.close()


def test_merge_across_requests_as_in_queue_example():
    # R1 reads block 0 into 5, R2 reads 1 into 6 (+ 3 into 9): first two merge (section 4.2)
    g = small_geom(num_layers=1)
    src_host = wl.host_pool_values(g, "bf16", 4)
    w = wl.Workload("queue", g, g, [wl.Request(16, np.array([0], np.int32), np.array([5], np.int32)),
                                    wl.Request(32, np.array([1, 3], np.int32), np.array([6, 9], np.int32))],
                    "bf16", 4)
    x = G.run_and_compare(w, src_host)
    d = x.plan.descriptors(x.stream.cuda_stream)
    tile = g.tile_elems * 2
    assert d.tolist() == [[0, 5 * tile, 2 * tile], [3 * tile, 9 * tile, tile]]
    assert np.array_equal(d, tl.oracle_plan_descriptors(w, 0, 0))
    x.close()


def test_requests_with_different_layers_do_not_merge():
    g = small_geom(num_layers=2)
    src_host = wl.host_pool_values(g, "bf16", 4)
    src, dst = G.device_pool_from_host(src_host), G.device_sentinel_pool(g)
    plan = kvd.Plan(kvd.Pool(src.data_ptr(), g), kvd.Pool(dst.data_ptr(), g), 2, 8)
    plan.build_descriptors([0], [5], 16, 0, 2)
    plan.build_descriptors([1], [6], 16, 1, 2)   # continues the first on both sides, but other layers
    plan.pull()
    torch.cuda.synchronize()
    assert plan.stats()["num_descriptors"] == 2
    want = wl.host_pool_sentinel(g)
    tl.oracle_pull_workload(wl.Workload("a", g, g, [wl.Request(16, np.array([0], np.int32), np.array([5], np.int32))], "bf16", 0), src_host, want)
    tl.oracle_pull_workload(wl.Workload("b", g, g, [wl.Request(16, np.array([1], np.int32), np.array([6], np.int32))], "bf16", 0, 1, 2), src_host, want)
    G.assert_bytes_equal(dst.cpu().numpy(), want, "different layers")
    plan.close()


@pytest.mark.parametrize("w", [wl.config2(num_layers=2, pool_blocks=1024, tokens=3000),
                               wl.config5(num_layers=2, src_pool_blocks=256, tokens=1500),
                               wl.config4(num_layers=3, pool_blocks=8192, tokens=48000),   # 3000 descriptors: two LDS windows
                               wl.config3(num_layers=2, num_requests=16, median=256.0, hi=2048)], ids=lambda w: w.name)
def test_persistent_grid_form_gives_the_same_bytes(w):
    x = G.run_and_compare(w, host_src(w), flags=kvd.KVD_PLAN_PERSISTENT)
    if w.name.startswith("cfg4"):
        assert x.plan.stats(x.stream.cuda_stream)["num_descriptors"] == 3000
    x.close()


def test_region_ordering_of_short_scattered_transactions():
    """Enough lone small blocks for the pull to group its work items by destination region first."""
    g = wl.PoolGeometry(16, 65536, 16, 1, 8, 2, wl.BHTD)        # 256-byte blocks, 16 MiB slabs
    rng = np.random.default_rng(41)
    n = 4096
    st, dt = wl.scattered_table(rng, g.num_blocks, n), wl.scattered_table(rng, g.num_blocks, n)
    big = wl.Request(n * 16 - 5, st, dt)
    extra = wl.Request(40, np.array([5, 9, 11], np.int32), np.setdiff1d(np.arange(g.num_blocks), dt)[:3].astype(np.int32))
    w = wl.Workload("ordered", g, g, [big, extra], "bf16", 41)
    src_host = host_src(w)
    src, dst = G.device_pool_from_host(src_host), G.device_sentinel_pool(g)
    x = G.GpuTransfer(w, src, dst)
    sh = x.stream.cuda_stream
    x.plan.build_descriptors(big.src_table, big.dst_table, big.seq_len, 0, g.num_layers, sh)
    x.pull()
    x.stream.synchronize()
    stt = x.plan.stats(sh)
    assert stt["num_work_items"] == n == stt["num_descriptors"] and stt["work_order"] == kvd.KVD_ORDER_REGIONS
    want = wl.host_pool_sentinel(g)
    tl.oracle_pull_workload(wl.Workload("big", g, g, [big], "bf16", 0), src_host, want)
    G.assert_bytes_equal(dst.cpu().numpy(), want, "region-ordered pull")
    # the ablation flag keeps the queue order and moves the same bytes
    dst2 = G.device_sentinel_pool(g)
    wq = wl.Workload("queue-order", g, g, [big], "bf16", 41)
    y = G.GpuTransfer(wq, src, dst2, flags=kvd.KVD_PLAN_QUEUE_ORDER).run()
    G.assert_bytes_equal(dst2.cpu().numpy(), want, "queue-order pull")
    assert y.plan.stats(y.stream.cuda_stream)["work_order"] == kvd.KVD_ORDER_QUEUE
    y.close()
    # appending to the plan re-orders on the next pull; a second pull reuses the order
    x.plan.build_descriptors(extra.src_table, extra.dst_table, extra.seq_len, 0, g.num_layers, sh)
    x.pull(); x.pull()
    x.stream.synchronize()
    tl.oracle_pull_workload(wl.Workload("extra", g, g, [extra], "bf16", 0), src_host, want)
    G.assert_bytes_equal(dst.cpu().numpy(), want, "after appending")
    x.close()


@pytest.mark.parametrize("case", ["lone-16KiB", "lone-16KiB-two-sort-chunks", "mixed-runs", "partial-heads",
                                  "block-major-wide", "batch-per-request", "no-coalesce", "long-after-all", "mostly-long"])
def test_descriptor_sort_of_lone_medium_blocks(case):
    """Descriptors of four to eight work items are sorted by destination address before the pull
    (KVD_PLAN_DESTINATION_ORDER asks for it at any size): the bytes moved and the descriptor list stay the oracle's.
    Covered: 16 and 32 KiB lone blocks, more descriptors than are sorted together (8192), lone blocks mixed with
    short runs, a partial last block split per head, 48-bit offsets, several requests in one plan (the ordering is
    left out by kvd_pull_notify and redone after an append), and the same through kvd_pull_noalloc."""
    flags = kvd.KVD_PLAN_DESTINATION_ORDER
    rng = np.random.default_rng(len(case))
    if case == "lone-16KiB":
        g = wl.PoolGeometry(2, 4096, 64, 1, 128, 2, wl.BHTD)            # 16 KiB per block and slab: 4 work items
        reqs = [wl.Request(700 * 64 - 9, wl.scattered_table(rng, 4096, 700), wl.scattered_table(rng, 4096, 700))]
    elif case == "lone-16KiB-two-sort-chunks":
        g = wl.PoolGeometry(1, 9600, 64, 1, 128, 2, wl.BHTD)            # 9000 descriptors: more than are sorted together
        reqs = [wl.Request(9000 * 64, wl.scattered_table(rng, 9600, 9000), wl.scattered_table(rng, 9600, 9000))]
    elif case == "mixed-runs":
        g = wl.PoolGeometry(2, 4096, 16, 4, 128, 2, wl.BHTD)            # 16 KiB blocks; runs of 1 and 2 (4 and 8 work items)
        free_s, free_d = np.ones(4096, bool), np.ones(4096, bool)
        reqs = [wl.Request(500 * 16, wl.fragmented_allocation(rng, free_s, 500, 2), wl.fragmented_allocation(rng, free_d, 500, 2))]
    elif case == "partial-heads":
        g = wl.PoolGeometry(2, 2048, 64, 4, 64, 2, wl.BHTD)             # 32 KiB blocks, tail of 5 tokens: 4 pieces of 640 B
        reqs = [wl.Request(300 * 64 + 5, wl.scattered_table(rng, 2048, 301), wl.scattered_table(rng, 2048, 301))]
    elif case == "block-major-wide":
        g = wl.PoolGeometry(1, 3000, 16, 2, 128, 2, wl.BHTD, block_major=True)  # 16 KiB per block over K and V
        flags |= kvd.KVD_PLAN_WIDE_OFFSETS
        reqs = [wl.Request(1000 * 16, wl.scattered_table(rng, 3000, 1000), wl.scattered_table(rng, 3000, 1000))]
    elif case == "batch-per-request":
        g = wl.PoolGeometry(2, 4096, 64, 1, 128, 2, wl.BHTD)
        flags |= kvd.KVD_PLAN_COMPLETE_PER_REQUEST
        free_s, free_d = np.ones(4096, bool), np.ones(4096, bool)
        reqs = []
        for n in (300, 1, 40, 500):
            reqs.append(wl.Request(n * 64 - 1, wl.fragmented_allocation(rng, free_s, n, 1), wl.fragmented_allocation(rng, free_d, n, 1)))
    elif case == "mostly-long":
        # lone blocks and runs of up to six: less than three quarters of the work sits in short pieces, the queue order stays
        g = wl.PoolGeometry(2, 4096, 16, 4, 128, 2, wl.BHTD)
        free_s, free_d = np.ones(4096, bool), np.ones(4096, bool)
        reqs = [wl.Request(700 * 16, wl.fragmented_allocation(rng, free_s, 700, 6), wl.fragmented_allocation(rng, free_d, 700, 6))]
    elif case == "no-coalesce":
        g = wl.PoolGeometry(2, 4096, 64, 1, 128, 2, wl.BHTD)            # lone 16 KiB blocks, nothing to merge either way
        flags |= kvd.KVD_PLAN_NO_COALESCE
        reqs = [wl.Request(600 * 64, wl.fixed_run_table(rng, 4096, 600, 1), wl.fixed_run_table(rng, 4096, 600, 1))]
    else:
        # blocks of 64 and 128 tokens: the host expects one descriptor per 16 KiB piece, but the tables are two
        # straight stretches, everything merges into two descriptors, and the device keeps the queue order after all
        g = wl.PoolGeometry(2, 1024, 64, 1, 128, 2, wl.BTHD)
        gd = wl.PoolGeometry(2, 512, 128, 1, 128, 2, wl.BTHD)
        reqs = [wl.Request(400 * 64, np.concatenate([np.arange(300, 500), np.arange(100, 300)]).astype(np.int32),
                           np.concatenate([np.arange(150, 250), np.arange(50, 150)]).astype(np.int32))]
    gd = gd if case == "long-after-all" else g
    w = wl.Workload(case, g, gd, reqs, "bf16", 77)
    src_host = host_src(w)
    want = G.oracle_expected(w, src_host)
    src, dst = G.device_pool_from_host(src_host), G.device_sentinel_pool(gd)
    x = G.GpuTransfer(w, src, dst, flags)
    sh = x.stream.cuda_stream
    # all but the last request, a pull, then the last one appended and two more pulls
    for r in reqs[:-1]:
        x.plan.build_descriptors(r.src_table, r.dst_table, r.seq_len, 0, g.num_layers, sh)
    x.pull()
    r = reqs[-1]
    x.plan.build_descriptors(r.src_table, r.dst_table, r.seq_len, 0, g.num_layers, sh)
    x.pull()
    x.pull()
    x.stream.synchronize()
    G.assert_bytes_equal(dst.cpu().numpy(), want, case)
    st = x.plan.stats(sh)
    if case == "long-after-all":
        assert st["num_descriptors"] == 2 and st["num_work_items"] == 1600 and st["work_order"] == kvd.KVD_ORDER_QUEUE, st
    elif case == "mostly-long":
        assert st["work_order"] == kvd.KVD_ORDER_QUEUE, st
    else:
        assert 4 * st["num_descriptors"] <= st["num_work_items"] <= 8 * st["num_descriptors"], st
        assert st["work_order"] == kvd.KVD_ORDER_SORTED, st
    if case == "batch-per-request":
        dst.view(torch.int16).fill_(wl.SENTINEL16)
        words = torch.zeros(len(reqs), dtype=torch.int64, device="cuda")
        x.after_torch()
        x.plan.pull_notify(words.data_ptr(), 5, sh)
        x.stream.synchronize()
        assert words.tolist() == [5] * len(reqs)
        G.assert_bytes_equal(dst.cpu().numpy(), want, case + ", request by request")
    elif not g.block_major:
        s_t, d_t = tl.oracle_tensors(g, None)[0], tl.oracle_tensors(gd, None)[0]
        q = np.concatenate([orc.request_transactions(s_t, d_t, 0, r.src_table, r.dst_table, r.seq_len) for r in reqs])
        assert np.array_equal(x.plan.descriptors(sh), q if case == "no-coalesce" else orc.coalesce(q))  # still in queue order
    x.close()
    if len(reqs) == 1 and not (flags & kvd.KVD_PLAN_WIDE_OFFSETS) and len(reqs[0].src_table) <= kvd.KVD_NOALLOC_MAX_BLOCKS:
        dst.view(torch.int16).fill_(wl.SENTINEL16)
        torch.cuda.synchronize()
        kvd.kvd_pull_noalloc(kvd.pool_desc(src.data_ptr(), g), kvd.pool_desc(dst.data_ptr(), gd), reqs[0].src_table, reqs[0].dst_table,
                             reqs[0].seq_len, 0, g.num_layers, flags, 0)
        torch.cuda.synchronize()
        G.assert_bytes_equal(dst.cpu().numpy(), want, case + " through kvd_pull_noalloc")


@pytest.mark.parametrize("kind", ["runs", "short-scattered", "medium-scattered"])
def test_pull_recorded_into_a_hip_graph(kind):
    """kvd_pull inside a HIP graph: every replay moves the plan's bytes, also for plans whose work
    items are grouped by region or whose descriptors are sorted by destination first (those launches
    are then part of the graph); an eager pull between recording and the first replay is right as
    well; builds refuse to be recorded."""
    flags = 0
    if kind == "runs":
        w = wl.config2(num_layers=2, pool_blocks=2048, tokens=5000)
    elif kind == "medium-scattered":
        g = wl.PoolGeometry(2, 4096, 64, 1, 128, 2, wl.BHTD)  # lone 16 KiB blocks
        rng = np.random.default_rng(44)
        flags = kvd.KVD_PLAN_DESTINATION_ORDER
        w = wl.Workload("graph-medium", g, g, [wl.Request(900 * 64 - 7, wl.scattered_table(rng, 4096, 900),
                                                          wl.scattered_table(rng, 4096, 900))], "bf16", 44)
    else:
        g = wl.PoolGeometry(16, 65536, 16, 1, 8, 2, wl.BHTD)
        rng = np.random.default_rng(43)
        w = wl.Workload("graph-short", g, g, [wl.Request(4096 * 16 - 5, wl.scattered_table(rng, g.num_blocks, 4096),
                                                         wl.scattered_table(rng, g.num_blocks, 4096))], "bf16", 43)
    src_host = host_src(w)
    want = G.oracle_expected(w, src_host)
    src, dst = G.device_pool_from_host(src_host), G.device_sentinel_pool(w.dst)
    x = G.GpuTransfer(w, src, dst, flags)
    x.build()
    x.stream.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=x.stream):
        x.plan.pull(x.stream.cuda_stream)
        with pytest.raises(kvd.KvdError):
            r = w.requests[0]
            x.plan.build_descriptors(r.src_table, r.dst_table, r.seq_len, 0, 1, x.stream.cuda_stream)
    torch.cuda.synchronize()
    assert int((dst.view(torch.int16) != wl.SENTINEL16).sum()) == 0     # recording moved nothing
    x.pull()                                                             # eager, before any replay
    x.stream.synchronize()
    G.assert_bytes_equal(dst.cpu().numpy(), want, "eager pull after recording")
    for replay in range(3):
        dst.view(torch.int16).fill_(wl.SENTINEL16)                       # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        G.assert_bytes_equal(dst.cpu().numpy(), want, f"replay {replay}")
    del graph
    x.close()


def test_many_transactions_and_one_long_run():
    # 16-byte rows, one head: 10000 lone blocks -> several passes of the coalescing workgroup
    g = wl.PoolGeometry(2, 20000, 16, 1, 8, 2, wl.BHTD)
    rng = np.random.default_rng(6)
    st = wl.scattered_table(rng, g.num_blocks, 10000)
    dt = wl.scattered_table(rng, g.num_blocks, 10000)
    w = wl.Workload("groups", g, g, [wl.Request(10000 * 16 - 3, st, dt)], "bf16", 6)
    x = G.run_and_compare(w, host_src(w))
    st_ = x.plan.stats(x.stream.cuda_stream)
    assert st_["num_descriptors"] == 10000 == st_["num_work_items"]
    x.close()
    # the same as one long contiguous run: everything merges into a single descriptor
    ident = np.arange(10000, dtype=np.int32)
    w2 = wl.Workload("groups-contig", g, g, [wl.Request(10000 * 16, ident, ident + 5000)], "bf16", 6)
    x = G.run_and_compare(w2, host_src(w2))
    st_ = x.plan.stats(x.stream.cuda_stream)
    assert st_["num_descriptors"] == 1 and st_["num_work_items"] == 10000 * 256 // 4096
    x.close()


def _strides(kind, g):
    tile = g.tile_elems
    if kind == "padded":          # layers outermost, blocks padded to 3 tiles, V half a tile behind K
        sb, skv = 3 * tile, tile + tile // 2
        return g.num_blocks * sb, skv, sb
    if kind == "block-major":     # [block][layer][kv]: every block holds all its layers
        return 2 * tile, tile, 2 * g.num_layers * tile
    if kind == "block-major-padded":  # the same with a tile of padding behind every block: blocks never touch
        return 2 * tile, tile, 2 * g.num_layers * tile + tile
    if kind == "block-major-loose":   # [block][layer][kv] with a gap between a block's layers: only K and V touch
        return 3 * tile, tile, 3 * g.num_layers * tile
    if kind == "kv-outermost":    # [kv][layer][block]
        return g.num_blocks * tile, g.num_layers * g.num_blocks * tile, tile
    raise ValueError(kind)


@pytest.mark.parametrize("kind_src,kind_dst", [("padded", "padded"), ("block-major", "block-major"),
                                               ("kv-outermost", "block-major"), ("block-major", "padded"),
                                               ("block-major-padded", "block-major"),
                                               ("block-major-loose", "block-major-loose"),
                                               ("block-major", "block-major-loose")])
def test_pools_described_only_by_their_strides(kind_src, kind_dst):
    g = small_geom(num_layers=2, num_blocks=32)
    rng = np.random.default_rng(8)
    from oracle import kvd_oracle as orc

    def tensors(buf, strides):
        sl, skv, sb = strides
        return [orc.Tensor(buf, layer * sl * 2, [orc.KV, orc.B, orc.H, orc.L, orc.D],
                           [2, 32, 4, 16, 64], [skv, sb, 16 * 64, 64, 1], 2) for layer in range(2)]

    def extent(strides):
        sl, skv, sb = strides
        return (sl + skv + 31 * sb + g.tile_elems) * 2

    ss, ds = _strides(kind_src, g), _strides(kind_dst, g)
    src_host = wl.normal_bits(rng, extent(ss) // 2, "bf16").view(np.uint8)
    want = np.full(extent(ds) // 2, wl.SENTINEL16, np.uint16).view(np.uint8)
    st, dt = rng.permutation(32)[:7].astype(np.int32), rng.permutation(32)[:7].astype(np.int32)
    orc.pull(tensors(src_host, ss), tensors(want, ds), 0, 2, st, dt, 100)
    src, dst = G.device_pool_from_host(src_host), G.device_pool_from_host(want.copy())
    dst.view(torch.int16).fill_(wl.SENTINEL16)
    plan = kvd.Plan(kvd.Pool(src.data_ptr(), g, *ss), kvd.Pool(dst.data_ptr(), g, *ds), 1, 8)
    plan.build_descriptors(st, dt, 100, 0, 2)
    plan.pull()
    torch.cuda.synchronize()
    G.assert_bytes_equal(dst.cpu().numpy(), want, f"{kind_src} -> {kind_dst}")
    plan.close()


def test_plan_reuse_reset_repeat_and_round_trip():
    w = wl.config5(num_layers=2, src_pool_blocks=128, tokens=777)
    src_host = host_src(w)
    src, mid = G.device_pool_from_host(src_host), G.device_sentinel_pool(w.dst)
    x = G.GpuTransfer(w, src, mid).run()
    want = G.oracle_expected(w, src_host)
    G.assert_bytes_equal(mid.cpu().numpy(), want, "first pull")
    x.pull(); x.pull()                      # a pull is idempotent
    x.stream.synchronize()
    G.assert_bytes_equal(mid.cpu().numpy(), want, "repeated pull")
    # reset and reuse the plan for another request with other tables
    x.plan.reset()
    assert x.plan.stats(x.stream.cuda_stream)["num_requests"] == 0
    mid.view(torch.int16).fill_(wl.SENTINEL16)
    x.after_torch()
    r = w.requests[0]
    w2 = wl.Workload("again", w.src, w.dst, [wl.Request(300, r.src_table[::-1].copy(), r.dst_table[::-1].copy())], "bf16", 0)
    x.w = w2
    x.run()
    G.assert_bytes_equal(mid.cpu().numpy(), G.oracle_expected(w2, src_host), "after reset")
    x.close()
    # round trip: pull back through the inverse mapping restores the valid tokens of the source
    back = G.device_sentinel_pool(w.src)
    wb = wl.Workload("back", w.dst, w.src, [wl.Request(300, w2.requests[0].dst_table, w2.requests[0].src_table)], "bf16", 0)
    y = G.GpuTransfer(wb, mid, back).run()
    b = back.cpu().numpy().view(np.uint16)
    touched = b != wl.SENTINEL16
    assert np.count_nonzero(touched) == 300 * 2 * 2 * 8 * 128
    assert np.array_equal(b[touched], src_host.view(np.uint16)[touched])
    y.close()


@pytest.mark.parametrize("block_major", [False, True])
def test_one_plan_reused_for_a_hundred_random_batches(block_major):
    """reset / build / pull on one plan object a hundred times with different requests each time
    (single calls, batches, appended requests with other layer ranges); the destination pool, which
    keeps what earlier rounds wrote, is compared with the oracle's after every round."""
    g = wl.PoolGeometry(3, 512, 16, 2, 64, 2, wl.BHTD, block_major=block_major)
    rng = np.random.default_rng(1234)
    src_host = rng.integers(0, 256, size=g.total_bytes, dtype=np.uint8)
    want = wl.host_pool_sentinel(g)
    src, dst = G.device_pool_from_host(src_host), G.device_sentinel_pool(g)
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    sh = stream.cuda_stream
    plan = kvd.Plan(kvd.Pool(src.data_ptr(), g), kvd.Pool(dst.data_ptr(), g), 4, 512)
    for it in range(100):
        plan.reset()
        free_s, free_d = np.ones(512, bool), np.ones(512, bool)
        n_req = int(rng.integers(1, 5))
        lens = [int(rng.integers(1, 1800)) for _ in range(n_req)]
        reqs = [wl.Request(t, wl.fragmented_allocation(rng, free_s, wl.blocks_for(t, 16), 6),
                           wl.fragmented_allocation(rng, free_d, wl.blocks_for(t, 16), 6)) for t in lens]
        if rng.random() < 0.5:
            ranges = [(0, 3)] * n_req
            plan.build_descriptors_batch([r.src_table for r in reqs], [r.dst_table for r in reqs], lens, 0, 3, sh)
        else:
            ranges = []
            for r in reqs:
                l0 = int(rng.integers(0, 3))
                ranges.append((l0, int(rng.integers(l0 + 1, 4))))
                plan.build_descriptors(r.src_table, r.dst_table, r.seq_len, ranges[-1][0], ranges[-1][1], sh)
        plan.pull(sh)
        for r, (l0, l1) in zip(reqs, ranges):
            tl.oracle_pull_workload(wl.Workload("one", g, g, [r], "bf16", 0, l0, l1), src_host, want)
        stream.synchronize()
        G.assert_bytes_equal(dst.cpu().numpy(), want, f"round {it}")
    plan.close()


def test_two_host_threads_with_their_own_plans():
    """Handles are for one thread at a time, the library is not: two threads, each with its own pools, plan and stream,
    create, build, pull, check and release side by side (the handle list and the error text are the shared state)."""
    import threading
    errors = []

    def worker(seed):
        try:
            w = wl.config2(num_layers=2, pool_blocks=512, tokens=777 + 100 * seed)
            src_host = host_src(w, seed=seed)
            want = G.oracle_expected(w, src_host)
            src = G.device_pool_from_host(src_host)
            stream = torch.cuda.Stream()
            for i in range(40):
                dst = G.device_sentinel_pool(w.dst)
                x = G.GpuTransfer(w, src, dst, kvd.KVD_PLAN_DESTINATION_ORDER if i % 2 else 0, stream=stream)
                x.run()
                with pytest.raises(kvd.KvdError) as e:  # this thread's own error text
                    x.plan.pull_layers(5 + seed, 4, stream.cuda_stream)
                assert f"[{5 + seed}, 4)" in str(e.value)
                G.assert_bytes_equal(dst.cpu().numpy(), want, f"thread {seed}, round {i}")
                x.close()
        except BaseException as exc:  # noqa: BLE001 - reported by the main thread
            errors.append((seed, repr(exc)))

    threads = [threading.Thread(target=worker, args=(k,)) for k in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors


def test_plans_give_back_what_they_allocate():
    """300 plans created, built, pulled (with per-request completion: side streams and events too) and released:
    the device's free memory ends where it started."""
    w = wl.config2(num_layers=2, pool_blocks=512, tokens=1000)
    src_host = host_src(w)
    src, dst = G.device_pool_from_host(src_host), G.device_sentinel_pool(w.dst)
    words = torch.zeros(1, dtype=torch.int64, device="cuda")
    stream = torch.cuda.Stream()  # one for all plans: torch's own stream pool grows with every new stream up to 32

    def cycle(n):
        for i in range(n):
            x = G.GpuTransfer(w, src, dst, kvd.KVD_PLAN_COMPLETE_PER_REQUEST if i % 2 else kvd.KVD_PLAN_DESTINATION_ORDER,
                              stream=stream)
            x.build()
            if i % 2:
                x.plan.pull_notify(words.data_ptr(), i + 1, x.stream.cuda_stream)
            else:
                x.pull()
            x.stream.synchronize()
            x.close()
        torch.cuda.synchronize()
    cycle(20)  # whatever the runtime keeps for itself after first use is allocated by now
    free0 = torch.cuda.mem_get_info()[0]
    cycle(300)
    free1 = torch.cuda.mem_get_info()[0]
    assert free0 - free1 < (8 << 20), (free0, free1)
    G.assert_bytes_equal(dst.cpu().numpy(), G.oracle_expected(w, src_host), "after 320 plans")


def test_blockwise_memcpy_baseline_gives_the_same_bytes():
    w = wl.config2(num_layers=2, pool_blocks=512, tokens=1000)
    src_host = host_src(w)
    src, dst = G.device_pool_from_host(src_host), G.device_sentinel_pool(w.dst)
    x = G.GpuTransfer(w, src, dst)
    x.build()
    x.plan.pull_blockwise_memcpy(x.stream.cuda_stream)
    x.stream.synchronize()
    G.assert_bytes_equal(dst.cpu().numpy(), G.oracle_expected(w, src_host), "blockwise memcpy")
    x.close()
    w5 = wl.config5(num_layers=1, src_pool_blocks=64, tokens=64)
    y = G.GpuTransfer(w5, G.device_sentinel_pool(w5.src), G.device_sentinel_pool(w5.dst))
    y.build()
    with pytest.raises(kvd.KvdError) as e:
        y.plan.pull_blockwise_memcpy(y.stream.cuda_stream)
    assert e.value.code == kvd.KVD_ERR_MISMATCH
    y.close()


@pytest.mark.parametrize("w", [wl.config2(num_layers=2, pool_blocks=512, tokens=1000),
                               wl.config5(num_layers=2, src_pool_blocks=128, tokens=500),
                               wl.config3(num_layers=1, num_requests=6, median=100.0, hi=600)], ids=lambda w: w.name)
@pytest.mark.parametrize("buffer_bytes", [4096, 65536, 1 << 22])
def test_staged_gather_scatter_baseline_gives_the_same_bytes(w, buffer_bytes):
    src_host = host_src(w)
    src, dst = G.device_pool_from_host(src_host), G.device_sentinel_pool(w.dst)
    send = torch.zeros(buffer_bytes, dtype=torch.uint8, device="cuda")
    recv = torch.zeros(buffer_bytes, dtype=torch.uint8, device="cuda")
    x = G.GpuTransfer(w, src, dst)
    x.build()
    x.plan.pull_staged(send.data_ptr(), recv.data_ptr(), buffer_bytes, x.stream.cuda_stream)
    G.assert_bytes_equal(dst.cpu().numpy(), G.oracle_expected(w, src_host), "staged baseline")
    with pytest.raises(kvd.KvdError):
        x.plan.pull_staged(send.data_ptr(), recv.data_ptr(), 100, x.stream.cuda_stream)
    x.close()


def test_plain_copy():
    n = (1 << 24) + 4096 + 16
    a = torch.randint(0, 255, (n,), dtype=torch.uint8, device="cuda")
    b = torch.zeros_like(a)
    kvd.kvd_copy_plain(b.data_ptr(), a.data_ptr(), n)
    torch.cuda.synchronize()
    assert torch.equal(a, b)
    with pytest.raises(kvd.KvdError):
        kvd.kvd_copy_plain(b.data_ptr(), a.data_ptr() + 1, 16)


@pytest.mark.parametrize("mode", sorted(kvd.PROBE_MODES))
def test_stream_probes_touch_what_they_say(mode):
    n = 3 * 4096 * 257
    src = torch.randint(0, 255, (n,), dtype=torch.uint8, device="cuda")
    dst = torch.full((n,), 7, dtype=torch.uint8, device="cuda")
    keep = src.clone()
    torch.cuda.synchronize()
    kvd.kvd_stream_probe(dst.data_ptr(), src.data_ptr(), n, mode)
    torch.cuda.synchronize()
    assert torch.equal(src, keep)
    if mode.startswith("copy"):
        assert torch.equal(dst, src)
    elif mode.startswith("read"):
        assert int((dst != 7).sum()) == 0
    else:
        assert int((dst.view(torch.int16) != 0x3C00).sum()) == 0
    for bad in ((dst.data_ptr(), src.data_ptr(), 4095), (0, src.data_ptr(), 4096), (dst.data_ptr() + 8, src.data_ptr(), 4096)):
        with pytest.raises(kvd.KvdError):
            kvd.kvd_stream_probe(*bad, mode)


def _frag_request(gs, gd, tokens, seed):
    rng = np.random.default_rng(seed)
    return wl.Request(tokens,
                      wl.fragmented_allocation(rng, np.ones(gs.num_blocks, bool), wl.blocks_for(tokens, gs.block_tokens), 6),
                      wl.fragmented_allocation(rng, np.ones(gd.num_blocks, bool), wl.blocks_for(tokens, gd.block_tokens), 6))


@pytest.mark.parametrize("gs,gd", [
    (small_geom(kv_adjacent=True), small_geom(kv_adjacent=True)),
    (small_geom(kv_adjacent=True, layout=wl.BTHD), small_geom(kv_adjacent=True, layout=wl.BTHD)),
    (small_geom(kv_adjacent=True, layout=wl.BTHD), small_geom(kv_adjacent=True, layout=wl.BTHD, block_tokens=32, num_blocks=48)),
    (small_geom(kv_adjacent=True, block_tokens=32, num_blocks=48), small_geom(kv_adjacent=True, block_tokens=8, num_blocks=192)),
    (small_geom(kv_adjacent=True, num_kv_heads=1), small_geom(kv_adjacent=True, num_kv_heads=1, layout=wl.BTHD)),
], ids=["hm", "tm", "tm16-32", "hm32-8", "one-head"])
@pytest.mark.parametrize("tokens", [333, 1024])
def test_pools_with_k_and_v_of_a_block_adjacent(gs, gd, tokens):
    """K and V of a block merge into one range (byte-offset contiguity, section 4.1)."""
    w = wl.Workload("kv-adjacent", gs, gd, [_frag_request(gs, gd, tokens, 31)], "bf16", 31)
    x = G.run_and_compare(w, host_src(w))
    got = x.plan.descriptors(x.stream.cuda_stream)
    want = tl.oracle_plan_descriptors(w, 0, -1)
    assert np.array_equal(got, want)
    if gs.block_tokens == gd.block_tokens and tokens % 16 == 0:
        # whole blocks only: every run of r consecutive blocks is ONE descriptor of 2*r tiles
        r = w.requests[0]
        breaks = np.count_nonzero((r.src_table[1:] != r.src_table[:-1] + 1) | (r.dst_table[1:] != r.dst_table[:-1] + 1))
        assert len(got) == 1 + breaks and got[:, 2].sum() == 2 * tokens * gs.num_kv_heads * gs.head_dim * 2
    x.close()


@pytest.mark.parametrize("adj_src,adj_dst", [(True, False), (False, True)])
def test_one_side_with_adjacent_k_and_v(adj_src, adj_dst):
    gs, gd = small_geom(kv_adjacent=adj_src), small_geom(kv_adjacent=adj_dst)
    w = wl.Workload("kv-one-side", gs, gd, [_frag_request(gs, gd, 700, 32)], "bf16", 32)
    x = G.run_and_compare(w, host_src(w))
    assert np.array_equal(x.plan.descriptors(x.stream.cuda_stream), tl.oracle_plan_descriptors(w, 0, 0))
    x.close()


@pytest.mark.parametrize("gs,gd", [
    (small_geom(block_major=True), small_geom(block_major=True)),
    (small_geom(block_major=True, layout=wl.BTHD), small_geom(block_major=True, layout=wl.BTHD)),
    (small_geom(block_major=True, layout=wl.BTHD), small_geom(block_major=True, layout=wl.BTHD, block_tokens=32, num_blocks=48)),
    (small_geom(block_major=True, block_tokens=32, num_blocks=48), small_geom(block_major=True, block_tokens=8, num_blocks=192)),
    (small_geom(block_major=True, num_kv_heads=1), small_geom(block_major=True, num_kv_heads=1, layout=wl.BTHD)),
], ids=["hm", "tm", "tm16-32", "hm32-8", "one-head"])
@pytest.mark.parametrize("tokens", [333, 1024])
@pytest.mark.parametrize("layers", [(0, 3), (1, 3), (1, 2)])
@pytest.mark.parametrize("flags", [0, kvd.KVD_PLAN_WIDE_OFFSETS], ids=["offsets32", "offsets48"])
def test_block_major_pools(gs, gd, tokens, layers, flags):
    """Pools that keep all layers of a block together: what a request moves of a block is one byte range."""
    w = wl.Workload("block-major", gs, gd, [_frag_request(gs, gd, tokens, 41)], "bf16", 41, layers[0], layers[1])
    x = G.run_and_compare(w, host_src(w), flags)
    got = x.plan.descriptors(x.stream.cuda_stream)
    assert np.array_equal(got, tl.oracle_plan_descriptors_block_major(w))
    st = x.plan.stats(x.stream.cuda_stream)
    nl = layers[1] - layers[0]
    assert st["payload_bytes"] == tokens * nl * 2 * gs.num_kv_heads * gs.head_dim * 2 == got[:, 2].sum()
    if gs.block_tokens == gd.block_tokens and tokens % 16 == 0 and nl == 3:
        r = w.requests[0]
        breaks = np.count_nonzero((r.src_table[1:] != r.src_table[:-1] + 1) | (r.dst_table[1:] != r.dst_table[:-1] + 1))
        assert len(got) == 1 + breaks
    x.close()


@pytest.mark.parametrize("flags", [0, kvd.KVD_PLAN_WIDE_OFFSETS], ids=["offsets32", "offsets48"])
def test_block_major_with_several_thousand_transactions(flags):
    """More transactions than one pass of the build kernel takes (1024), in block-major pools: runs that
    continue across the passes, two requests, the second one continuing the first one's last run."""
    g = wl.PoolGeometry(2, 8192, 2, 2, 16, 2, wl.BHTD, block_major=True)     # 512-byte blocks
    rng = np.random.default_rng(81)
    free_s, free_d = np.ones(g.num_blocks, bool), np.ones(g.num_blocks, bool)
    free_s[:40] = free_d[100:140] = False
    n1 = 3300
    r1 = wl.Request(n1 * 2, np.concatenate([wl.fragmented_allocation(rng, free_s, n1 - 20, 9), np.arange(0, 20)]).astype(np.int32),
                    np.concatenate([wl.fragmented_allocation(rng, free_d, n1 - 20, 9), np.arange(100, 120)]).astype(np.int32))
    r2 = wl.Request(1501 * 2 - 1, np.concatenate([np.arange(20, 40), wl.fragmented_allocation(rng, free_s, 1481, 9)]).astype(np.int32),
                    np.concatenate([np.arange(120, 140), wl.fragmented_allocation(rng, free_d, 1481, 9)]).astype(np.int32))
    w = wl.Workload("many-block-major", g, g, [r1, r2], "bf16", 81)
    x = G.run_and_compare(w, host_src(w), flags)
    got = x.plan.descriptors(x.stream.cuda_stream)
    want = tl.oracle_plan_descriptors_block_major(w)
    assert np.array_equal(got, want)
    # the run 0..39 -> 100..139 crosses the two requests and is one descriptor
    assert [0, 100 * 512, 40 * 512] in got.tolist()
    x.close()


@pytest.mark.parametrize("gs,gd", [
    (small_geom(block_major=True), small_geom(block_major=True, layout=wl.BTHD, block_tokens=32, num_blocks=48)),
    (small_geom(block_major=True, layout=wl.BTHD, block_tokens=32, num_blocks=48), small_geom(block_major=True, block_tokens=8, num_blocks=192)),
    (small_geom(block_major=True, layout=wl.BTHD), small_geom(block_major=True)),
    (small_geom(block_major=True, num_kv_heads=3, head_dim=8, block_tokens=64, num_blocks=24),
     small_geom(block_major=True, num_kv_heads=3, head_dim=8, layout=wl.BTHD, block_tokens=1, num_blocks=1536)),
], ids=["ht16-th32", "th32-ht8", "th16-ht16", "ht64-th1"])
def test_relayout_between_block_major_pools(gs, gd):
    """Re-layout where both pools keep a block's layers together: pulled descriptor by descriptor.
    A batch, a request with another layer range, then the same plan layer by layer."""
    rng = np.random.default_rng(91)
    free_s, free_d = np.ones(gs.num_blocks, bool), np.ones(gd.num_blocks, bool)
    lens, ranges = [333, 64, 150], [(0, 3), (0, 3), (1, 2)]
    reqs = [wl.Request(t, wl.fragmented_allocation(rng, free_s, wl.blocks_for(t, gs.block_tokens), 4),
                       wl.fragmented_allocation(rng, free_d, wl.blocks_for(t, gd.block_tokens), 4)) for t in lens]
    src_host = rng.integers(0, 256, size=gs.total_bytes, dtype=np.uint8)
    want = wl.host_pool_sentinel(gd)
    for r, (l0, l1) in zip(reqs, ranges):
        tl.oracle_pull_workload(wl.Workload("one", gs, gd, [r], "bf16", 0, l0, l1), src_host, want)
    src, dst = G.device_pool_from_host(src_host), G.device_sentinel_pool(gd)
    plan = kvd.Plan(kvd.Pool(src.data_ptr(), gs), kvd.Pool(dst.data_ptr(), gd), 3, 2048)
    plan.build_descriptors_batch([r.src_table for r in reqs[:2]], [r.dst_table for r in reqs[:2]], lens[:2], 0, 3)
    plan.build_descriptors(reqs[2].src_table, reqs[2].dst_table, lens[2], 1, 2)
    assert plan.stats()["relayout"] == 1
    plan.pull()
    torch.cuda.synchronize()
    G.assert_bytes_equal(dst.cpu().numpy(), want, "descriptor-by-descriptor pull")
    dst.view(torch.int16).fill_(wl.SENTINEL16)
    for layer in (2, 0, 1):
        plan.pull_layers(layer, layer + 1)
    torch.cuda.synchronize()
    G.assert_bytes_equal(dst.cpu().numpy(), want, "the same, layer by layer")
    G.assert_bytes_equal(src.cpu().numpy(), src_host, "source changed")
    plan.close()


@pytest.mark.parametrize("major_src,major_dst", [(True, False), (False, True)])
def test_one_side_block_major(major_src, major_dst):
    """Only one pool keeps a block's layers together: nothing merges across layers, K and V still do."""
    gs = small_geom(block_major=major_src, kv_adjacent=not major_src)
    gd = small_geom(block_major=major_dst, kv_adjacent=not major_dst)
    w = wl.Workload("block-major-one-side", gs, gd, [_frag_request(gs, gd, 700, 42)], "bf16", 42)
    x = G.run_and_compare(w, host_src(w))
    assert np.array_equal(x.plan.descriptors(x.stream.cuda_stream), tl.oracle_plan_descriptors(w, 0, -1))
    x.close()


def test_block_major_batch_mixed_layer_ranges_and_baselines():
    """Several requests in one block-major plan: a batch, then requests with other layer ranges; the
    comparison forms of the pull move the same bytes."""
    g = small_geom(block_major=True, num_blocks=256)
    rng = np.random.default_rng(43)
    free_s, free_d = np.ones(256, bool), np.ones(256, bool)
    lens = [100, 16, 333, 7, 64]
    reqs = [wl.Request(t, wl.fragmented_allocation(rng, free_s, wl.blocks_for(t, 16), 4),
                       wl.fragmented_allocation(rng, free_d, wl.blocks_for(t, 16), 4)) for t in lens]
    ranges = [(0, 3), (0, 3), (0, 3), (1, 3), (2, 3)]
    src_host = rng.integers(0, 256, size=g.total_bytes, dtype=np.uint8)
    want = wl.host_pool_sentinel(g)
    for r, (l0, l1) in zip(reqs, ranges):
        tl.oracle_pull_workload(wl.Workload("one", g, g, [r], "bf16", 0, l0, l1), src_host, want)
    for flags in (0, kvd.KVD_PLAN_NO_COALESCE, kvd.KVD_PLAN_WIDE_OFFSETS):
        src, dst = G.device_pool_from_host(src_host), G.device_sentinel_pool(g)
        plan = kvd.Plan(kvd.Pool(src.data_ptr(), g), kvd.Pool(dst.data_ptr(), g), len(reqs), 64, flags)
        plan.build_descriptors_batch([r.src_table for r in reqs[:3]], [r.dst_table for r in reqs[:3]], lens[:3], 0, 3)
        for r, (l0, l1) in zip(reqs[3:], ranges[3:]):
            plan.build_descriptors(r.src_table, r.dst_table, r.seq_len, l0, l1)
        plan.pull()
        torch.cuda.synchronize()
        G.assert_bytes_equal(dst.cpu().numpy(), want, f"block-major batch, flags {flags}")
        if flags != kvd.KVD_PLAN_NO_COALESCE:
            wb = wl.Workload("batch", g, g, reqs[:3], "bf16", 0)
            head = tl.oracle_plan_descriptors_block_major(wb)
            assert np.array_equal(plan.descriptors()[:len(head)], head)
        # staged and per-block memcpy forms of the same plan
        for form in ("staged", "memcpy"):
            dst2 = G.device_sentinel_pool(g)
            plan2 = kvd.Plan(kvd.Pool(src.data_ptr(), g), kvd.Pool(dst2.data_ptr(), g), len(reqs), 64, flags)
            for r, (l0, l1) in zip(reqs, ranges):
                plan2.build_descriptors(r.src_table, r.dst_table, r.seq_len, l0, l1)
            if form == "staged":
                send = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
                recv = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
                plan2.pull_staged(send.data_ptr(), recv.data_ptr(), 1 << 16)
            else:
                plan2.pull_blockwise_memcpy()
            torch.cuda.synchronize()
            G.assert_bytes_equal(dst2.cpu().numpy(), want, f"block-major {form}, flags {flags}")
            plan2.close()
        plan.close()
    # persistent form: one layer range for the whole plan
    src, dst = G.device_pool_from_host(src_host), G.device_sentinel_pool(g)
    want1 = wl.host_pool_sentinel(g)
    plan = kvd.Plan(kvd.Pool(src.data_ptr(), g), kvd.Pool(dst.data_ptr(), g), len(reqs), 64, kvd.KVD_PLAN_PERSISTENT)
    for r in reqs:
        plan.build_descriptors(r.src_table, r.dst_table, r.seq_len, 1, 3)
        tl.oracle_pull_workload(wl.Workload("one", g, g, [r], "bf16", 0, 1, 3), src_host, want1)
    plan.pull()
    torch.cuda.synchronize()
    G.assert_bytes_equal(dst.cpu().numpy(), want1, "block-major persistent")
    plan.close()


@pytest.mark.parametrize("g", [small_geom(), small_geom(layout=wl.BTHD), small_geom(kv_adjacent=True),
                               small_geom(block_major=True)],
                         ids=["hm", "tm", "kv-adjacent", "block-major"])
def test_whole_block_mode_moves_every_slot_of_the_last_block(g):
    tokens = 16 * 9 + 5
    w = wl.Workload("whole", g, g, [_frag_request(g, g, tokens, 33)], "bf16", 33)
    src_host = host_src(w)
    src, dst = G.device_pool_from_host(src_host), G.device_sentinel_pool(g)
    x = G.GpuTransfer(w, src, dst, flags=kvd.KVD_PLAN_WHOLE_BLOCKS).run()
    # block-granular transfer = the definition applied to all 16 slots of the 10 blocks
    r = w.requests[0]
    w_full = wl.Workload("whole-oracle", g, g, [wl.Request(160, r.src_table, r.dst_table)], "bf16", 33)
    G.assert_bytes_equal(dst.cpu().numpy(), G.oracle_expected(w_full, src_host), "whole-block mode")
    st = x.plan.stats(x.stream.cuda_stream)
    assert st["payload_bytes"] == 160 * g.num_layers * 2 * g.num_kv_heads * g.head_dim * 2
    want = tl.oracle_plan_descriptors_block_major(w_full) if g.block_major else \
        tl.oracle_plan_descriptors(w_full, 0, -1 if g.kv_adjacent else 0)
    assert np.array_equal(x.plan.descriptors(x.stream.cuda_stream), want)
    x.close()


@pytest.mark.parametrize("gs,gd", [
    (wl.PoolGeometry(2, 6, 1024, 2, 8, 2, wl.BHTD), wl.PoolGeometry(2, 24, 256, 2, 8, 2, wl.BTHD)),
    (wl.PoolGeometry(2, 6, 1024, 3, 8, 2, wl.BTHD), wl.PoolGeometry(2, 6, 1024, 3, 8, 2, wl.BHTD)),
    (wl.PoolGeometry(2, 6, 1024, 2, 8, 2, wl.BHTD), wl.PoolGeometry(2, 6, 1024, 2, 8, 2, wl.BHTD)),
], ids=["1024-to-256-relayout", "1024-relayout-back", "1024-same"])
def test_largest_block_size(gs, gd):
    w = one_request(gs, gd, 5000)
    G.run_and_compare(w, host_src(w)).close()


@pytest.mark.parametrize("row_units", [256, 255, 129, 128, 86])
@pytest.mark.parametrize("lay_s,lay_d,tb_d", [(wl.BHTD, wl.BHTD, 4), (wl.BTHD, wl.BTHD, 8), (wl.BHTD, wl.BTHD, 8),
                                               (wl.BTHD, wl.BHTD, 2)])
def test_widest_rows(row_units, lay_s, lay_d, tb_d):
    """(token, head) rows up to the limit of 4096 bytes: one row per work item, rows that do not
    divide a work item, re-layout with a single row per item."""
    hd = row_units * 16 // 2
    gs = wl.PoolGeometry(2, 40, 4, 3, hd, 2, lay_s)
    gd = wl.PoolGeometry(2, 4 * 40 // tb_d + 2, tb_d, 3, hd, 2, lay_d)
    w = one_request(gs, gd, 4 * 31 + 3, seed=row_units)
    G.run_and_compare(w, host_src(w)).close()


@pytest.mark.parametrize("block_major", [False, True])
def test_many_layers(block_major):
    """Several hundred layers: as many slabs in the grid, or one folded range per block of 600 planes."""
    g = wl.PoolGeometry(300, 24, 4, 1, 8, 2, wl.BHTD, block_major=block_major)
    w = one_request(g, g, 4 * 9 + 1, seed=300)
    G.run_and_compare(w, host_src(w)).close()
    w2 = one_request(g, g, 4 * 9 + 1, seed=301, layer_begin=257, layer_end=300)
    G.run_and_compare(w2, host_src(w2)).close()


def test_slab_larger_than_4_gib():
    """Block offsets beyond 2^32 bytes inside one (layer, K/V) slab; checked through a compact
    renumbering of the blocks that are used (the oracle never sees the 10 GiB pools)."""
    nb = 163840  # x 32 KiB = 5 GiB per slab
    g = wl.PoolGeometry(1, nb, 16, 8, 128, 2, wl.BHTD)
    rng = np.random.default_rng(21)
    n = 300
    st = np.concatenate([rng.choice(np.arange(nb - 5000, nb), n - 20, replace=False), rng.choice(5000, 20, replace=False)])
    dt = np.concatenate([rng.choice(np.arange(nb - 5000, nb), n - 20, replace=False), rng.choice(5000, 20, replace=False)])
    st, dt = rng.permutation(st).astype(np.int32), rng.permutation(dt).astype(np.int32)
    st[10:14] = [nb - 4, nb - 3, nb - 2, nb - 1]          # a run that ends at the pool's last block
    dt[10:14] = [nb - 8, nb - 7, nb - 6, nb - 5]
    seq = n * 16 - 7
    say("allocating two 10 GiB pools")
    src = G.device_random_pool(g, "bf16", 21)
    dst = G.device_sentinel_pool(g)
    w = wl.Workload("big-slab", g, g, [wl.Request(seq, st, dt)], "bf16", 21)
    x = G.GpuTransfer(w, src, dst).run()
    # compact copies: used blocks only, renumbered by rank
    us, ud = np.unique(st), np.unique(dt)
    gs_c = wl.PoolGeometry(1, len(us), 16, 8, 128, 2, wl.BHTD)
    gd_c = wl.PoolGeometry(1, len(ud), 16, 8, 128, 2, wl.BHTD)
    s4 = src.view(torch.int16).view(2, nb, -1)
    d4 = dst.view(torch.int16).view(2, nb, -1)
    src_c = s4[:, torch.from_numpy(us.astype(np.int64)).cuda()].contiguous().cpu().numpy().view(np.uint8).reshape(-1)
    got_c = d4[:, torch.from_numpy(ud.astype(np.int64)).cuda()].contiguous().cpu().numpy().view(np.uint8).reshape(-1)
    wc = wl.Workload("compact", gs_c, gd_c, [wl.Request(seq, np.searchsorted(us, st).astype(np.int32),
                                                        np.searchsorted(ud, dt).astype(np.int32))], "bf16", 21)
    want_c = wl.host_pool_sentinel(gd_c)
    tl.oracle_pull_workload(wc, src_c, want_c)
    G.assert_bytes_equal(got_c, want_c, "compact view of the destination")
    # nothing outside the used blocks was written
    touched = int((d4 != wl.SENTINEL16).sum())
    assert touched == seq * 2 * 8 * 128
    x.close()
    del src, dst, s4, d4
    torch.cuda.empty_cache()


def _random_case(seed):
    """A seeded random small transfer: geometry, layouts, block sizes, several requests with their own
    layer ranges, plan flags."""
    rng = np.random.default_rng(5000 + seed)
    elem = int(rng.choice([1, 2, 2, 2, 4, 8]))
    row_units = int(rng.choice([1, 2, 3, 4, 8, 12, 16]))            # 16-byte units per (token, head) row
    head_dim = row_units * 16 // elem
    hk = int(rng.choice([1, 1, 2, 3, 4, 8]))
    layers = int(rng.integers(1, 5))
    tb_s = int(rng.choice([1, 2, 4, 8, 16, 32, 64]))
    ratio = int(rng.choice([1, 1, 1, 2, 4]))
    tb_d = tb_s * ratio if rng.random() < 0.5 else max(1, tb_s // ratio)
    lay_s, lay_d = (str(rng.choice([wl.BHTD, wl.BTHD])) for _ in range(2))
    adj_s, adj_d = (bool(rng.random() < 0.3) for _ in range(2))
    n_req = int(rng.integers(1, 5))
    lens = [int(rng.integers(1, 400)) for _ in range(n_req)]
    need_s = sum(wl.blocks_for(t, tb_s) for t in lens)
    need_d = sum(wl.blocks_for(t, tb_d) for t in lens)
    gs = wl.PoolGeometry(layers, need_s + int(rng.integers(1, 40)), tb_s, hk, head_dim, elem, lay_s, adj_s)
    gd = wl.PoolGeometry(layers, need_d + int(rng.integers(1, 40)), tb_d, hk, head_dim, elem, lay_d, adj_d)
    free_s, free_d = np.ones(gs.num_blocks, bool), np.ones(gd.num_blocks, bool)
    reqs, ranges = [], []
    uniform = rng.random() < 0.6
    for t in lens:
        reqs.append(wl.Request(t, wl.fragmented_allocation(rng, free_s, wl.blocks_for(t, tb_s), 5),
                               wl.fragmented_allocation(rng, free_d, wl.blocks_for(t, tb_d), 5)))
        l0 = 0 if uniform else int(rng.integers(0, layers))
        ranges.append((l0, layers if uniform else int(rng.integers(l0 + 1, layers + 1))))
    flags = 0
    if rng.random() < 0.2:
        flags |= kvd.KVD_PLAN_NO_COALESCE
    if uniform and rng.random() < 0.25:
        flags |= kvd.KVD_PLAN_PERSISTENT
    if tb_s == tb_d and rng.random() < 0.25:
        flags |= kvd.KVD_PLAN_WHOLE_BLOCKS
    batch = bool(uniform and n_req > 1 and rng.random() < 0.5)
    if seed >= 60:  # the later seeds also draw pools that keep all layers of a block together
        gs = dataclasses.replace(gs, block_major=bool(rng.random() < 0.6))
        gd = dataclasses.replace(gd, block_major=bool(rng.random() < 0.6))
        foldable = gs.block_major and gd.block_major and (lay_s == lay_d or hk == 1)
        if foldable and not (flags & kvd.KVD_PLAN_PERSISTENT) and rng.random() < 0.5:
            flags |= kvd.KVD_PLAN_WIDE_OFFSETS
    if not (flags & kvd.KVD_PLAN_PERSISTENT) and rng.random() < 0.5:
        flags |= kvd.KVD_PLAN_DESTINATION_ORDER  # short descriptors are grouped or sorted however small the transfer
    return gs, gd, reqs, ranges, flags, batch


@pytest.mark.parametrize("seed", range(300))
def test_random_small_transfers(seed):
    gs, gd, reqs, ranges, flags, batch = _random_case(seed)
    say(f"seed {seed}: {gs} -> {gd}, lens {[r.seq_len for r in reqs]}, layers {ranges}, flags {flags}, batch {batch}")
    rng = np.random.default_rng(seed)
    src_host = rng.integers(0, 256, size=gs.total_bytes, dtype=np.uint8)
    want = wl.host_pool_sentinel(gd)
    src, dst = G.device_pool_from_host(src_host), G.device_pool_from_host(want.copy())
    plan = kvd.Plan(kvd.Pool(src.data_ptr(), gs), kvd.Pool(dst.data_ptr(), gd), len(reqs),
                    sum(max(len(r.src_table), len(r.dst_table)) for r in reqs), flags)
    whole = bool(flags & kvd.KVD_PLAN_WHOLE_BLOCKS)
    if batch:
        plan.build_descriptors_batch([r.src_table for r in reqs], [r.dst_table for r in reqs],
                                     [r.seq_len for r in reqs], ranges[0][0], ranges[0][1])
    for r, (l0, l1) in zip(reqs, ranges):
        if not batch:
            plan.build_descriptors(r.src_table, r.dst_table, r.seq_len, l0, l1)
        t = wl.blocks_for(r.seq_len, gs.block_tokens) * gs.block_tokens if whole else r.seq_len
        w1 = wl.Workload("one", gs, gd, [wl.Request(t, r.src_table, r.dst_table)], "bf16", 0, l0, l1)
        tl.oracle_pull_workload(w1, src_host, want)
    plan.pull()
    torch.cuda.synchronize()
    G.assert_bytes_equal(dst.cpu().numpy(), want, f"random case {seed}")
    G.assert_bytes_equal(src.cpu().numpy(), src_host, f"random case {seed}: source changed")
    plan.close()
    # the same requests, one call each, through the entry point that allocates nothing
    carried = flags & (kvd.KVD_PLAN_NO_COALESCE | kvd.KVD_PLAN_WHOLE_BLOCKS | kvd.KVD_PLAN_DESTINATION_ORDER)
    dst2 = G.device_pool_from_host(wl.host_pool_sentinel(gd))
    sd, dd = kvd.pool_desc(src.data_ptr(), gs), kvd.pool_desc(dst2.data_ptr(), gd)
    torch.cuda.synchronize()
    for r, (l0, l1) in zip(reqs, ranges):
        kvd.kvd_pull_noalloc(sd, dd, r.src_table, r.dst_table, r.seq_len, l0, l1, carried)
    torch.cuda.synchronize()
    G.assert_bytes_equal(dst2.cpu().numpy(), want, f"random case {seed}: kvd_pull_noalloc")
    # and as a plan that completes request by request (every other seed; not for the persistent form, nor for
    # re-layout between block-major pools, which kvd_pull_notify refuses)
    relayout_bm = gs.block_major and gd.block_major and gs.layout != gd.layout and gs.num_kv_heads > 1
    if seed % 2 == 0 and not (flags & kvd.KVD_PLAN_PERSISTENT) and not relayout_bm:
        dst3 = G.device_pool_from_host(wl.host_pool_sentinel(gd))
        words = torch.zeros(len(reqs), dtype=torch.int64, device="cuda")
        plan = kvd.Plan(kvd.Pool(src.data_ptr(), gs), kvd.Pool(dst3.data_ptr(), gd), len(reqs),
                        sum(max(len(r.src_table), len(r.dst_table)) for r in reqs), flags | kvd.KVD_PLAN_COMPLETE_PER_REQUEST)
        torch.cuda.synchronize()
        if batch:
            plan.build_descriptors_batch([r.src_table for r in reqs], [r.dst_table for r in reqs],
                                         [r.seq_len for r in reqs], ranges[0][0], ranges[0][1])
        else:
            for r, (l0, l1) in zip(reqs, ranges):
                plan.build_descriptors(r.src_table, r.dst_table, r.seq_len, l0, l1)
        plan.pull_notify(words.data_ptr(), seed + 1)
        torch.cuda.synchronize()
        assert words.tolist() == [seed + 1] * len(reqs)
        G.assert_bytes_equal(dst3.cpu().numpy(), want, f"random case {seed}: kvd_pull_notify")
        plan.close()


# ------------------------------------------------------------------ full-size configurations

def _check_full(w, sample_layers):
    say(f"{w.name}: allocating pools {w.src.total_bytes / 2**30:.1f} + {w.dst.total_bytes / 2**30:.1f} GiB")
    src = G.device_random_pool(w.src, w.dtype, w.seed)
    dst = G.device_sentinel_pool(w.dst)
    checksum = [int(src.view(torch.int16)[i::9973][:4096].sum()) for i in range(3)]
    x = G.GpuTransfer(w, src, dst)
    say(f"{w.name}: build + pull")
    x.run(batch=len(w.requests) > 1)  # the launch configuration bench.py times
    st = x.plan.stats(x.stream.cuda_stream)
    say(f"{w.name}: {st}")
    moved16 = st["payload_bytes"] // 2
    # property on every layer: exactly the payload's words differ from the sentinel
    sv = dst.view(torch.int16).view(w.dst.num_layers, -1)
    nonsent = sum(int((sv[layer] != wl.SENTINEL16).sum()) for layer in range(w.dst.num_layers))
    assert nonsent == moved16
    # property on every layer (equal layout and block size): whole blocks arrive as whole blocks
    if w.src.layout == w.dst.layout and w.src.block_tokens == w.dst.block_tokens:
        s5 = src.view(torch.int16).view(w.src.num_layers, 2, w.src.num_blocks, -1)
        d5 = dst.view(torch.int16).view(w.dst.num_layers, 2, w.dst.num_blocks, -1)
        for r in w.requests:
            n = r.seq_len // w.src.block_tokens
            si = torch.from_numpy(r.src_table[:n].astype(np.int64)).cuda()
            di = torch.from_numpy(r.dst_table[:n].astype(np.int64)).cuda()
            for layer in range(w.layer_begin, w.layer_end):
                assert torch.equal(d5[layer][:, di], s5[layer][:, si])
    # oracle, element by element, on the given layers (all of them except for the batch of 64)
    for layer in sample_layers:
        say(f"{w.name}: oracle on layer {layer}")
        G.compare_layer_with_oracle(w, src, dst, layer)
    assert checksum == [int(src.view(torch.int16)[i::9973][:4096].sum()) for i in range(3)]
    x.close()
    # the other entry points at full size, against the pool just verified: the call that allocates nothing
    # (single requests), a completion word per request (the batch)
    verified = dst.clone()
    dst.view(torch.int16).fill_(wl.SENTINEL16)
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    if len(w.requests) == 1:
        say(f"{w.name}: kvd_pull_noalloc")
        r = w.requests[0]
        kvd.kvd_pull_noalloc(kvd.pool_desc(src.data_ptr(), w.src), kvd.pool_desc(dst.data_ptr(), w.dst), r.src_table, r.dst_table,
                             r.seq_len, w.layer_begin, w.layer_end, 0, stream.cuda_stream)
        stream.synchronize()
    else:
        say(f"{w.name}: kvd_pull_notify")
        y = G.GpuTransfer(w, src, dst, kvd.KVD_PLAN_COMPLETE_PER_REQUEST, stream=stream)
        y.build(batch=True)
        words = torch.zeros(len(w.requests), dtype=torch.int64, device="cuda")
        stream.wait_stream(torch.cuda.current_stream())
        y.plan.pull_notify(words.data_ptr(), 11, stream.cuda_stream)
        stream.synchronize()
        assert words.tolist() == [11] * len(w.requests)
        y.close()
    assert torch.equal(dst, verified)
    del src, dst, verified
    torch.cuda.empty_cache()


def test_full_config2():
    _check_full(wl.config2(), range(32))


def test_full_config3():
    _check_full(wl.config3(), [0, 3, 8, 13, 17, 22, 27, 31])


def test_full_config4():
    _check_full(wl.config4(), range(80))


def test_full_config5():
    _check_full(wl.config5(), range(32))


def test_full_config2_block_major_with_every_block_alone():
    """cfg2's shape in block-major pools, every block alone on both sides: one 2 MiB range per block."""
    base = wl.config2()
    g = dataclasses.replace(base.src, block_major=True)
    rng = np.random.default_rng(77)
    n = wl.blocks_for(8192 - 5, 16)
    w = wl.Workload("cfg2-block-major-lone", g, g, [wl.Request(8192 - 5, wl.scattered_table(rng, g.num_blocks, n),
                                                              wl.scattered_table(rng, g.num_blocks, n))], "bf16", 77)
    say(f"{w.name}: allocating pools 2 x {g.total_bytes / 2**30:.1f} GiB")
    src = G.device_random_pool(g, "bf16", 77)
    dst = G.device_sentinel_pool(g)
    x = G.GpuTransfer(w, src, dst).run()
    st = x.plan.stats(x.stream.cuda_stream)
    say(f"{w.name}: {st}")
    r = w.requests[0]
    assert st["num_descriptors"] == (n - 1) + g.num_layers * 2 * g.num_kv_heads
    assert st["payload_bytes"] == r.seq_len * g.num_layers * 2 * g.num_kv_heads * g.head_dim * 2
    # exactly the payload's words differ from the sentinel
    dv = dst.view(torch.int16).view(g.num_blocks, g.num_layers, 2, -1)
    sv = src.view(torch.int16).view(g.num_blocks, g.num_layers, 2, -1)
    nonsent = sum(int((dv[b0:b0 + 1024] != wl.SENTINEL16).sum()) for b0 in range(0, g.num_blocks, 1024))
    assert nonsent == st["payload_bytes"] // 2
    # whole blocks arrive as whole blocks, all layers
    si = torch.from_numpy(r.src_table[:n - 1].astype(np.int64)).cuda()
    di = torch.from_numpy(r.dst_table[:n - 1].astype(np.int64)).cuda()
    for lo in range(0, n - 1, 128):
        assert torch.equal(dv[di[lo:lo + 128]], sv[si[lo:lo + 128]])
    # oracle, element by element, on every layer: torch's strided view hands the layer over as a one-layer
    # pool in [kv][block] order, which the oracle addresses with that pool's own strides
    for layer in range(g.num_layers):
        say(f"{w.name}: oracle on layer {layer}")
        G.compare_layer_with_oracle(w, src, dst, layer)
    x.close()


def test_block_major_pools_above_64_gib():
    """Two 66 GiB block-major pools: offsets beyond 2^32 sixteen-byte units, blocks that straddle the
    32 GiB and 64 GiB marks, runs that cross them.  Bytes are checked through a compact renumbering of
    the used blocks (the oracle never sees the pools); descriptors against the oracle's merged queue,
    which the library may only differ from by splitting a run where it enters the next 32 GiB window."""
    layers, hk, hd, tb = 3, 8, 128, 16
    tile = tb * hk * hd * 2                       # 32 KiB
    block = layers * 2 * tile                     # 192 KiB: does not divide 32 GiB
    nb = 66 * 2**30 // block
    g = wl.PoolGeometry(layers, nb, tb, hk, hd, 2, wl.BHTD, block_major=True)
    assert g.total_bytes == 66 * 2**30
    rng = np.random.default_rng(61)
    m32, m64 = 2**35 // block, 2**36 // block     # the blocks that straddle the marks
    assert m32 * block < 2**35 < (m32 + 1) * block and m64 * block < 2**36 < (m64 + 1) * block
    # source: a run across the 64 GiB mark, one across the 32 GiB mark, lone blocks everywhere, the last block
    st = np.concatenate([np.arange(m64 - 3, m64 + 4), np.arange(m32 - 2, m32 + 3),
                         rng.choice(np.arange(m64 + 10, nb - 1), 40, replace=False), [nb - 1],
                         rng.choice(np.arange(2000, m32 - 10), 40, replace=False), np.arange(1000, 1006)])
    # destination: runs of the same lengths placed so that its marks fall at other positions of the runs
    dt = np.concatenate([np.arange(m32 - 5, m32 + 2), np.arange(m64 - 1, m64 + 4),
                         rng.choice(np.arange(m32 + 10, m64 - 10), 40, replace=False), [0],
                         rng.choice(np.arange(m64 + 10, nb - 3000), 40, replace=False), np.arange(nb - 2000, nb - 1994)])
    st, dt = st.astype(np.int32), dt.astype(np.int32)
    assert len(set(st.tolist())) == len(st) == len(dt) == len(set(dt.tolist()))
    seq = len(st) * tb - 5
    say("allocating two 66 GiB pools")
    free_bytes, _ = torch.cuda.mem_get_info()
    torch.cuda.empty_cache()
    if torch.cuda.mem_get_info()[0] < 2 * g.total_bytes + (8 << 30):
        pytest.skip("needs 140 GiB of free device memory")
    src = G.device_random_pool(g, "bf16", 61)
    dst = G.device_sentinel_pool(g)
    w = wl.Workload("wide", g, g, [wl.Request(seq, st, dt)], "bf16", 61)
    x = G.GpuTransfer(w, src, dst).run()
    st_ = x.plan.stats(x.stream.cuda_stream)
    say(f"{st_}")
    assert st_["payload_bytes"] == seq * layers * 2 * hk * hd * 2
    # descriptors: the oracle's queue merges the two long runs whole; the library may differ from it only by
    # splitting a run, so merging its list again (the oracle's own greedy merge) must give the oracle's list
    got = x.plan.descriptors(x.stream.cuda_stream)
    want = tl.oracle_plan_descriptors_block_major(w)
    assert got[:, 2].sum() == want[:, 2].sum() == st_["payload_bytes"]
    assert orc.coalesce(got).tolist() == want.tolist() and len(got) > len(want)
    # the documented rule for 48-bit offsets: every block piece of a descriptor starts in the 32 GiB window, on
    # either side, that the descriptor starts in (here a piece is a whole block, but for the ragged last one) ...
    window = 2**35
    for s0, d0, n in got.tolist():
        starts = np.arange(0, n, block)
        assert ((s0 + starts) // window == s0 // window).all() and ((d0 + starts) // window == d0 // window).all()
    # ... and a run is split only there: where two descriptors continue each other, the second starts a new window
    splits = 0
    for (s0, d0, n), (s1, d1, _) in zip(got.tolist()[:-1], got.tolist()[1:]):
        if s0 + n == s1 and d0 + n == d1:
            splits += 1
            assert s1 // window != s0 // window or d1 // window != d0 // window
    assert splits == len(got) - len(want) == 4  # each of the two long runs crosses a mark of either pool
    # compact copies of the used blocks
    us, ud = np.unique(st), np.unique(dt)
    gs_c = wl.PoolGeometry(layers, len(us), tb, hk, hd, 2, wl.BHTD, block_major=True)
    gd_c = wl.PoolGeometry(layers, len(ud), tb, hk, hd, 2, wl.BHTD, block_major=True)
    s2 = src.view(torch.int16).view(nb, -1)
    d2 = dst.view(torch.int16).view(nb, -1)
    src_c = s2[torch.from_numpy(us.astype(np.int64)).cuda()].contiguous().cpu().numpy().view(np.uint8).reshape(-1)
    got_c = d2[torch.from_numpy(ud.astype(np.int64)).cuda()].contiguous().cpu().numpy().view(np.uint8).reshape(-1)
    wc = wl.Workload("compact", gs_c, gd_c, [wl.Request(seq, np.searchsorted(us, st).astype(np.int32),
                                                        np.searchsorted(ud, dt).astype(np.int32))], "bf16", 61)
    want_c = wl.host_pool_sentinel(gd_c)
    tl.oracle_pull_workload(wc, src_c, want_c)
    G.assert_bytes_equal(got_c, want_c, "compact view of the destination")
    # nothing outside the used blocks was written
    touched = sum(int((d2[b0:b0 + 32768] != wl.SENTINEL16).sum()) for b0 in range(0, nb, 32768))
    assert touched == st_["payload_bytes"] // 2
    x.close()
    del src, dst, s2, d2
    torch.cuda.empty_cache()
