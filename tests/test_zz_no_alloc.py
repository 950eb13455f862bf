"""kvd_pull_noalloc, the entry point for callers that cannot allocate: its output against the
output of kvd_build_descriptors + kvd_pull for the same arguments, bit for bit, through the C ABI.
Every case makes two calls in a row on one stream, the second with a smaller input, so that what
the first call left in the library's static scratch array is still there when the second runs."""
import dataclasses

import numpy as np
import pytest
import torch

from paper_2501_14743_amd import kvd
from paper_2501_14743_amd import workloads as wl

gpu = pytest.mark.gpu

if torch.cuda.is_available():
    import kvd_gpu as G


def say(msg):
    print(f"[kvd-test] {msg}", flush=True)


def _block_major(w):
    gs, gd = dataclasses.replace(w.src, block_major=True), dataclasses.replace(w.dst, block_major=True)
    return wl.Workload(w.name + "-block-major", gs, gd, w.requests, w.dtype, w.seed, w.layer_begin, w.layer_end)


def _smaller(w, tokens):
    r = w.requests[0]
    return wl.Workload(w.name + f"-{tokens}", w.src, w.dst, [wl.Request(tokens, r.src_table[::-1].copy(), r.dst_table.copy())],
                       w.dtype, w.seed + 1, w.layer_begin, w.layer_end)


def cases():
    c2 = wl.config2(num_layers=3, pool_blocks=2048, tokens=8192)      # runs of blocks, 4096 work items
    c4 = wl.config4(num_layers=32, pool_blocks=2560, tokens=32768)    # lone 4 KiB blocks: region ordering, 3 table pieces
    c5 = wl.config5(num_layers=2, src_pool_blocks=512, tokens=2000)   # re-layout, ragged
    bm = _block_major(wl.config2(num_layers=4, pool_blocks=1024, tokens=8000))  # layers folded, wide expansion
    return [(c2, 1000), (c4, 4099), (c5, 333), (bm, 17)]


def _reference(w, src, flags):
    """The existing entry points on a fresh sentinel pool."""
    dst = G.device_sentinel_pool(w.dst)
    x = G.GpuTransfer(w, src, dst, flags)
    x.run()
    out = dst.cpu().numpy()
    x.close()
    return out


def _noalloc(w, src, flags, stream):
    dst = G.device_sentinel_pool(w.dst)
    stream.wait_stream(torch.cuda.current_stream())
    r = w.requests[0]
    kvd.kvd_pull_noalloc(kvd.pool_desc(src.data_ptr(), w.src), kvd.pool_desc(dst.data_ptr(), w.dst), r.src_table, r.dst_table,
                         r.seq_len, w.layer_begin, w.layer_end, flags, stream.cuda_stream)
    return dst


@gpu
@pytest.mark.parametrize("w,second_tokens", cases(), ids=lambda v: v.name if hasattr(v, "name") else str(v))
@pytest.mark.parametrize("flags", [0, kvd.KVD_PLAN_WHOLE_BLOCKS])
def test_noalloc_equals_build_plus_pull_twice_in_a_row(w, second_tokens, flags):
    if flags == kvd.KVD_PLAN_WHOLE_BLOCKS and w.src.block_tokens != w.dst.block_tokens:
        pytest.skip("whole-block transfers need equal block sizes")
    w2 = _smaller(w, second_tokens)
    say(f"{w.name}: {w.total_tokens} tokens, then {w2.total_tokens}; flags {flags}")
    src_host = wl.host_pool_values(w.src, w.dtype, w.seed)
    src = G.device_pool_from_host(src_host)
    want1, want2 = _reference(w, src, flags), _reference(w2, src, flags)
    stream = torch.cuda.Stream()
    # both calls are enqueued before anything is waited for
    got1 = _noalloc(w, src, flags, stream)
    got2 = _noalloc(w2, src, flags, stream)
    stream.synchronize()
    G.assert_bytes_equal(got1.cpu().numpy(), want1, f"{w.name}: first call")
    G.assert_bytes_equal(got2.cpu().numpy(), want2, f"{w.name}: second, smaller call")
    G.assert_bytes_equal(src.cpu().numpy(), src_host, f"{w.name}: source changed")
    if flags == 0:  # and both against the oracle itself
        G.assert_bytes_equal(want1, G.oracle_expected(w, src_host), f"{w.name}: oracle")
        G.assert_bytes_equal(want2, G.oracle_expected(w2, src_host), f"{w2.name}: oracle")


@gpu
def test_noalloc_layer_sub_range_and_no_coalesce():
    w = wl.config2(num_layers=5, pool_blocks=512, tokens=1500)
    w = dataclasses.replace(w, layer_begin=1, layer_end=4)
    src_host = wl.host_pool_values(w.src, w.dtype, w.seed)
    src = G.device_pool_from_host(src_host)
    stream = torch.cuda.Stream()
    for flags in (0, kvd.KVD_PLAN_NO_COALESCE, kvd.KVD_PLAN_QUEUE_ORDER):
        got = _noalloc(w, src, flags, stream)
        stream.synchronize()
        G.assert_bytes_equal(got.cpu().numpy(), G.oracle_expected(w, src_host), f"layers 1..3, flags {flags}")


@gpu
@pytest.mark.parametrize("kind", ["runs", "short-scattered"])
def test_noalloc_recorded_into_a_hip_graph(kind):
    """The call allocates nothing and carries the tables by value, so a recording stream records all of it (the
    table pieces, the build, the region ordering of short transactions, the pull): three replays with eager fills
    between them, each checked against the oracle."""
    w = wl.config2(num_layers=3, pool_blocks=1024, tokens=5000) if kind == "runs" else \
        wl.config4(num_layers=40, pool_blocks=2560, tokens=32768)
    src_host = wl.host_pool_values(w.src, w.dtype, w.seed)
    want = G.oracle_expected(w, src_host)
    src, dst = G.device_pool_from_host(src_host), G.device_sentinel_pool(w.dst)
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    r = w.requests[0]
    sd, dd = kvd.pool_desc(src.data_ptr(), w.src), kvd.pool_desc(dst.data_ptr(), w.dst)

    def call():
        kvd.kvd_pull_noalloc(sd, dd, r.src_table, r.dst_table, r.seq_len, w.layer_begin, w.layer_end, 0, stream.cuda_stream)
    call()  # eager first: the device's copy of the scratch array is looked up outside the recording
    stream.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        call()
    for replay in range(3):
        dst.view(torch.int16).fill_(wl.SENTINEL16)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        G.assert_bytes_equal(dst.cpu().numpy(), want, f"{kind}: replay {replay}")
    del graph


@gpu
def test_noalloc_largest_table_and_refusals():
    """8192 blocks per side is taken (19 pieces of the tables); one more block, or more work items than
    the array holds, is refused with KVD_ERR_CAPACITY before anything is enqueued."""
    g = wl.PoolGeometry(1, 8300, 16, 1, 64, 2, wl.BHTD)
    rng = np.random.default_rng(3)
    n = kvd.KVD_NOALLOC_MAX_BLOCKS
    w = wl.Workload("largest", g, g, [wl.Request(n * 16 - 3, wl.scattered_table(rng, g.num_blocks, n),
                                                 wl.scattered_table(rng, g.num_blocks, n))], "bf16", 3)
    src_host = wl.host_pool_values(g, "bf16", 3)
    src = G.device_pool_from_host(src_host)
    stream = torch.cuda.Stream()
    got = _noalloc(w, src, 0, stream)
    stream.synchronize()
    G.assert_bytes_equal(got.cpu().numpy(), G.oracle_expected(w, src_host), "8192 blocks per side")
    dst = G.device_sentinel_pool(g)
    torch.cuda.synchronize()
    sd, dd = kvd.pool_desc(src.data_ptr(), g), kvd.pool_desc(dst.data_ptr(), g)
    tbl = np.arange(n + 1, dtype=np.int32)
    with pytest.raises(kvd.KvdError) as e:
        kvd.kvd_pull_noalloc(sd, dd, tbl, tbl, (n + 1) * 16, 0, 1, 0, stream.cuda_stream)
    assert e.value.code == kvd.KVD_ERR_CAPACITY and "8192" in str(e.value)
    stream.synchronize()
    assert int((dst.view(torch.int16) != wl.SENTINEL16).sum()) == 0  # nothing was moved


def test_noalloc_validates_on_the_host_before_any_gpu_call():
    """Every refusal comes before the first HIP call, so it can be seen without a GPU."""
    g = wl.PoolGeometry(2, 64, 16, 4, 64, 2, wl.BHTD)
    fake_src, fake_dst = 0x10_0000_0000, 0x20_0000_0000  # never dereferenced
    sd, dd = kvd.pool_desc(fake_src, g), kvd.pool_desc(fake_dst, g)
    ok = np.arange(8, dtype=np.int32)

    def expect(code, *a):
        with pytest.raises(kvd.KvdError) as e:
            kvd.kvd_pull_noalloc(*a)
        assert e.value.code == code, str(e.value)
        return str(e.value)

    expect(kvd.KVD_ERR_INVALID, kvd.pool_desc(0, g), dd, ok, ok, 128, 0, 2)                  # null base
    expect(kvd.KVD_ERR_INVALID, sd, kvd.pool_desc(fake_dst + 8, g), ok, ok, 128, 0, 2)       # misaligned base
    expect(kvd.KVD_ERR_ALIAS, sd, sd, ok, ok, 128, 0, 2)                                     # pools overlap
    expect(kvd.KVD_ERR_MISMATCH, sd, kvd.pool_desc(fake_dst, dataclasses.replace(g, head_dim=128)), ok, ok, 128, 0, 2)
    expect(kvd.KVD_ERR_INVALID, sd, dd, ok, ok, 128, 1, 1)                                   # empty layer range
    expect(kvd.KVD_ERR_RANGE, sd, dd, ok, ok, 128, 0, 3)                                     # layers outside the pool
    expect(kvd.KVD_ERR_RANGE, sd, dd, ok[:7], ok, 128, 0, 2)                                 # table short
    bad = ok.copy(); bad[3] = 64
    expect(kvd.KVD_ERR_RANGE, sd, dd, bad, ok, 128, 0, 2)
    expect(kvd.KVD_ERR_RANGE, sd, dd, ok, bad, 128, 0, 2)
    dup = ok.copy(); dup[5] = dup[2]
    assert "destination block 2" in expect(kvd.KVD_ERR_ALIAS, sd, dd, ok, dup, 128, 0, 2)
    expect(kvd.KVD_ERR_INVALID, sd, dd, ok, ok, 128, 0, 2, kvd.KVD_PLAN_PERSISTENT)          # a flag that does not apply
    # more blocks than the static array's tables hold
    big = dataclasses.replace(g, num_blocks=10000)
    tbl = np.arange(kvd.KVD_NOALLOC_MAX_BLOCKS + 1, dtype=np.int32)
    msg = expect(kvd.KVD_ERR_CAPACITY, kvd.pool_desc(fake_src, big), kvd.pool_desc(fake_dst, big), tbl, tbl, len(tbl) * 16, 0, 2)
    assert str(kvd.KVD_NOALLOC_MAX_BLOCKS) in msg
    # more work items than it holds: 8192 blocks of 512 KiB per (layer, K/V) are a million items of 4 KiB
    fat = wl.PoolGeometry(1, 8192, 256, 8, 128, 2, wl.BHTD)
    tbl = np.arange(8192, dtype=np.int32)
    msg = expect(kvd.KVD_ERR_CAPACITY, kvd.pool_desc(fake_src, fat), kvd.pool_desc(fake_src + (1 << 40), fat), tbl, tbl, 8192 * 256, 0, 1)
    assert str(kvd.KVD_NOALLOC_MAX_WORK_ITEMS) in msg
    # nothing to move: succeeds without touching a GPU
    kvd.kvd_pull_noalloc(sd, dd, ok, ok, 0, 0, 2)
    if not torch.cuda.is_available():
        assert "hip" in expect(kvd.KVD_ERR_HIP, sd, dd, ok, ok, 128, 0, 2).lower()
