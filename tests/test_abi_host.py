"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol
the header declares, and rejects bad arguments before anything is launched."""
import ctypes
import os
import re
import subprocess

import numpy as np
import pytest

from paper_2501_14743_amd import kvd
from paper_2501_14743_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE_SRC = 0x10_0000_0000  # never dereferenced: no kernel is launched in this file
FAKE_DST = 0x20_0000_0000


def header_functions():
    text = open(os.path.join(ROOT, "include", "kvd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(kvd_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = header_functions()
    assert {"kvd_pool_create", "kvd_plan_create", "kvd_build_descriptors", "kvd_pull", "kvd_free",
            "kvd_last_error"} <= set(names)
    L = kvd.lib()
    for n in names:
        assert hasattr(L, n), n


def test_binding_mirrors_every_declared_symbol():
    for n in header_functions():
        assert callable(getattr(kvd, n)), n


def geom(**kw):
    base = dict(num_layers=2, num_blocks=64, block_tokens=16, num_kv_heads=4, head_dim=64, elem_bytes=2,
                layout=wl.BHTD)
    base.update(kw)
    return wl.PoolGeometry(**base)


def expect(code, fn, *a, **k):
    with pytest.raises(kvd.KvdError) as e:
        fn(*a, **k)
    assert e.value.code == code, str(e.value)
    assert kvd.kvd_last_error() != ""
    return str(e.value)


def test_pool_create_rejects_bad_metadata():
    g = geom()
    expect(kvd.KVD_ERR_INVALID, kvd.Pool, 0, g)                       # null base
    expect(kvd.KVD_ERR_INVALID, kvd.Pool, FAKE_SRC + 8, g)            # misaligned base
    expect(kvd.KVD_ERR_INVALID, kvd.Pool, FAKE_SRC, geom(head_dim=4))  # 8-byte rows
    expect(kvd.KVD_ERR_INVALID, kvd.Pool, FAKE_SRC, geom(num_kv_heads=0))
    expect(kvd.KVD_ERR_INVALID, kvd.Pool, FAKE_SRC, geom(elem_bytes=3))
    expect(kvd.KVD_ERR_INVALID, kvd.Pool, FAKE_SRC, g, stride_block=g.tile_elems - 8)
    expect(kvd.KVD_ERR_INVALID, kvd.Pool, FAKE_SRC, geom(block_tokens=2048))
    # axes that overlap: V of a block on top of the next block's K; layers closer than one layer's extent
    expect(kvd.KVD_ERR_INVALID, kvd.Pool, FAKE_SRC, g, g.stride_layer, g.tile_elems, g.tile_elems)
    expect(kvd.KVD_ERR_INVALID, kvd.Pool, FAKE_SRC, g, g.stride_kv, g.stride_kv, g.stride_block)
    # any nesting order of the three axes is fine: blocks outermost, then layers, then K/V
    kvd.Pool(FAKE_SRC, g, 2 * g.tile_elems, g.tile_elems, 2 * g.num_layers * g.tile_elems).close()
    expect(kvd.KVD_ERR_INVALID, kvd.kvd_pool_create, FAKE_SRC, 2, 64, 16, 4, 64, 2, 7, 1 << 20, 1 << 19, 4096)
    expect(kvd.KVD_ERR_RANGE, kvd.Pool, FAKE_SRC, geom(num_blocks=1 << 30, head_dim=2048, num_kv_heads=64))  # 2^53 bytes
    expect(kvd.KVD_ERR_RANGE, kvd.Pool, FAKE_SRC, g, g.stride_layer, g.stride_kv, 1 << 35)       # 64 GiB between blocks
    expect(kvd.KVD_ERR_RANGE, kvd.Pool, FAKE_SRC, g, 1 << 44, g.stride_kv, g.stride_block)   # absurd stride
    # a block axis whose size wraps around 64 bits must not slip under the limit: 2^29 + 1 blocks, 2^35 bytes apart
    expect(kvd.KVD_ERR_RANGE, kvd.Pool, FAKE_SRC, geom(num_blocks=(1 << 29) + 1), 0, 0, 1 << 34)
    expect(kvd.KVD_ERR_RANGE, kvd.Pool, FAKE_SRC, geom(num_blocks=(1 << 32) - 1), 1 << 43, 1 << 42, 1 << 34)
    p = kvd.Pool(FAKE_SRC, g)
    assert p.handle
    p.close()
    kvd.kvd_free(None)


def test_plan_create_rejects_mismatch_and_overlap():
    g = geom()
    s, d = kvd.Pool(FAKE_SRC, g), kvd.Pool(FAKE_DST, g)
    expect(kvd.KVD_ERR_MISMATCH, kvd.Plan, s, kvd.Pool(FAKE_DST, geom(num_kv_heads=2)), 1, 8)
    expect(kvd.KVD_ERR_MISMATCH, kvd.Plan, s, kvd.Pool(FAKE_DST, geom(head_dim=128)), 1, 8)
    expect(kvd.KVD_ERR_MISMATCH, kvd.Plan, s, kvd.Pool(FAKE_DST, geom(elem_bytes=4)), 1, 8)
    expect(kvd.KVD_ERR_MISMATCH, kvd.Plan, s, kvd.Pool(FAKE_DST, geom(block_tokens=24)), 1, 8)
    expect(kvd.KVD_ERR_ALIAS, kvd.Plan, s, s, 1, 8)
    expect(kvd.KVD_ERR_ALIAS, kvd.Plan, s, kvd.Pool(FAKE_SRC + g.total_bytes - 4096, g), 1, 8)
    expect(kvd.KVD_ERR_MISMATCH, kvd.Plan, s, kvd.Pool(FAKE_DST, geom(block_tokens=32, num_blocks=32)), 1, 8,
           kvd.KVD_PLAN_WHOLE_BLOCKS)
    expect(kvd.KVD_ERR_INVALID, kvd.Plan, s, d, 0, 8)
    expect(kvd.KVD_ERR_CAPACITY, kvd.Plan, s, d, 1, (1 << 32) - 1)                      # more blocks than any launch could take
    expect(kvd.KVD_ERR_CAPACITY, kvd.Plan, kvd.Pool(FAKE_SRC, geom(num_kv_heads=1 << 10, block_tokens=1 << 10, head_dim=2048, num_blocks=2)),
           kvd.Pool(FAKE_SRC + (1 << 44), geom(num_kv_heads=1 << 10, block_tokens=1, head_dim=2048, num_blocks=2)), (1 << 32) - 1, (1 << 32) - 1)
    expect(kvd.KVD_ERR_INVALID, kvd.Plan, s, d, 1, 0)
    # touching but not overlapping is fine
    kvd.Plan(s, kvd.Pool(FAKE_SRC + g.total_bytes, g), 1, 8).close()
    # a slab of 512 GiB is a legal pool, but only block-major pools on both sides can use one in a plan
    big = geom(num_blocks=1 << 24, head_dim=128, num_kv_heads=8)
    big_bm = geom(num_blocks=1 << 24, head_dim=128, num_kv_heads=8, block_major=True)
    far = FAKE_SRC + (1 << 44)
    expect(kvd.KVD_ERR_RANGE, kvd.Plan, kvd.Pool(FAKE_SRC, big), kvd.Pool(far, big), 1, 8)
    expect(kvd.KVD_ERR_RANGE, kvd.Plan, kvd.Pool(FAKE_SRC, big_bm), kvd.Pool(far, big), 1, 8)
    kvd.Plan(kvd.Pool(FAKE_SRC, big_bm), kvd.Pool(far, big_bm), 1, 8).close()
    expect(kvd.KVD_ERR_MISMATCH, kvd.Plan, kvd.Pool(FAKE_SRC, big_bm), kvd.Pool(far, big_bm), 1, 8, kvd.KVD_PLAN_PERSISTENT)
    expect(kvd.KVD_ERR_MISMATCH, kvd.Plan, s, d, 1, 8, kvd.KVD_PLAN_WIDE_OFFSETS)                 # not block-major
    with pytest.raises(kvd.KvdError):
        kvd.kvd_plan_create(s.handle, 0, 1, 8)


def test_released_and_foreign_handles_are_refused_without_being_read():
    g = geom()
    s, d = kvd.Pool(FAKE_SRC, g), kvd.Pool(FAKE_DST, g)
    plan = kvd.kvd_plan_create(s.handle, d.handle, 1, 8)
    kvd.kvd_free(plan)
    kvd.kvd_free(plan)                                    # second release: ignored
    expect(kvd.KVD_ERR_INVALID, kvd.kvd_pull, plan)       # a released plan is no plan
    expect(kvd.KVD_ERR_INVALID, kvd.kvd_plan_reset, plan)
    old_pool = s.handle
    s.close()
    expect(kvd.KVD_ERR_INVALID, kvd.kvd_plan_create, old_pool, d.handle, 1, 8)
    kvd.kvd_free(old_pool)
    # memory that never was a handle, whatever it holds, and an address that is not mapped at all
    fake = (ctypes.c_uint32 * 64)(*([0x6b76504c] * 64))   # looks like a plan's tag
    kvd.kvd_free(ctypes.addressof(fake))
    expect(kvd.KVD_ERR_INVALID, kvd.kvd_pull, ctypes.addressof(fake))
    kvd.kvd_free(0x10)
    expect(kvd.KVD_ERR_INVALID, kvd.kvd_pull, 0x10)
    # a pool handle where a plan is expected
    expect(kvd.KVD_ERR_INVALID, kvd.kvd_pull, d.handle)


def test_pull_notify_and_probe_refusals_need_no_gpu():
    g = geom()
    s, d = kvd.Pool(FAKE_SRC, g), kvd.Pool(FAKE_DST, g)
    words = np.zeros(4, np.int64)
    plain = kvd.Plan(s, d, 2, 8)
    expect(kvd.KVD_ERR_MISMATCH, plain.pull_notify, words.ctypes.data, 1)       # plan without per-request completion
    per_request = kvd.Plan(s, d, 2, 8, kvd.KVD_PLAN_COMPLETE_PER_REQUEST)
    per_request.pull_notify(words.ctypes.data, 1)                               # empty plan: nothing to announce
    expect(kvd.KVD_ERR_MISMATCH, kvd.Plan(s, d, 2, 8, kvd.KVD_PLAN_COMPLETE_PER_REQUEST | kvd.KVD_PLAN_PERSISTENT).pull_notify,
           words.ctypes.data, 1)
    expect(kvd.KVD_ERR_INVALID, kvd.kvd_pull_notify, 0x10, words.ctypes.data, 1)  # not a plan
    expect(kvd.KVD_ERR_INVALID, kvd.Plan, s, d, 2, 8, 128)                       # unknown flag bit
    expect(kvd.KVD_ERR_INVALID, kvd.Plan, s, d, 2, 8, kvd.KVD_PLAN_QUEUE_ORDER | kvd.KVD_PLAN_DESTINATION_ORDER)
    kvd.Plan(s, d, 2, 8, kvd.KVD_PLAN_DESTINATION_ORDER).close()
    expect(kvd.KVD_ERR_MISMATCH, plain.set_completion_granularity, 1024)         # no completions to group
    per_request.set_completion_granularity(1024)
    per_request.set_completion_granularity(0)
    expect(kvd.KVD_ERR_INVALID, kvd.kvd_plan_set_completion_granularity, 0x10, 1)
    expect(kvd.KVD_ERR_INVALID, kvd.kvd_stream_probe, FAKE_DST, FAKE_SRC, 4095, "copy")
    expect(kvd.KVD_ERR_INVALID, kvd.kvd_stream_probe, FAKE_DST, FAKE_SRC, 4096, 6)
    expect(kvd.KVD_ERR_INVALID, kvd.kvd_stream_probe, 0, FAKE_SRC, 4096, "read")


def test_build_descriptors_validates_before_launching():
    g = geom()
    s, d = kvd.Pool(FAKE_SRC, g), kvd.Pool(FAKE_DST, g)
    plan = kvd.Plan(s, d, 2, 8)
    ok = np.arange(8, dtype=np.int32)
    expect(kvd.KVD_ERR_INVALID, plan.build_descriptors, ok, ok, 128, 1, 1)        # empty layer range
    expect(kvd.KVD_ERR_INVALID, plan.build_descriptors, ok, ok, 128, 2, 1)
    expect(kvd.KVD_ERR_RANGE, plan.build_descriptors, ok, ok, 128, 0, 3)          # layers outside pool
    expect(kvd.KVD_ERR_RANGE, plan.build_descriptors, ok[:7], ok, 128, 0, 2)      # source table short
    expect(kvd.KVD_ERR_RANGE, plan.build_descriptors, ok, ok[:7], 113, 0, 2)      # destination table short
    bad = ok.copy(); bad[3] = 64
    expect(kvd.KVD_ERR_RANGE, plan.build_descriptors, bad, ok, 128, 0, 2)
    bad[3] = -1
    expect(kvd.KVD_ERR_RANGE, plan.build_descriptors, ok, bad, 128, 0, 2)
    dup = ok.copy(); dup[5] = dup[2]
    msg = expect(kvd.KVD_ERR_ALIAS, plan.build_descriptors, ok, dup, 128, 0, 2)   # destination block twice
    assert "destination block 2" in msg
    expect(kvd.KVD_ERR_CAPACITY, plan.build_descriptors, np.arange(9), np.arange(9), 144, 0, 2)
    expect(kvd.KVD_ERR_RANGE, plan.build_descriptors, ok, ok, (1 << 30) + 1, 0, 2)  # seq_len beyond the limit
    # entries beyond ceil(seq_len / block_tokens) are ignored, even invalid ones
    long_tbl = np.array([0, 1, 99999], dtype=np.int32)
    # seq_len 0 appends nothing and succeeds, whatever the tables hold
    plan.build_descriptors(long_tbl, long_tbl, 0, 0, 2)
    assert plan.stats()["num_requests"] == 0
    # a pull of an empty plan is a no-op
    plan.pull()
    plan.reset()
    with pytest.raises(kvd.KvdError):
        kvd.kvd_pull(0)


def test_batch_is_all_or_nothing():
    g = geom()
    plan = kvd.Plan(kvd.Pool(FAKE_SRC, g), kvd.Pool(FAKE_DST, g), 4, 32)
    a, b = np.arange(0, 4, dtype=np.int32), np.arange(4, 8, dtype=np.int32)
    # second request reuses a destination block of the first: nothing is appended, marks are undone
    msg = expect(kvd.KVD_ERR_ALIAS, plan.build_descriptors_batch, [a, b], [a, np.array([4, 5, 2, 7], np.int32)],
                 [64, 64], 0, 2)
    assert "request 1" in msg
    msg = expect(kvd.KVD_ERR_RANGE, plan.build_descriptors_batch, [a, b], [a, np.array([4, 5, 64, 7], np.int32)],
                 [64, 64], 0, 2)
    assert "request 1" in msg
    expect(kvd.KVD_ERR_RANGE, plan.build_descriptors_batch, [a, b[:3]], [a, b], [64, 64], 0, 2)
    expect(kvd.KVD_ERR_CAPACITY, plan.build_descriptors_batch, [a] * 5, [a, b, a + 8, a + 12, a + 16], [64] * 5, 0, 2)
    assert plan.stats()["num_requests"] == 0
    # zero-length requests are skipped, an all-empty batch succeeds without a GPU
    plan.build_descriptors_batch([a, b], [a, b], [0, 0], 0, 2)
    plan.build_descriptors_batch([], [], [], 0, 2)
    import torch
    if not torch.cuda.is_available():
        # a valid batch gets as far as the GPU allocation and leaves no marks behind
        expect(kvd.KVD_ERR_HIP, plan.build_descriptors_batch, [a, b], [a, b], [64, 64], 0, 2)
        expect(kvd.KVD_ERR_HIP, plan.build_descriptors_batch, [a, b], [a, b], [64, 64], 0, 2)


def test_valid_build_needs_a_gpu_and_says_so():
    import torch
    if torch.cuda.is_available():
        pytest.skip("GPU present: covered by the gpu tests")
    g = geom()
    plan = kvd.Plan(kvd.Pool(FAKE_SRC, g), kvd.Pool(FAKE_DST, g), 2, 8)
    ok = np.arange(8, dtype=np.int32)
    msg = expect(kvd.KVD_ERR_HIP, plan.build_descriptors, ok, ok, 128, 0, 2)
    assert "hip" in msg.lower()
    # the failed call left no trace: the same destination blocks can be used again
    expect(kvd.KVD_ERR_HIP, plan.build_descriptors, ok, ok, 128, 0, 2)


def test_host_checks_survive_random_arguments():
    """3000 calls with arguments drawn from edge values (zero, huge, misaligned, negative, inconsistent): every one
    returns a documented status, with a message on failure, and nothing is dereferenced or launched.  Without a GPU a
    call that passes every check fails at its first HIP call; on a machine with one it would move bytes between the
    fake pool addresses, so the calls that could get that far are left out there.  A crash of the process is the
    failure this test is for."""
    import torch
    rng = np.random.default_rng(20250114)
    edge32 = [0, 1, 2, 3, 15, 16, 17, 64, 255, 1024, 1025, 32767, 32768, 1 << 20, (1 << 31) - 1, 1 << 31, (1 << 32) - 1]
    edge64 = [-1, 0, 1, 8, 16, 24, 4096, 1 << 20, 1 << 35, (1 << 36) - 16, 1 << 36, 1 << 43, 1 << 44, (1 << 62)]
    codes = {kvd.KVD_OK, kvd.KVD_ERR_INVALID, kvd.KVD_ERR_RANGE, kvd.KVD_ERR_MISMATCH, kvd.KVD_ERR_ALIAS,
             kvd.KVD_ERR_CAPACITY, kvd.KVD_ERR_HIP}

    def pick(values):
        return int(values[int(rng.integers(len(values)))])

    def random_desc(base):
        if rng.random() < 0.8:  # a sane pool, mostly with one field disturbed
            g = geom()
            f = [base, g.num_layers, g.num_blocks, g.block_tokens, g.num_kv_heads, g.head_dim, g.elem_bytes, 0,
                 g.stride_layer, g.stride_kv, g.stride_block]
            if rng.random() < 0.7:
                k = int(rng.integers(len(f)))
                f[k] = pick(edge64 if k in (0, 8, 9, 10) else edge32)
        else:
            f = [pick([0, 8, 16, base]), pick(edge32), pick(edge32), pick(edge32), pick(edge32), pick(edge32),
                 pick([0, 1, 2, 3, 4, 8, 16]), pick([0, 1, 2, 7]), pick(edge64), pick(edge64), pick(edge64)]
        f[7] = f[7] % (1 << 31)
        return kvd.kvd_pool_desc_t(*f)

    L = kvd.lib()
    have_gpu = torch.cuda.is_available()
    accepted = 0
    for _ in range(3000):
        sd, dd = random_desc(FAKE_SRC), random_desc(FAKE_DST)
        ps, pd = ctypes.c_void_p(), ctypes.c_void_p()
        rs = L.kvd_pool_create(ctypes.byref(sd), ctypes.byref(ps))
        rd = L.kvd_pool_create(ctypes.byref(dd), ctypes.byref(pd))
        for rc in (rs, rd):
            assert rc in codes and (rc == kvd.KVD_OK or kvd.kvd_last_error())
        n = int(rng.integers(0, 12))
        st = np.asarray(rng.integers(-3, 80, size=n), np.int32)
        dt = np.asarray(rng.integers(-3, 80, size=n), np.int32)
        seq, l0, l1 = pick([0, 1, 15, 16, 17, 100, 1 << 30, (1 << 32) - 1]), pick([0, 1, 2, 5]), pick([0, 1, 2, 3, 1 << 20])
        i32p = ctypes.POINTER(ctypes.c_int32)
        if not have_gpu:  # with a GPU a call that passes every check would move bytes between fake addresses
            rc = L.kvd_pull_noalloc(ctypes.byref(sd), ctypes.byref(dd), st.ctypes.data_as(i32p), n, dt.ctypes.data_as(i32p), n,
                                    seq, l0, l1, pick([0, 1, 4, 8, 2, 64]), None)
            assert rc in codes and (rc == kvd.KVD_OK or kvd.kvd_last_error())
        if rs == kvd.KVD_OK and rd == kvd.KVD_OK:
            plan = ctypes.c_void_p()
            rc = L.kvd_plan_create(ps, pd, pick([0, 1, 4, (1 << 32) - 1]), pick([0, 1, 16, 1 << 20, (1 << 32) - 1]),
                                   pick([0, 1, 2, 4, 8, 16, 32, 63]), ctypes.byref(plan))
            assert rc in codes and (rc == kvd.KVD_OK or kvd.kvd_last_error())
            if rc == kvd.KVD_OK:
                accepted += 1
                if not have_gpu:
                    rc = L.kvd_build_descriptors(plan, st.ctypes.data_as(i32p), n, dt.ctypes.data_as(i32p), n, seq, l0, l1, None)
                    assert rc in codes and (rc == kvd.KVD_OK or kvd.kvd_last_error())
                assert L.kvd_pull(plan, None) in codes
                assert L.kvd_plan_reset(plan) in codes
                L.kvd_free(plan)
        L.kvd_free(ps)
        L.kvd_free(pd)
    assert accepted > 50, accepted  # the draw does reach the deeper checks


C_PROGRAM = r"""
#include <stdio.h>
#include <string.h>
#include "kvd.h"
int main(void)
{
    kvd_pool_desc_t d;
    kvd_pool_t *src = NULL, *dst = NULL;
    kvd_plan_t *plan = NULL;
    kvd_stats_t st;
    int32_t tbl[4] = {0, 1, 2, 99};
    memset(&d, 0, sizeof d);
    if (kvd_pool_create(&d, &src) != KVD_ERR_INVALID || kvd_last_error()[0] == 0) return 1;
    d.base = (void *)0x100000000ull; d.num_layers = 2; d.num_blocks = 8; d.block_tokens = 16;
    d.num_kv_heads = 2; d.head_dim = 64; d.elem_bytes = 2; d.layout = KVD_LAYOUT_BHTD;
    d.stride_block = 16 * 2 * 64; d.stride_kv = 8 * d.stride_block; d.stride_layer = 2 * d.stride_kv;
    if (kvd_pool_create(&d, &src) != KVD_OK) return 2;
    d.base = (void *)0x200000000ull;
    if (kvd_pool_create(&d, &dst) != KVD_OK) return 3;
    if (kvd_plan_create(src, dst, 4, 16, KVD_PLAN_NO_COALESCE, &plan) != KVD_OK) return 4;
    kvd_free(src); kvd_free(dst);                       /* the plan keeps its own copy of the metadata */
    if (kvd_build_descriptors(plan, tbl, 4, tbl, 4, 64, 0, 2, NULL) != KVD_ERR_RANGE) return 5;
    if (kvd_build_descriptors(plan, tbl, 4, tbl, 4, 0, 0, 2, NULL) != KVD_OK) return 6;
    if (kvd_pull(plan, NULL) != KVD_OK) return 7;       /* empty plan: nothing to launch */
    if (kvd_plan_stats(plan, NULL, &st) != KVD_OK || st.num_requests != 0) return 8;
    if (kvd_plan_reset(plan) != KVD_OK) return 9;
    kvd_free(plan); kvd_free(NULL);
    printf("ok %s\n", kvd_last_error());
    return 0;
}
"""


def test_header_is_plain_c_and_usable_from_c(tmp_path):
    src, exe = tmp_path / "abi.c", tmp_path / "abi"
    src.write_text(C_PROGRAM)
    pkg = os.path.join(ROOT, "paper_2501_14743_amd")
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                           str(src), "-o", str(exe), "-L", pkg, "-lkvd", f"-Wl,-rpath,{pkg}",
                           "-Wl,-rpath,/opt/rocm/lib"])
    out = subprocess.run([str(exe)], capture_output=True, text=True, timeout=120)
    assert out.returncode == 0, (out.returncode, out.stdout, out.stderr)
    assert out.stdout.startswith("ok")


def test_product_path_never_touches_the_oracle():
    """The oracle is test infrastructure: nothing in the package or the header may name it, and
    the oracle may not name the package's library either."""
    pkg = os.path.join(ROOT, "paper_2501_14743_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower() or f == "workloads.py" and "import" not in \
                    [ln for ln in text.splitlines() if "oracle" in ln.lower()][0], f
    assert "oracle" not in open(os.path.join(ROOT, "include", "kvd.h")).read().lower()
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "libkvd.so" not in text and "paper_2501_14743_amd" not in text, f


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(kvd, "_lib", None)
    monkeypatch.setattr(kvd, "LIB_PATH", "/nonexistent/libkvd.so")
    with pytest.raises(RuntimeError, match="no fallback"):
        kvd.kvd_pull(1)


def test_bench_refuses_more_than_one_gpu():
    """bench.py is a one-GPU benchmark: with --gpus above 1 it says so and exits before touching a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout.strip() == ""
