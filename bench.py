#!/usr/bin/env python3
"""Benchmark of the paged KV-cache pull on one MI355X.

One "step" is one pass of the whole transfer path for one batch of synthetic requests:
reset the plan, translate + coalesce every request's block tables (kvd_build_descriptors),
and move the bytes (kvd_pull).  Pools and their contents are resident in HBM before the
timed region starts.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2]
"""
from __future__ import annotations

import argparse
import dataclasses
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def _checker():
    """The CPU oracle's test glue (tests/): loaded only by the cpu_baseline leg and by the check of
    the result after the timed steps, never by the timed path."""
    tests = os.path.join(ROOT, "tests")
    if tests not in sys.path:
        sys.path.insert(0, tests)

PEAK_HBM_GBPS = 8000.0  # MI355X published HBM3E bandwidth
METRIC = "achieved HBM GB/s (% of peak) for paged KV pull; µs per 8K-token request"


def log(msg: str) -> None:
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def _one_layer_workload(cfg_no: int):
    from paper_2501_14743_amd import workloads as wl
    full = wl.CONFIGS[cfg_no]()
    gs, gd = (wl.PoolGeometry(1, g.num_blocks, g.block_tokens, g.num_kv_heads, g.head_dim, g.elem_bytes, g.layout)
              for g in (full.src, full.dst))
    w = wl.Workload(full.name, gs, gd, full.requests, full.dtype, full.seed)
    payload = w.total_tokens * 2 * gs.num_kv_heads * gs.head_dim * gs.elem_bytes
    return full, w, payload


def _oracle_worker(cfg_no: int, reps: int, barrier, out) -> None:
    """One host core's share of the all-core leg: the oracle on one layer (K and V) of the workload,
    on pools of this process's own."""
    import numpy as np
    _checker()
    import kvd_testlib as tl
    _, w, _ = _one_layer_workload(cfg_no)
    src = np.ones(w.src.total_bytes, np.uint8)
    dst = np.empty(w.dst.total_bytes, np.uint8)
    tl.oracle_pull_workload(w, src, dst)  # untimed: pages in what the pull touches
    barrier.wait()
    t0 = time.perf_counter()
    for _ in range(reps):
        tl.oracle_pull_workload(w, src, dst)
    out.put(time.perf_counter() - t0)


def host_cores() -> int:
    """Cores this process may use: its affinity mask, capped by the thread count the environment
    sets for this process's share of the host (OMP_NUM_THREADS), at most 16."""
    n = len(os.sched_getaffinity(0))
    try:
        n = min(n, int(os.environ.get("OMP_NUM_THREADS", n)))
    except ValueError:
        pass
    return max(1, min(n, 16))


def cpu_baseline(cfg_no: int, budget_s: float = 10.0) -> dict:
    """Time the oracle as it stands on a bounded sample of the workload: one layer (K and V), repeated
    until about `budget_s` seconds of work have been spent, first on one core, then on all host cores
    at once (one worker process per core, each moving one layer on pools of its own: the layers of a
    request share its block tables, so every worker does what one layer of the workload costs).
    Must run before this process touches the GPU: the workers are forked."""
    import multiprocessing as mp
    import numpy as np
    _checker()
    import kvd_testlib as tl

    full, w, payload = _one_layer_workload(cfg_no)
    src = np.ones(w.src.total_bytes, np.uint8)
    dst = np.empty(w.dst.total_bytes, np.uint8)
    t0 = time.perf_counter()
    tl.oracle_pull_workload(w, src, dst)
    first = time.perf_counter() - t0
    reps = max(1, min(256, int(budget_s / max(first, 1e-3))))
    t0 = time.perf_counter()
    for _ in range(reps):
        tl.oracle_pull_workload(w, src, dst)
    dt = (time.perf_counter() - t0) / reps
    del src, dst
    one = 2 * payload / dt / 1e9

    cores = host_cores()
    ctx = mp.get_context("fork")
    barrier, out = ctx.Barrier(cores), ctx.Queue()
    procs = [ctx.Process(target=_oracle_worker, args=(cfg_no, reps, barrier, out)) for _ in range(cores)]
    for p in procs:
        p.start()
    times = [out.get(timeout=600) for _ in procs]
    for p in procs:
        p.join()
    all_cores = cores * reps * 2 * payload / max(times) / 1e9
    return {
        "value": all_cores, "unit": "GB/s", "cores": cores, "kind": "oracle",
        "sample": f"one layer (K and V) of {full.name} per core: {w.total_tokens} tokens, {payload} payload bytes, "
                  f"{reps} passes per worker process after one untimed pass, {cores} worker processes at once "
                  f"(slowest worker's time); host shows {os.cpu_count()} cpus, affinity {len(os.sched_getaffinity(0))}",
        "one_core": {"value": one, "unit": "GB/s", "cores": 1, "seconds_per_layer": dt},
        "seconds_per_layer_all_cores_busy": max(times) / reps,
    }


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=2, choices=[1, 2, 3, 4, 5])
    ap.add_argument("--event-stride", type=int, default=4,
                    help="HIP events bracket the pull kernel of every n-th timed step (an event record sits on the "
                         "GPU's queue between the build and the pull and costs that step a few microseconds)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-gc-freeze", action="store_true",
                    help="leave the objects alive before the timed region in the garbage collector's sight (shows the "
                         "pause of a full collection as the longest step)")
    ap.add_argument("--no-extras", action="store_true", help="skip the reported GPU baselines")
    ap.add_argument("--no-slow-baselines", action="store_true",
                    help="skip the staged and the per-block memcpy baselines (hundreds of thousands of launches)")
    ap.add_argument("--per-layer", action="store_true",
                    help="also time the transfer issued one layer per launch, alone and next to GEMMs")
    ap.add_argument("--run-length-sweep", action="store_true",
                    help="also time the pull of the same token count with block tables made of runs of exactly "
                         "1, 2, 4, ... consecutive blocks (both sides, source only, destination only)")
    ap.add_argument("--locality-sweep", action="store_true",
                    help="also time the pull of lone blocks whose queue neighbours are a fixed distance apart, and of lone "
                         "blocks queued in address order of one or both sides")
    ap.add_argument("--size-sweep", action="store_true",
                    help="also time the pull of 1/8 ... 2x the configuration's token count (configurations 2 and 4), "
                         "the bandwidth-against-transfer-size curve of the paper's motivation")
    ap.add_argument("--block-size-sweep", action="store_true",
                    help="also time the pull of 1024 and 2048 lone blocks of 4 ... 128 KiB per (layer, K/V) (one KV head of "
                         "128 bf16 values, 16 ... 512 tokens per block) in the configuration's pool memory: the "
                         "bandwidth-against-block-size curve of the paper's motivation")
    ap.add_argument("--order-ab", action="store_true",
                    help="also time a range of fragmented workloads (lone blocks, short runs, batches of short requests, in "
                         "the configuration's pool memory) as the library orders their work items and in queue order")
    ap.add_argument("--lone-blocks", action="store_true",
                    help="replace the configuration's block tables by tables in which every block is alone on both sides")
    ap.add_argument("--block-major", action="store_true",
                    help="describe the same pool memory as [block][layer][K/V] pools")
    ap.add_argument("--stream-probes", action="store_true",
                    help="also time read-only, write-only and copy streams over plain 1 GiB buffers, dispatched in address "
                         "order and from a persistent grid (the measurements behind the pull kernel's design)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also launch the plain copy kernel a few times (for counter calibration runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this benchmark runs on ONE GPU only (both pools live in one MI355X's HBM); "
              "run with --gpus 1", file=sys.stderr)
        return 2

    # the CPU leg runs first: its worker processes are forked, which must happen before this
    # process touches the GPU, and it must not share the host with the timed GPU steps
    cpu = None
    if not args.no_cpu_baseline:
        log("timing the oracle on the host (one core, then all cores)")
        cpu = cpu_baseline(args.config)
        log(f"oracle: {cpu['one_core']['value']:.2f} GB/s on one core, {cpu['value']:.2f} GB/s on {cpu['cores']} cores")

    import numpy as np
    import torch
    from paper_2501_14743_amd import kvd, workloads as wl
    from paper_2501_14743_amd import device as G

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    kvd.lib()  # fail now if the library is missing
    torch.cuda.set_device(0)
    w = wl.CONFIGS[args.config]()
    if args.lone_blocks or args.block_major:
        # variants of a single-request configuration for diagnosis: the same pools and token count with every
        # block alone on both sides, and/or the same memory described as [block][layer][K/V] pools

        assert len(w.requests) == 1, "--lone-blocks / --block-major are for the single-request configurations"
        gs, gd, r = w.src, w.dst, w.requests[0]
        name = w.name
        if args.block_major:
            gs, gd = dataclasses.replace(gs, block_major=True), dataclasses.replace(gd, block_major=True)
            name += "-block-major"
        if args.lone_blocks:
            rng = np.random.default_rng(w.seed + 3000)
            r = wl.Request(r.seq_len, wl.fixed_run_table(rng, gs.num_blocks, wl.blocks_for(r.seq_len, gs.block_tokens), 1),
                           wl.fixed_run_table(rng, gd.num_blocks, wl.blocks_for(r.seq_len, gd.block_tokens), 1))
            name += "-lone-blocks"
        w = wl.Workload(name, gs, gd, [r], w.dtype, w.seed, w.layer_begin, w.layer_end)
    log(f"{w.name}: pools {w.src.total_bytes / 2**30:.2f} + {w.dst.total_bytes / 2**30:.2f} GiB, "
        f"{len(w.requests)} requests, {w.total_tokens} tokens")
    src = G.device_random_pool(w.src, w.dtype, w.seed)
    dst = G.device_sentinel_pool(w.dst)
    stream = torch.cuda.Stream()
    x = G.GpuTransfer(w, src, dst, stream=stream)
    sh = stream.cuda_stream

    batch = len(w.requests) > 1  # several requests are appended with the one batched call

    calls = np.zeros((max(args.steps, 1), 3))  # host time inside reset / build / pull of every timed step
    clock = time.perf_counter

    def step(ev=None, i=None):
        t0 = clock()
        x.plan.reset()
        t1 = clock()
        x.build(batch)
        t2 = clock()
        if ev is not None:
            ev[0].record(stream)
        x.plan.pull(sh)
        if ev is not None:
            ev[1].record(stream)
        if i is not None:
            calls[i] = (t1 - t0, t2 - t1, clock() - t2)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # CPython's cyclic garbage collector belongs to this harness, not to the library: a full
    # collection over the million objects that torch and numpy keep alive takes tens of milliseconds
    # and would land on whichever step's allocations trigger it.  Everything alive now is moved out
    # of the collector's sight; collections that still happen inside the timed region are timed by
    # a callback and reported.
    if not args.no_gc_freeze:
        gc.collect()
        gc.freeze()
    gc_pauses = []

    def on_gc(phase, info, _start=[0.0]):
        if phase == "start":
            _start[0] = time.perf_counter()
        else:
            gc_pauses.append((info["generation"], (time.perf_counter() - _start[0]) * 1e3))
    gc.callbacks.append(on_gc)
    stride = max(1, args.event_stride)
    events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
              for _ in range(0, args.steps, stride)]
    torch.cuda.synchronize()
    returned = np.empty(args.steps + 1)  # when each step's calls returned to the host
    t0 = returned[0] = time.perf_counter()
    for i in range(args.steps):
        step(events[i // stride] if i % stride == 0 else None, i)
        returned[i + 1] = time.perf_counter()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    gc.callbacks.remove(on_gc)
    # host time per step: in the steady state the host waits in kvd_plan_reset for the previous
    # step's build, so this follows the GPU's step time; an outlier is a call that blocked
    host_us = np.diff(returned) * 1e6
    stats = x.plan.stats(sh)  # of the last step's plan
    payload = stats["payload_bytes"]
    pull_ms = np.array([a.elapsed_time(b) for a, b in events])
    ms_per_step = elapsed / args.steps * 1e3
    value = 2 * payload * args.steps / elapsed / 1e9
    achieved = 2 * payload / (pull_ms.mean() * 1e-3) / 1e9
    log(f"step {ms_per_step * 1e3:.1f} us, pull kernel mean {pull_ms.mean() * 1e3:.1f} us "
        f"(min {pull_ms.min() * 1e3:.1f}), {achieved:.0f} GB/s = {achieved / PEAK_HBM_GBPS:.1%} of peak")
    # what the bracket itself costs: two event records with nothing between them, behind a kernel like in a step
    # (reported beside the kernel time, not subtracted from it)
    empty = []
    for _ in range(20):
        x.plan.reset()
        x.build(batch)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        e1.record(stream)
        torch.cuda.synchronize()
        empty.append(e0.elapsed_time(e1) * 1e3)
    event_pair_us = float(np.mean(empty))

    # the timed work produced the right bytes: oracle on the first and the last layer
    _checker()
    import kvd_gpu
    check_layers = sorted({w.layer_begin, w.layer_end - 1})
    for layer in check_layers:
        kvd_gpu.compare_layer_with_oracle(w, src, dst, layer)
    log(f"layers {check_layers} match the oracle")

    extras = {}
    if not args.no_extras:
        def timed(fn, reps):
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(stream)
            for _ in range(reps):
                fn()
            b.record(stream)
            torch.cuda.synchronize()
            return a.elapsed_time(b) / reps * 1e3  # us

        # build alone (host validation + one translate/coalesce kernel per request)
        def build_only():
            x.plan.reset()
            x.build(batch)
        t = time.perf_counter()
        for _ in range(20):
            build_only()
        torch.cuda.synchronize()
        extras["build_us"] = (time.perf_counter() - t) / 20 * 1e6
        if batch:
            t = time.perf_counter()
            for _ in range(5):
                x.plan.reset()
                x.build(False)
            torch.cuda.synchronize()
            extras["build_one_call_per_request_us"] = (time.perf_counter() - t) / 5 * 1e6
            build_only()
        # a completion per request inside the batched pull (section 4.2): the cost against the plain pull of the
        # same plan, and when the first and the last request are announced
        if batch:
            y = G.GpuTransfer(w, src, dst, flags=kvd.KVD_PLAN_COMPLETE_PER_REQUEST, stream=stream)
            y.build(True)
            words = torch.zeros(len(w.requests), dtype=torch.int64).pin_memory()
            y.plan.pull_notify(words.data_ptr(), 1, sh)
            torch.cuda.synchronize()
            epoch = [1]

            def notify():
                epoch[0] += 1
                y.plan.pull_notify(words.data_ptr(), epoch[0], sh)
            extras["per_request_completion_pull_notify_us"] = timed(notify, 10)
            extras["per_request_completion_plain_pull_of_same_plan_us"] = timed(lambda: y.plan.pull(sh), 10)
            extras["per_request_completion_descriptors"] = y.plan.stats(sh)["num_descriptors"]
            torch.cuda.synchronize()
            epoch[0] += 1
            t = time.perf_counter()
            y.plan.pull_notify(words.data_ptr(), epoch[0], sh)
            seen = {}
            while len(seen) < len(w.requests) and time.perf_counter() - t < 10:
                for k in np.nonzero(words.numpy() == epoch[0])[0]:
                    seen.setdefault(int(k), time.perf_counter() - t)
            torch.cuda.synchronize()
            extras["per_request_completion_first_word_us"] = min(seen.values()) * 1e6
            extras["per_request_completion_median_word_us"] = float(np.median(list(seen.values()))) * 1e6
            extras["per_request_completion_last_word_us"] = max(seen.values()) * 1e6
            # neighbouring short requests announced together: a launch holds at least that many tokens
            grouped = {}
            for min_tokens in (512, 1024, 2048, 4096):
                y.plan.set_completion_granularity(min_tokens)
                notify()
                torch.cuda.synchronize()
                launches, tokens = 0, min_tokens
                for r in w.requests:
                    if tokens >= min_tokens:
                        launches, tokens = launches + 1, 0
                    tokens += r.seq_len
                grouped[str(min_tokens)] = {"us": timed(notify, 10), "launches": launches}
            extras["per_request_completion_grouped"] = grouped
            y.close()
        # the same request through the entry point that allocates nothing (tables in kernel arguments, scratch in the
        # library's static device array): whole call, wall clock
        if not batch and wl.blocks_for(w.requests[0].seq_len, min(w.src.block_tokens, w.dst.block_tokens)) <= kvd.KVD_NOALLOC_MAX_BLOCKS:
            r0 = w.requests[0]
            sd, dd = kvd.pool_desc(src.data_ptr(), w.src), kvd.pool_desc(dst.data_ptr(), w.dst)

            def noalloc():
                kvd.kvd_pull_noalloc(sd, dd, r0.src_table, r0.dst_table, r0.seq_len, w.layer_begin, w.layer_end, 0, sh)
            noalloc()
            torch.cuda.synchronize()
            t = time.perf_counter()
            for _ in range(20):
                noalloc()
            torch.cuda.synchronize()
            extras["noalloc_call_us"] = (time.perf_counter() - t) / 20 * 1e6
        # practical ceilings: one contiguous device-to-device copy of the payload
        n = min(payload, 1 << 30)
        a = torch.empty(n, dtype=torch.uint8, device="cuda")
        b = torch.empty(n, dtype=torch.uint8, device="cuda")
        with torch.cuda.stream(stream):
            us = timed(lambda: b.copy_(a, non_blocking=True), 10)
            extras["contiguous_memcpy_GBps"] = 2 * n / us / 1e3
            us = timed(lambda: kvd.kvd_copy_plain(b.data_ptr(), a.data_ptr(), n, sh), 10)
            extras["plain_copy_kernel_GBps"] = 2 * n / us / 1e3
        del a, b
        # the same plan without coalescing (every block its own descriptor)
        y = G.GpuTransfer(w, src, dst, flags=kvd.KVD_PLAN_NO_COALESCE, stream=stream)
        y.build()
        us = timed(lambda: y.plan.pull(sh), 10)
        extras["no_coalesce_pull_us"] = us
        extras["no_coalesce_descriptors"] = y.plan.stats(sh)["num_descriptors"]
        y.close()
        # plans whose work items the library puts in destination order: the same pull in queue order
        if stats["work_order"] != kvd.KVD_ORDER_QUEUE:
            y = G.GpuTransfer(w, src, dst, flags=kvd.KVD_PLAN_QUEUE_ORDER, stream=stream)
            y.build(batch)
            extras["queue_order_pull_us"] = timed(lambda: y.plan.pull(sh), 10)
            y.close()
        # the same work items walked by a persistent grid instead of one workgroup per item
        y = G.GpuTransfer(w, src, dst, flags=kvd.KVD_PLAN_PERSISTENT, stream=stream)
        y.build()
        extras["persistent_grid_pull_us"] = timed(lambda: y.plan.pull(sh), 10)
        y.close()
        # the buffer-based scheme: gather kernel -> copy -> host wait -> scatter kernel -> host wait, with a
        # staging buffer that holds two blocks (the paper's figure) and one that holds 64 MiB
        tile = w.src.tile_elems * w.src.elem_bytes
        for label, nbytes in (() if args.no_slow_baselines else (("two_blocks", max(4096, 2 * tile)), ("64MiB", 64 << 20))):
            sb = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
            rb = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
            torch.cuda.synchronize()
            t = time.perf_counter()
            x.plan.pull_staged(sb.data_ptr(), rb.data_ptr(), nbytes, sh)
            extras[f"staged_{label}_buffer_us"] = (time.perf_counter() - t) * 1e6
            del sb, rb
        # push-mode-like use (section 4.3): one layer per launch, as a prefill worker would issue them,
        # alone and next to a compute-bound kernel on another stream
        if args.per_layer and len(w.requests) == 1 and not stats["relayout"]:
            r = w.requests[0]
            layers = range(w.layer_begin, w.layer_end)

            def per_layer():
                for layer in layers:
                    x.plan.reset()
                    x.plan.build_descriptors(r.src_table, r.dst_table, r.seq_len, layer, layer + 1, sh)
                    x.plan.pull(sh)
            per_layer()
            torch.cuda.synchronize()
            t = time.perf_counter()
            per_layer()
            torch.cuda.synchronize()
            extras["per_layer_launches_total_us"] = (time.perf_counter() - t) * 1e6
            # the same with ONE build for all layers and one kvd_pull_layers per layer, eagerly and as one HIP graph
            x.plan.reset()
            x.build(batch)

            def per_layer_pulls():
                for layer in layers:
                    x.plan.pull_layers(layer, layer + 1, sh)
            per_layer_pulls()
            torch.cuda.synchronize()
            t = time.perf_counter()
            x.plan.reset()
            x.build(batch)
            per_layer_pulls()
            torch.cuda.synchronize()
            extras["one_build_per_layer_pulls_total_us"] = (time.perf_counter() - t) * 1e6
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                per_layer_pulls()
            graph.replay()
            torch.cuda.synchronize()
            t = time.perf_counter()
            for _ in range(5):
                graph.replay()
            torch.cuda.synchronize()
            extras["per_layer_pulls_graph_replay_us"] = (time.perf_counter() - t) / 5 * 1e6
            del graph
            # push mode next to the prefill's own compute: one 8192^3 bf16 GEMM stands in for a layer's
            # prefill work on torch's stream; when it is done, that layer's KV is pulled on the transfer stream
            # while the next layer's GEMM runs
            ma = torch.randn(8192, 8192, dtype=torch.bfloat16, device="cuda")
            mb = torch.randn(8192, 8192, dtype=torch.bfloat16, device="cuda")
            mc = torch.empty(8192, 8192, dtype=torch.bfloat16, device="cuda")
            compute = torch.cuda.Stream()  # same (default) priority as the transfer stream
            compute.wait_stream(torch.cuda.current_stream())
            done = [torch.cuda.Event() for _ in layers]

            def wall_us(fn):
                torch.cuda.synchronize()
                t = time.perf_counter()
                fn()
                torch.cuda.synchronize()
                return (time.perf_counter() - t) * 1e6

            def gemms_alone():
                with torch.cuda.stream(compute):
                    for _ in layers:
                        torch.matmul(ma, mb, out=mc)

            def gemms_with_pulls():
                with torch.cuda.stream(compute):
                    for k, layer in enumerate(layers):
                        torch.matmul(ma, mb, out=mc)
                        done[k].record(compute)
                        stream.wait_event(done[k])
                        x.plan.pull_layers(layer, layer + 1, sh)

            def gemms_then_single_shot():
                gemms_alone()
                done[0].record(compute)
                stream.wait_event(done[0])
                x.plan.pull(sh)
            for fn in (gemms_alone, gemms_with_pulls, gemms_then_single_shot):
                fn()
            extras["layer_gemms_alone_us"] = min(wall_us(gemms_alone) for _ in range(3))
            extras["per_layer_pulls_alone_us"] = min(wall_us(per_layer_pulls) for _ in range(3))
            extras["layer_gemms_with_per_layer_pulls_us"] = min(wall_us(gemms_with_pulls) for _ in range(3))
            extras["layer_gemms_then_single_shot_pull_us"] = min(wall_us(gemms_then_single_shot) for _ in range(3))
            del ma, mb, mc
            x.plan.reset()
            x.build(batch)
        # worst-case fragmentation (every block alone on both sides) of the same token count, in these pools and
        # in the same memory described as block-major pools ([block][layer][K/V]: one range per block over all layers)
        if len(w.requests) == 1 and not w.src.block_major:

            tokens = w.requests[0].seq_len
            nblk_s, nblk_d = wl.blocks_for(tokens, w.src.block_tokens), wl.blocks_for(tokens, w.dst.block_tokens)
            for label, geo in (("lone_blocks", (w.src, w.dst)),
                               ("lone_blocks_block_major", (dataclasses.replace(w.src, block_major=True),
                                                            dataclasses.replace(w.dst, block_major=True)))):
                rng = np.random.default_rng(w.seed + 3000)
                wr = wl.Workload(f"{w.name}-{label}", geo[0], geo[1],
                                 [wl.Request(tokens, wl.fixed_run_table(rng, geo[0].num_blocks, nblk_s, 1),
                                             wl.fixed_run_table(rng, geo[1].num_blocks, nblk_d, 1))],
                                 w.dtype, w.seed, w.layer_begin, w.layer_end)
                y = G.GpuTransfer(wr, src, dst, stream=stream)
                y.build()
                y.plan.pull(sh)
                extras[f"{label}_pull_us"] = timed(lambda: y.plan.pull(sh), 10)
                y.close()
            x.plan.reset()
            x.build(batch)
            x.plan.pull(sh)
            torch.cuda.synchronize()
        # bandwidth against the size of the transfer: the same recipe for the block tables, other token counts
        if args.size_sweep and args.config in (2, 4):
            sweep = {}
            tokens0 = w.requests[0].seq_len
            for tokens in [tokens0 // 8, tokens0 // 4, tokens0 // 2, tokens0, 2 * tokens0]:
                if wl.blocks_for(tokens, w.src.block_tokens) * 2 > w.src.num_blocks:
                    continue
                ws = wl.CONFIGS[args.config](tokens=tokens)
                y = G.GpuTransfer(ws, src, dst, stream=stream)
                y.build()
                y.plan.pull(sh)
                us = timed(lambda: y.plan.pull(sh), 10)
                p_bytes = y.plan.stats(sh)["payload_bytes"]
                groups = []  # best of three groups of ten steps (wall clock on a shared host)
                for _ in range(3):
                    t_step = time.perf_counter()
                    for _ in range(10):
                        y.plan.reset()
                        y.build()
                        y.plan.pull(sh)
                    torch.cuda.synchronize()
                    groups.append((time.perf_counter() - t_step) / 10 * 1e6)
                step_us = min(groups)
                sweep[str(tokens)] = {"payload_bytes": p_bytes, "pull_us": us, "pct_of_peak": 2 * p_bytes / us / 1e3 / PEAK_HBM_GBPS * 100,
                                      "step_us": step_us, "step_pct_of_peak": 2 * p_bytes / step_us / 1e3 / PEAK_HBM_GBPS * 100}
                y.close()
            extras["size_sweep"] = sweep
            x.plan.reset()
            x.build(batch)
            x.plan.pull(sh)
            torch.cuda.synchronize()
        # bandwidth against the block size (section 3 of the paper: 1024 / 2048 blocks of 4 KB and more): every block
        # alone on both sides, one KV head per GPU as in a tensor-parallel share, the configuration's layer count
        if args.block_size_sweep and not stats["relayout"]:
            sweep = {}
            pool_bytes = min(w.src.total_bytes, w.dst.total_bytes)
            layers = w.src.num_layers
            for block_tokens in (16, 32, 64, 128, 256, 512):
                block_bytes = block_tokens * 128 * 2
                pool_blocks = min(16384, pool_bytes // (2 * layers * block_bytes))
                gb = wl.PoolGeometry(layers, pool_blocks, block_tokens, 1, 128, 2, wl.BHTD)
                for n_blocks in (1024, 2048):
                    if 2 * n_blocks > pool_blocks:
                        continue
                    rng = np.random.default_rng(w.seed + 4000 + block_tokens + n_blocks)
                    wr = wl.Workload(f"lone-{block_bytes >> 10}KiB-x{n_blocks}", gb, gb,
                                     [wl.Request(n_blocks * block_tokens, wl.scattered_table(rng, pool_blocks, n_blocks),
                                                 wl.scattered_table(rng, pool_blocks, n_blocks))], "bf16", w.seed)
                    y = G.GpuTransfer(wr, src, dst, stream=stream)
                    y.build()
                    y.plan.pull(sh)
                    us = timed(lambda: y.plan.pull(sh), 10)
                    st_y = y.plan.stats(sh)
                    assert st_y["num_descriptors"] == n_blocks, st_y  # nothing merged: every block is alone
                    p_bytes = st_y["payload_bytes"]
                    sweep[f"{block_bytes >> 10}KiB_x{n_blocks}"] = {"payload_bytes": p_bytes, "pull_us": us,
                                                                   "pct_of_peak": 2 * p_bytes / us / 1e3 / PEAK_HBM_GBPS * 100}
                    y.close()
            extras["block_size_sweep"] = sweep
            x.plan.reset()
            x.build(batch)
            x.plan.pull(sh)
            torch.cuda.synchronize()
        # sensitivity to fragmentation: the same pools and token count, tables made of fixed-length runs
        if args.run_length_sweep and len(w.requests) == 1 and not stats["relayout"]:
            tokens = w.requests[0].seq_len
            nblk = wl.blocks_for(tokens, w.src.block_tokens)
            straight = np.arange(nblk, dtype=np.int32)
            sweep = {}
            for side in ("both", "src", "dst"):
                for run in (1, 2, 4, 8, 16, 64):
                    rng = np.random.default_rng(w.seed + 1000 + run)
                    ts = wl.fixed_run_table(rng, w.src.num_blocks, nblk, run) if side != "dst" else straight
                    td = wl.fixed_run_table(rng, w.dst.num_blocks, nblk, run) if side != "src" else straight
                    wr = wl.Workload(f"{w.name}-runs{run}-{side}", w.src, w.dst, [wl.Request(tokens, ts, td)],
                                     w.dtype, w.seed, w.layer_begin, w.layer_end)
                    # a descriptor ends where either side breaks, so one-sided cases have as many as two-sided ones
                    y = G.GpuTransfer(wr, src, dst, stream=stream)
                    y.build()
                    y.plan.pull(sh)
                    us = timed(lambda: y.plan.pull(sh), 10)
                    sweep[f"{side}_runs_of_{run}"] = {"pull_us": us, "pct_of_peak": 2 * payload / us / 1e3 / PEAK_HBM_GBPS * 100,
                                                     "descriptors": y.plan.stats(sh)["num_descriptors"]}
                    y.close()
            # the same bytes described as block-major pools ([block][layer][K/V]): a lone block is one range over all layers

            gbm = dataclasses.replace(w.src, block_major=True)
            for run in (1, 2):
                rng = np.random.default_rng(w.seed + 2000 + run)
                wr = wl.Workload(f"{w.name}-block-major-runs{run}", gbm, gbm,
                                 [wl.Request(tokens, wl.fixed_run_table(rng, gbm.num_blocks, nblk, run),
                                             wl.fixed_run_table(rng, gbm.num_blocks, nblk, run))],
                                 w.dtype, w.seed, w.layer_begin, w.layer_end)
                y = G.GpuTransfer(wr, src, dst, stream=stream)
                y.build()
                y.plan.pull(sh)
                us = timed(lambda: y.plan.pull(sh), 10)
                sweep[f"block_major_both_runs_of_{run}"] = {"pull_us": us, "pct_of_peak": 2 * payload / us / 1e3 / PEAK_HBM_GBPS * 100,
                                                             "descriptors": y.plan.stats(sh)["num_descriptors"]}
                y.close()
            extras["run_length_sweep"] = sweep
            x.plan.reset()
            x.build(batch)
            x.plan.pull(sh)
            torch.cuda.synchronize()
        # the library's choice of the order of the work against the queue order, over a range of fragmented workloads
        if args.order_ab and not stats["relayout"]:
            pool_bytes = min(w.src.total_bytes, w.dst.total_bytes)
            rng = np.random.default_rng(w.seed + 6000)
            results = {}

            def ab(name, wx, batched=False):
                row = {}
                for label, flags in (("default", 0), ("queue_order", kvd.KVD_PLAN_QUEUE_ORDER)):
                    y = G.GpuTransfer(wx, src, dst, flags, stream=stream)
                    y.build(batched)
                    y.plan.pull(sh)
                    us = min(timed(lambda: y.plan.pull(sh), 10) for _ in range(2))

                    def one_step():
                        y.plan.reset()
                        y.build(batched)
                        y.plan.pull(sh)
                    one_step()
                    step_us = min(timed(one_step, 10) for _ in range(2))
                    st_y = y.plan.stats(sh)
                    y.close()
                    row[label] = {"pull_us": us, "step_us": step_us, "pct_of_peak": 2 * st_y["payload_bytes"] / us / 1e3 / PEAK_HBM_GBPS * 100}
                    if label == "default":
                        row.update(work_order=st_y["work_order"], descriptors=st_y["num_descriptors"], work_items=st_y["num_work_items"],
                                   payload_bytes=st_y["payload_bytes"])
                results[name] = row

            def fragmented(g, tokens, max_run):
                fs, fd = np.ones(g.num_blocks, bool), np.ones(g.num_blocks, bool)
                n = wl.blocks_for(tokens, g.block_tokens)
                return wl.Workload("ab", g, g, [wl.Request(tokens, wl.fragmented_allocation(rng, fs, n, max_run),
                                                           wl.fragmented_allocation(rng, fd, n, max_run))], "bf16", w.seed)
            layers = w.src.num_layers
            g8 = wl.PoolGeometry(layers, min(16384, pool_bytes // (2 * layers * 32768)), 16, 8, 128, 2, wl.BHTD)   # 32 KiB blocks
            g1 = wl.PoolGeometry(layers, min(8192, pool_bytes // (2 * layers * 4096)), 16, 1, 128, 2, wl.BHTD)     # 4 KiB blocks
            ga = dataclasses.replace(g8, kv_adjacent=True)                                                         # 64 KiB pieces
            def fits(g, tokens):  # a request takes at most half of the pool, so that runs find room
                return 2 * wl.blocks_for(tokens, g.block_tokens) <= g.num_blocks
            for tokens in (8192, 32768, 65536):
                for max_run in (1, 2, 3, 4, 8):
                    if fits(g8, tokens):
                        ab(f"32KiB_blocks_{tokens}_tokens_runs_up_to_{max_run}", fragmented(g8, tokens, max_run))
            for tokens in (16384, 65536):
                for max_run in (1, 2, 4, 8):
                    if fits(g1, tokens):
                        ab(f"4KiB_blocks_{tokens}_tokens_runs_up_to_{max_run}", fragmented(g1, tokens, max_run))
            if fits(ga, 32768):
                ab("kv_adjacent_64KiB_pieces_32768_tokens_lone", fragmented(ga, 32768, 1))
            if fits(g8, 32763):
                ab("32KiB_blocks_32763_tokens_lone_partial_last_block", fragmented(g8, 32763, 1))
            for n_req, median, hi, max_run in ((256, 256.0, 4096, 1), (256, 256.0, 4096, 2), (1024, 64.0, 1024, 1), (1024, 64.0, 1024, 8),
                                               (32, 2048.0, 16384, 1), (32, 2048.0, 16384, 8)):
                lens = wl.lognormal_lengths(rng, n_req, median, 1.0, 16, hi)
                need = sum(wl.blocks_for(int(t), 16) for t in lens)
                gb = dataclasses.replace(g8, num_blocks=min(g8.num_blocks, int(need * 1.25) + 1))
                if need * 1.2 > gb.num_blocks:
                    continue
                fs, fd = np.ones(gb.num_blocks, bool), np.ones(gb.num_blocks, bool)
                reqs = [wl.Request(int(t), wl.fragmented_allocation(rng, fs, wl.blocks_for(int(t), 16), max_run),
                                   wl.fragmented_allocation(rng, fd, wl.blocks_for(int(t), 16), max_run)) for t in lens]
                ab(f"batch_of_{n_req}_median_{int(median)}_tokens_runs_up_to_{max_run}_pool_{gb.num_blocks}",
                   wl.Workload("ab", gb, gb, reqs, "bf16", w.seed), batched=True)
            extras["order_ab"] = results
            x.plan.reset()
            x.build(batch)
            x.plan.pull(sh)
            torch.cuda.synchronize()
        # where lone pieces lose their bandwidth: (a) every block alone, but queue neighbours a fixed distance apart
        # (groups of `group` blocks, `distance` blocks between members), (b) the same block ids paired and queued
        # so that one or both sides are swept in address order -- what the order of the queue is worth at best
        if args.locality_sweep and len(w.requests) == 1 and not stats["relayout"]:
            tokens = w.requests[0].seq_len
            nblk = wl.blocks_for(tokens, w.src.block_tokens)
            keep = kvd.KVD_PLAN_QUEUE_ORDER | kvd.KVD_PLAN_NO_COALESCE  # the queue as given, every block its own descriptor

            def pull_pct(ts, td, flags=keep):
                wr = wl.Workload(f"{w.name}-locality", w.src, w.dst,
                                 [wl.Request(tokens, np.asarray(ts, np.int32), np.asarray(td, np.int32))],
                                 w.dtype, w.seed, w.layer_begin, w.layer_end)
                y = G.GpuTransfer(wr, src, dst, flags, stream=stream)
                y.build()
                y.plan.pull(sh)
                us = min(timed(lambda: y.plan.pull(sh), 10) for _ in range(2))
                y.close()
                return {"pull_us": us, "pct_of_peak": 2 * payload / us / 1e3 / PEAK_HBM_GBPS * 100}

            def spaced(rng, pool_blocks, group, distance):
                span = 1
                while span < group * distance + 2:
                    span *= 2
                slots = rng.permutation(pool_blocks // span)
                ids = np.concatenate([sl * span + np.arange(group) * distance for sl in slots[:-(-nblk // group)]])
                return ids[:nblk]
            sweep = {}
            for group in (2, 4):
                for distance in (2, 3, 4, 8, 32):
                    if (nblk // group + 1) * group * distance * 2 > w.src.num_blocks:
                        continue
                    rng = np.random.default_rng(w.seed + 4000)
                    sweep[f"lone_blocks_in_groups_of_{group}_members_{distance}_blocks_apart"] = pull_pct(
                        spaced(rng, w.src.num_blocks, group, distance), spaced(rng, w.dst.num_blocks, group, distance))
            rng = np.random.default_rng(w.seed + 3000)
            ts = wl.fixed_run_table(rng, w.src.num_blocks, nblk, 1)
            td = wl.fixed_run_table(rng, w.dst.num_blocks, nblk, 1)
            o_d, o_s = np.argsort(td), np.argsort(ts)
            sweep["lone_blocks_queue_order"] = pull_pct(ts, td)
            sweep["lone_blocks_as_the_library_orders_them"] = pull_pct(ts, td, kvd.KVD_PLAN_NO_COALESCE)
            sweep["lone_blocks_queue_sorted_by_destination"] = pull_pct(ts[o_d], td[o_d])
            sweep["lone_blocks_queue_sorted_by_source"] = pull_pct(ts[o_s], td[o_s])
            sweep["lone_blocks_both_sides_in_address_order"] = pull_pct(np.sort(ts), np.sort(td))
            # what the library's ordering is worth against the share of the pool the request takes: more lone blocks
            # out of the same pool, in queue order and as the library orders them; pull alone, and the whole step
            # (reset + build + ordering launches + pull)
            for n in (nblk, 2 * nblk, 4 * nblk, 8 * nblk):
                if 2 * n > min(w.src.num_blocks, w.dst.num_blocks):
                    continue
                rng = np.random.default_rng(w.seed + 5000 + n)
                ts_n, td_n = wl.scattered_table(rng, w.src.num_blocks, n), wl.scattered_table(rng, w.dst.num_blocks, n)
                for label, flags in (("queue_order", keep), ("as_the_library_orders_them", kvd.KVD_PLAN_NO_COALESCE)):
                    wr = wl.Workload(f"{w.name}-density", w.src, w.dst, [wl.Request(n * w.src.block_tokens, ts_n, td_n)],
                                     w.dtype, w.seed, w.layer_begin, w.layer_end)
                    y = G.GpuTransfer(wr, src, dst, flags, stream=stream)
                    y.build()
                    y.plan.pull(sh)
                    us = min(timed(lambda: y.plan.pull(sh), 10) for _ in range(2))

                    def one_step():
                        y.plan.reset()
                        y.build()
                        y.plan.pull(sh)
                    step_us = min(timed(one_step, 10) for _ in range(2))
                    y.close()
                    sweep[f"{n}_lone_blocks_of_{w.src.num_blocks}_{label}"] = {
                        "pull_us": us, "pct_of_peak": 2 * payload * n / nblk / us / 1e3 / PEAK_HBM_GBPS * 100, "step_us": step_us}
            # the configuration's own block ids: as queued, and paired / queued in address order
            r0 = w.requests[0]
            cs, cd = np.asarray(r0.src_table[:nblk]), np.asarray(r0.dst_table[:nblk])
            q = kvd.KVD_PLAN_QUEUE_ORDER
            o_d = np.argsort(cd)
            sweep["configured_tables_as_the_library_orders_them"] = pull_pct(cs, cd, 0)
            sweep["configured_tables_queue_order"] = pull_pct(cs, cd, q)
            sweep["configured_tables_queue_sorted_by_destination"] = pull_pct(cs[o_d], cd[o_d], q)
            sweep["configured_tables_both_sides_in_address_order"] = pull_pct(np.sort(cs), np.sort(cd), q | kvd.KVD_PLAN_NO_COALESCE)
            extras["locality_sweep"] = sweep
            x.plan.reset()
            x.build(batch)
            x.plan.pull(sh)
            torch.cuda.synchronize()
        # re-layout plans: the configuration's own block ids, and the same ids with both sides swept in address order
        if args.locality_sweep and len(w.requests) == 1 and stats["relayout"]:
            r0 = w.requests[0]

            def relayout_pct(ts, td):
                wr = wl.Workload(f"{w.name}-locality", w.src, w.dst, [wl.Request(r0.seq_len, np.asarray(ts, np.int32), np.asarray(td, np.int32))],
                                 w.dtype, w.seed, w.layer_begin, w.layer_end)
                y = G.GpuTransfer(wr, src, dst, stream=stream)
                y.build()
                y.plan.pull(sh)
                us = min(timed(lambda: y.plan.pull(sh), 10) for _ in range(2))
                y.close()
                return {"pull_us": us, "pct_of_peak": 2 * payload / us / 1e3 / PEAK_HBM_GBPS * 100}
            extras["locality_sweep"] = {
                "configured_tables": relayout_pct(r0.src_table, r0.dst_table),
                "configured_tables_both_sides_in_address_order": relayout_pct(np.sort(r0.src_table), np.sort(r0.dst_table)),
                "dense_identity_tables": relayout_pct(np.arange(len(r0.src_table)), np.arange(len(r0.dst_table))),
            }
            x.plan.reset()
            x.build(batch)
            x.plan.pull(sh)
            torch.cuda.synchronize()
        # one hipMemcpyAsync per (layer, K/V, block)
        if not stats["relayout"] and not args.no_slow_baselines:
            torch.cuda.synchronize()
            t = time.perf_counter()
            x.plan.pull_blockwise_memcpy(sh)
            torch.cuda.synchronize()
            extras["blockwise_memcpy_us"] = (time.perf_counter() - t) * 1e6
        log(f"extras: {extras}")

    if args.stream_probes:
        # what the memory system gives a read stream, a write stream and a copy on plain 1 GiB buffers, one access per
        # lane with the workgroups dispatched in address order against a persistent grid striding over the buffer
        n = 1 << 30
        a = torch.empty(n, dtype=torch.uint8, device="cuda")
        b = torch.empty(n, dtype=torch.uint8, device="cuda")
        a.view(torch.int16).fill_(0x3C00)
        probes = {}
        for mode in kvd.PROBE_MODES:
            kvd.kvd_stream_probe(b.data_ptr(), a.data_ptr(), n, mode, sh)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(10):
                kvd.kvd_stream_probe(b.data_ptr(), a.data_ptr(), n, mode, sh)
            e1.record(stream)
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) / 10 * 1e3
            moved = (2 if mode.startswith("copy") else 1) * n
            probes[mode] = {"us": us, "GBps": moved / us / 1e3, "pct_of_peak": moved / us / 1e3 / PEAK_HBM_GBPS * 100}
        extras["stream_probes_1GiB"] = probes
        log(f"stream probes: { {k: round(v['GBps']) for k, v in probes.items()} }")
        del a, b

    if args.copy_calibration:
        n = 1 << 30
        a = torch.empty(n, dtype=torch.uint8, device="cuda")
        b = torch.empty(n, dtype=torch.uint8, device="cuda")
        for _ in range(5):
            kvd.kvd_copy_plain(b.data_ptr(), a.data_ptr(), n, sh)
        torch.cuda.synchronize()

    from paper_2501_14743_amd import traffic as traffic_record
    rec = traffic_record.load_record(w.name)
    traffic = rec["traffic_bytes_per_launch"] if rec else None
    # the counters cannot be read inside this run: the figure comes from the recorded rocprofv3 --pmc
    # runs of this same kernel source on this workload (profiles/), or is null when there is none
    traffic_source = "recorded rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE) of this kernel source" if rec else None

    out = {
        "metric": METRIC, "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": w.name, "requests": len(w.requests), "tokens": w.total_tokens,
                   "layers": w.layer_end - w.layer_begin, "kv_heads": w.src.num_kv_heads,
                   "head_dim": w.src.head_dim, "elem_bytes": w.src.elem_bytes,
                   "block_tokens": [w.src.block_tokens, w.dst.block_tokens],
                   "layouts": [w.src.layout, w.dst.layout], "pool_blocks": [w.src.num_blocks, w.dst.num_blocks],
                   "payload_bytes": payload, "descriptors": stats["num_descriptors"],
                   "transactions": stats["num_transactions"], "work_items": stats["num_work_items"],
                   "work_order": ("queue", "destination regions", "sorted by destination")[stats["work_order"]]},
        "us_per_request_batch": ms_per_step * 1e3,
        "pct_of_peak": 100.0 * achieved / PEAK_HBM_GBPS,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                     "frac": achieved / PEAK_HBM_GBPS, "traffic": traffic, "traffic_source": traffic_source,
                     "kernel": "kvd_pull_kernel", "kernel_us_mean": float(pull_ms.mean() * 1e3),
                     "kernel_us_min": float(pull_ms.min() * 1e3), "launches_timed": int(pull_ms.size),
                     "empty_event_pair_us": event_pair_us,
                     "algorithmic_bytes_per_launch": 2 * payload},
        "step_host_us": {"p50": float(np.percentile(host_us, 50)), "p99": float(np.percentile(host_us, 99)),
                         "max": float(host_us.max()), "max_at_step": int(host_us.argmax()),
                         "max_step_reset_build_pull_us": [float(v * 1e6) for v in calls[int(host_us.argmax())]],
                         "gc_collections_in_timed_region": len(gc_pauses),
                         "gc_longest_ms": max((ms for _, ms in gc_pauses), default=0.0),
                         "gc_full_collections_ms": [round(ms, 3) for g, ms in gc_pauses if g == 2]},
        "verified": f"layers {check_layers} bit-exact vs oracle after the timed steps",
        "extras": extras,
    }
    if cpu is not None:
        out["cpu_baseline"] = cpu
    assert isinstance(out["value"], float) and out["value"] > 0 and isinstance(out["ms_per_step"], float)
    print(json.dumps(out), flush=True)
    x.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
