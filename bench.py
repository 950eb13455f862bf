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
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
for p in (ROOT, os.path.join(ROOT, "tests")):
    if p not in sys.path:
        sys.path.insert(0, p)

PEAK_HBM_GBPS = 8000.0  # MI355X published HBM3E bandwidth
METRIC = "achieved HBM GB/s (% of peak) for paged KV pull; µs per 8K-token request"


def log(msg: str) -> None:
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def cpu_baseline(cfg_no: int, budget_s: float = 12.0) -> dict:
    """Time the oracle (as it stands, one thread) on a bounded sample: layer 0 of the same
    workload, repeated (at most 256 times) until about `budget_s` seconds of CPU work have been spent."""
    import numpy as np
    import kvd_testlib as tl
    from paper_2501_14743_amd import workloads as wl

    full = wl.CONFIGS[cfg_no]()
    gs = wl.PoolGeometry(1, full.src.num_blocks, full.src.block_tokens, full.src.num_kv_heads,
                         full.src.head_dim, full.src.elem_bytes, full.src.layout)
    gd = wl.PoolGeometry(1, full.dst.num_blocks, full.dst.block_tokens, full.dst.num_kv_heads,
                         full.dst.head_dim, full.dst.elem_bytes, full.dst.layout)
    w = wl.Workload(full.name, gs, gd, full.requests, full.dtype, full.seed)
    src = np.ones(gs.total_bytes, np.uint8)
    dst = np.ones(gd.total_bytes, np.uint8)
    payload = w.total_tokens * 2 * gs.num_kv_heads * gs.head_dim * gs.elem_bytes
    t0 = time.perf_counter()
    tl.oracle_pull_workload(w, src, dst)
    first = time.perf_counter() - t0
    reps = max(1, min(256, int(budget_s / max(first, 1e-3))))
    t0 = time.perf_counter()
    for _ in range(reps):
        tl.oracle_pull_workload(w, src, dst)
    dt = (time.perf_counter() - t0) / reps
    return {
        "value": 2 * payload / dt / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
        "sample": f"layer 0 (K and V) of {full.name}: {w.total_tokens} tokens, {payload} payload bytes, "
                  f"mean of {reps} passes after one untimed pass; host has {os.cpu_count()} cpus",
        "seconds_per_layer": dt,
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
    ap.add_argument("--no-extras", action="store_true", help="skip the reported GPU baselines")
    ap.add_argument("--no-slow-baselines", action="store_true",
                    help="skip the staged and the per-block memcpy baselines (hundreds of thousands of launches)")
    ap.add_argument("--per-layer", action="store_true",
                    help="also time the transfer issued one layer per launch, alone and next to GEMMs")
    ap.add_argument("--run-length-sweep", action="store_true",
                    help="also time the pull of the same token count with block tables made of runs of exactly "
                         "1, 2, 4, ... consecutive blocks (both sides, source only, destination only)")
    ap.add_argument("--size-sweep", action="store_true",
                    help="also time the pull of 1/8 ... 2x the configuration's token count (configurations 2 and 4), "
                         "the bandwidth-against-transfer-size curve of the paper's motivation")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also launch the plain copy kernel a few times (for counter calibration runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (both pools live in one MI355X's HBM); "
              "run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2501_14743_amd import kvd, workloads as wl
    import kvd_gpu as G

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    kvd.lib()  # fail now if the library is missing
    torch.cuda.set_device(0)
    w = wl.CONFIGS[args.config]()
    log(f"{w.name}: pools {w.src.total_bytes / 2**30:.2f} + {w.dst.total_bytes / 2**30:.2f} GiB, "
        f"{len(w.requests)} requests, {w.total_tokens} tokens")
    src = G.device_random_pool(w.src, w.dtype, w.seed)
    dst = G.device_sentinel_pool(w.dst)
    stream = torch.cuda.Stream()
    x = G.GpuTransfer(w, src, dst, stream=stream)
    sh = stream.cuda_stream

    batch = len(w.requests) > 1  # several requests are appended with the one batched call

    def step(ev=None):
        x.plan.reset()
        x.build(batch)
        if ev is not None:
            ev[0].record(stream)
        x.plan.pull(sh)
        if ev is not None:
            ev[1].record(stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    stride = max(1, args.event_stride)
    events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
              for _ in range(0, args.steps, stride)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(events[i // stride] if i % stride == 0 else None)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    stats = x.plan.stats(sh)  # of the last step's plan
    payload = stats["payload_bytes"]
    pull_ms = np.array([a.elapsed_time(b) for a, b in events])
    ms_per_step = elapsed / args.steps * 1e3
    value = 2 * payload * args.steps / elapsed / 1e9
    achieved = 2 * payload / (pull_ms.mean() * 1e-3) / 1e9
    log(f"step {ms_per_step * 1e3:.1f} us, pull kernel mean {pull_ms.mean() * 1e3:.1f} us "
        f"(min {pull_ms.min() * 1e3:.1f}), {achieved:.0f} GB/s = {achieved / PEAK_HBM_GBPS:.1%} of peak")

    # the timed work produced the right bytes: oracle on one layer
    check_layer = w.layer_end - 1
    G.compare_layer_with_oracle(w, src, dst, check_layer)
    log(f"layer {check_layer} matches the oracle")

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
        # plans of short transactions: the same pull without grouping the work items by destination region
        if stats["num_work_items"] < 4 * stats["num_transactions"]:
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
            ma = torch.randn(8192, 8192, dtype=torch.bfloat16, device="cuda")
            mb = torch.randn(8192, 8192, dtype=torch.bfloat16, device="cuda")

            def gemms(n):
                for _ in range(n):
                    torch.matmul(ma, mb)
            gemms(2)
            torch.cuda.synchronize()
            t = time.perf_counter()
            gemms(10)
            torch.cuda.synchronize()
            extras["ten_gemms_alone_us"] = (time.perf_counter() - t) * 1e6
            t = time.perf_counter()
            gemms(10)
            per_layer()
            torch.cuda.synchronize()
            extras["ten_gemms_with_per_layer_pulls_us"] = (time.perf_counter() - t) * 1e6
            del ma, mb
            x.plan.reset()
            x.build(batch)
        # worst-case fragmentation (every block alone on both sides) of the same token count, in these pools and
        # in the same memory described as block-major pools ([block][layer][K/V]: one range per block over all layers)
        if len(w.requests) == 1 and not w.src.block_major:
            import dataclasses
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
                groups = []  # best of three groups of ten steps: the HIP runtime stalls once, for tens of
                for _ in range(3):  # milliseconds, after some five hundred launches of a process
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
            import dataclasses
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
        # one hipMemcpyAsync per (layer, K/V, block)
        if not stats["relayout"] and not args.no_slow_baselines:
            torch.cuda.synchronize()
            t = time.perf_counter()
            x.plan.pull_blockwise_memcpy(sh)
            torch.cuda.synchronize()
            extras["blockwise_memcpy_us"] = (time.perf_counter() - t) * 1e6
        log(f"extras: {extras}")

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
                   "transactions": stats["num_transactions"], "work_items": stats["num_work_items"]},
        "us_per_request_batch": ms_per_step * 1e3,
        "pct_of_peak": 100.0 * achieved / PEAK_HBM_GBPS,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                     "frac": achieved / PEAK_HBM_GBPS, "traffic": traffic,
                     "kernel": "kvd_pull_kernel", "kernel_us_mean": float(pull_ms.mean() * 1e3),
                     "kernel_us_min": float(pull_ms.min() * 1e3), "launches_timed": int(pull_ms.size),
                     "algorithmic_bytes_per_launch": 2 * payload},
        "verified": f"layer {check_layer} bit-exact vs oracle after the timed steps",
        "extras": extras,
    }
    if not args.no_cpu_baseline:
        log("timing the oracle on the host")
        out["cpu_baseline"] = cpu_baseline(args.config)
    print(json.dumps(out), flush=True)
    x.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
