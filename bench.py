#!/usr/bin/env python3
"""Benchmark of the offloaded sparse-decode layer-step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 3]

A "step" is one kvd_step: score -> select -> resolve -> fetch -> attend for one
layer over the whole batch.  The workload is the benchmark definition's
configuration 3 (1 layer, batch 16, 131072-token context, page 16, 32 q / 8 kv
heads, bf16, budget 4096 tokens, GPU cache 25 % of the pages, the rest in pinned
host memory) with synthetic Zipf-importance K/V; the drifting query stream is
continued past the configuration's 32 steps when more steps are asked for.

Prints one JSON line: `value` is end-to-end layer-steps/s of the K timed steps
(fetch of missed pages from pinned host memory included, index / cache / queries
resident in HBM).  `gpu_resident` is the same step with every selected page
already resident (nothing crosses the host link), timed with HIP events on the
stream, against the HBM roofline; `roofline` is for the dominant kernel: the
one-launch `step_kernel` on those resident launches when the step runs as one
launch, else the larger of the scoring / attention kernels of the chain, from a
pass with HIP events around every kernel launch (`kernels_ms`, the stage
breakdown); `cpu_baseline` is the CPU oracle timed on a bounded sample of the
same workload on the host cores.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
HOST_LINK_PEAK_GBPS = 63.0      # PCIe Gen5 x16, one direction: 32 GT/s x 16 lanes x 128/130
# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command, scaled by
# what the same counters read for a plain copy of known size (profiles/pmc_traffic_cfg3.md)
PMC_TRAFFIC_BYTES = {("cfg3", "step"): 552530944, ("cfg3", "attend"): 270542848, ("cfg3", "score"): 273769472}


def describe(w) -> str:
    return (f"{w.name}: L={w.n_layers} B={w.batch} ctx={w.ctx} page={w.page} heads={w.n_q_heads}q/{w.n_kv_heads}kv "
            f"D={w.head_dim} {w.dtype} k={w.topk_pages} pages ({w.topk_pages * w.page} tokens) "
            f"{'flat index' if w.index_centroids == 0 else str(w.index_centroids) + ' centroids'} cache={w.capacity} pages/unit ({100.0 * w.capacity / w.n_pages:.0f}%, {w.policy}) {w.importance} importance, rho={w.rho}")


def cpu_baseline(w, store, q_list, seconds: float):
    """Times the oracle, as it stands, on as many (unit, step) pairs of the same workload as fit
    in about `seconds`; returns layer-steps/s (one layer-step = all U units)."""
    import numpy as np
    import torch
    from oracle import kvd_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = 1
    code = orc.F16 if w.dtype == "f16" else orc.BF16
    scale = 1.0 / math.sqrt(w.head_dim)
    done, spent, units = 0, 0.0, 0
    for u in range(w.units):
        b, h = divmod(u, w.n_kv_heads)
        kv = store[0, b, h].to(torch.float64).numpy()
        keys, vals = kv[:, 0].reshape(-1, w.head_dim), kv[:, 1].reshape(-1, w.head_dim)
        summ = orc.page_summaries(keys, w.page, w.ctx, code)            # set-up, not timed
        cent = members = None
        if w.index_centroids > 0:                                        # index build: set-up, not timed
            cent, assign, _ = orc.kmeans_centroids(summ, w.index_centroids, w.index_iterations, code)
            members = orc.cluster_members(assign, w.index_centroids)
        win = (orc.LookaheadWindow if w.policy == "lookahead" else orc.LruWindow)(w.capacity)
        units += 1
        for t, q in enumerate(q_list):
            qg = q[b, h * w.group:(h + 1) * w.group].to(torch.float64).numpy()
            t0 = time.perf_counter()
            orc.decode_unit_step(qg, summ, keys, vals, win, t, k=w.topk_pages, page_size=w.page, seq_len=w.ctx,
                                 scale=scale, sink_pages=w.sink_pages, recent_pages=w.recent_pages, centroids=cent,
                                 members=members)
            spent += time.perf_counter() - t0
            done += 1
        if spent >= seconds or (w.index_centroids > 0 and units >= 8):   # (the oracle's k-means is slow set-up)
            break
    per_unit_step = spent / max(done, 1)
    return {
        "value": 1.0 / (per_unit_step * w.units),
        "unit": "layer-steps/s",
        "cores": int(threads),
        "kind": "oracle",
        "sample": f"{done} unit-steps ({units} of {w.units} units x {len(q_list)} steps) in {spent:.1f} s, "
                  f"scaled to one layer-step = {w.units} units",
    }


def layers_in_flight(args, cfg_w, K, W, torch, dev):
    """The configuration's layer-step over `--layers` layers of one decode step, layers one by one
    (kvd_step per layer) against two layers in flight (kvd_step_layers): end-to-end ms per
    layer-step including the fetch of missed pages, cold start, the first `warmup` decode steps
    untimed."""
    n = args.layers
    w = cfg_w.replace(n_layers=n, physical_layers=min(n, 2), policy=args.policy)
    L, B, Hkv, NP, P, D = w.n_layers, w.batch, w.n_kv_heads, w.n_pages, w.page, w.head_dim
    q0 = W.initial_queries(w, dev)
    store = W.make_kv_store(w, q0, dev)
    summ = torch.zeros((L, B, Hkv, NP, D), dtype=w.torch_dtype, device=dev)
    pool = torch.zeros((L, B, Hkv, w.capacity, 2, P, D), dtype=w.torch_dtype, device=dev)
    steps, warm = max(2, args.steps // n), max(4, args.warmup)
    qs = [q.contiguous() for q in W.query_stream(w, q0, warm + steps, dev)]
    out = torch.empty((L, B, w.n_q_heads, D), dtype=torch.float32, device=dev)
    res = {"what": f"{L} layers of one decode step (host store of {w.phys_layers} layers shared by them), {steps} timed decode "
                   f"steps after {warm} from a cold cache: end-to-end ms per layer-step", "layers": L}
    keep = None
    for mode in ("one_by_one", "two_in_flight"):
        ctx = K.Kvd(n_layers=L, batch=B, n_q_heads=w.n_q_heads, n_kv_heads=Hkv, page_size=P, max_pages=NP,
                    topk_pages=w.topk_pages, capacity_max=w.capacity, kv_dtype=w.torch_dtype, sink_pages=w.sink_pages,
                    recent_pages=w.recent_pages, physical_layers=w.physical_layers, micro_batches=args.micro_batches,
                    policy=w.policy)
        ctx.bind_summaries(summ)
        ctx.bind_host_store(store)
        ctx.bind_slot_pool(pool)
        for l in range(L):
            ctx.build_summaries(l)
        pages = W.warm_pages(w)
        if pages is not None:
            for l in range(L):
                ctx.cache_warm(l, pages.tolist() * w.units, [len(pages)] * w.units)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for t, q in enumerate(qs):
            if t == warm:
                torch.cuda.synchronize()
                ctx.reset_stats()
                e0.record()
            if mode == "one_by_one":
                for l in range(L):
                    ctx.step(l, t, q[l], out[l])
            else:
                ctx.step_layers(0, L, t, q, out)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / (steps * L)
        st = ctx.stats()
        res[mode] = {"ms_per_layer_step": ms, "layer_steps_per_s": 1e3 / ms,
                     "host_link_GBps": st.gathered_bytes / (steps * L) / (ms * 1e-3) / 1e9,
                     "hit_rate": st.hits / max(1, st.hits + st.misses)}
        res["step_form"] = ctx.step_form()
        if keep is None:
            keep = out.clone()
        else:
            res["max_abs_output_difference"] = float((out - keep).abs().max())
        ctx.close()
    return res


def _max_clock_mhz():
    """Peak engine clock from the HIP runtime that torch has already loaded (torch does not expose it)."""
    import ctypes
    try:
        hip = ctypes.CDLL("libamdhip64.so")
        khz = ctypes.c_int(0)
        hip_device_attribute_clock_rate = 5                        # hipDeviceAttributeClockRate
        if hip.hipDeviceGetAttribute(ctypes.byref(khz), hip_device_attribute_clock_rate, 0) == 0:
            return khz.value / 1e3
    except OSError:
        pass
    return None


def step_timeline(ctx, t, q, out, stream):
    """One more all-hit step of the single-launch kernel with its per-workgroup clock readings on:
    when each role's workgroups were dispatched, how long they waited for their inputs, how long
    they worked (microseconds from the first workgroup's start; GPU wall clock, 100 MHz)."""
    import numpy as np
    import torch
    ctx.set_profiling(2)
    ctx.step(0, t, q, out, stream=stream)
    torch.cuda.synchronize()
    rec = ctx.step_timeline().numpy()
    ctx.set_profiling(0)
    us = (rec[:, :4] - rec[:, 0].min()) / 100.0
    role = rec[:, 4] & 0xff
    res = {"workgroups": int(len(rec)), "kernel_us": float(us[:, 3].max())}
    for r, name in enumerate(["score", "select_resolve", "attend"]):
        x = us[role == r]
        res[name] = {"workgroups": int(len(x)), "first_start_us": float(x[:, 0].min()), "last_start_us": float(x[:, 0].max()),
                     "median_wait_us": float(np.median(x[:, 1] - x[:, 0])), "median_work_us": float(np.median(x[:, 2] - x[:, 1])),
                     "last_end_us": float(x[:, 3].max())}
    return res


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=62)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=3)
    ap.add_argument("--micro-batches", type=int, default=0, help="kvd_config.micro_batches (0 = library chooses, 1 = chain of kernels, -1 = one launch)")
    ap.add_argument("--policy", choices=["lru", "lookahead"], default="lru", help="cache replacement policy")
    ap.add_argument("--centroids", type=int, default=0,
                    help="hierarchical index with this many centroids per unit (0 = flat page index)")
    ap.add_argument("--index-iterations", type=int, default=4, help="k-means rounds of the hierarchical index build")
    ap.add_argument("--window", type=float, default=0.0,
                    help="cache capacity as a multiple of the per-step budget k (the paper's window size); "
                         "0 keeps the configuration's capacity")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="0 skips the oracle baseline")
    ap.add_argument("--no-profile-pass", action="store_true", help="skip the per-kernel HIP-event pass")
    ap.add_argument("--calibrate", type=int, default=0, metavar="STEPS",
                    help="before the warm-up, let the library time every form of the step on STEPS real steps each "
                         "and keep the fastest (kvd_calibrate_step_form)")
    ap.add_argument("--tier", metavar="PATH", default="",
                    help="put the third tier behind the GPU window: the K/V pages are written to a backing file at PATH "
                         "(removed afterwards), host DRAM holds a pool of extents, and the timed steps are kvd_step_tiered")
    ap.add_argument("--tier-extent-pages", type=int, default=8)
    ap.add_argument("--tier-pool-frac", type=float, default=0.25, help="DRAM pool as a fraction of the file's extents")
    ap.add_argument("--tier-queue-depth", type=int, default=16)
    ap.add_argument("--tier-max-run", type=int, default=8)
    ap.add_argument("--tier-buffered", action="store_true", help="read through the page cache instead of O_DIRECT")
    ap.add_argument("--tier-layout", choices=["page", "semantic"], default="page",
                    help="order of a unit's pages in the file: page order, or cluster by cluster (needs --centroids)")
    ap.add_argument("--batch", type=int, default=0, metavar="B", help="B > 0: the configuration's shape with B sequences instead of its own batch")
    ap.add_argument("--layers", type=int, default=1, metavar="N",
                    help="N > 1: add a leg that steps N layers per decode step, one by one and two in flight (kvd_step_layers)")
    ap.add_argument("--timeline", action="store_true",
                    help="when the step runs as one launch: add the per-workgroup timeline of one all-hit step")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this path is built and measured on one GPU only (no collectives, no sharding); "
              "run with --gpus 1", file=sys.stderr)
        return 2

    import torch
    from paper_2605_18071_amd import kvd as K
    from paper_2605_18071_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    K.load()                                     # fails loudly if libkvd.so is not built
    dev = "cuda:0"
    torch.cuda.set_device(0)
    w = W.CONFIGS[args.config]
    if args.batch > 0:
        w = w.replace(batch=args.batch, name=f"{w.name}-batch{args.batch}")
    cfg_w = w
    if w.n_layers != 1:
        # multi-layer configurations are benchmarked on one layer's worth of state at full per-layer shape
        w = w.replace(n_layers=1, physical_layers=1)
    if args.window > 0:
        w = w.replace(capacity=max(w.topk_pages, int(round(args.window * w.topk_pages))))
    w = w.replace(policy=args.policy, index_centroids=args.centroids, index_iterations=args.index_iterations)
    L, B, Hkv, NP, P, D, U, k = w.n_layers, w.batch, w.n_kv_heads, w.n_pages, w.page, w.head_dim, w.units, w.topk_pages

    t_setup = time.perf_counter()
    q0 = W.initial_queries(w, dev)
    store = W.make_kv_store(w, q0, dev)
    summ = torch.zeros((L, B, Hkv, NP, D), dtype=w.torch_dtype, device=dev)
    pool = torch.zeros((L, B, Hkv, w.capacity, 2, P, D), dtype=w.torch_dtype, device=dev)
    ctx = K.Kvd(n_layers=L, batch=B, n_q_heads=w.n_q_heads, n_kv_heads=Hkv, page_size=P, max_pages=NP, topk_pages=k,
                capacity_max=w.capacity, kv_dtype=w.torch_dtype, sink_pages=w.sink_pages, recent_pages=w.recent_pages,
                physical_layers=w.physical_layers, micro_batches=args.micro_batches, policy=w.policy,
                index_centroids=w.index_centroids)
    ctx.bind_summaries(summ)
    ctx.bind_host_store(store)
    ctx.bind_slot_pool(pool)
    ctx.build_summaries(0)
    if w.index_centroids > 0:
        centroids = torch.zeros((L, B, Hkv, w.index_centroids, D), dtype=w.torch_dtype, device=dev)
        cluster_start = torch.zeros((L, U, w.index_centroids + 1), dtype=torch.int32, device=dev)
        cluster_pages = torch.zeros((L, U, NP), dtype=torch.int32, device=dev)
        ctx.bind_centroids(centroids, cluster_start, cluster_pages)
        torch.cuda.synchronize()
        t_index = time.perf_counter()
        ctx.build_centroids(0, w.index_iterations)
        torch.cuda.synchronize()
        t_index = time.perf_counter() - t_index
    pages = W.warm_pages(w)
    if pages is not None:
        ctx.cache_warm(0, pages.tolist() * U, [len(pages)] * U)
    tier = None
    if args.tier:
        E = args.tier_extent_pages
        n_ext = U * (-(-NP // E))
        pool_extents = max(int(args.tier_pool_frac * n_ext), args.tier_queue_depth * args.tier_max_run)
        tier_pool = torch.zeros(pool_extents * E * w.page_bytes, dtype=torch.uint8).pin_memory()
        tier = K.KvdTier(args.tier, tier_pool, n_layers=1, n_units=U, max_pages=NP, extent_pages=E, page_bytes=w.page_bytes,
                         pool_extents=pool_extents, queue_depth=args.tier_queue_depth, max_run_extents=args.tier_max_run,
                         direct_io=not args.tier_buffered)
        if args.tier_layout == "semantic":
            tier.set_layout(0, ctx.layout_from_clusters(0))
        t_write = time.perf_counter()
        tier.write_layer(0, store[0])
        t_write = time.perf_counter() - t_write
        ctx.bind_tier(tier)
    step_fn = ctx.step_tiered if tier is not None else ctx.step
    n_cal = args.calibrate + 1 if args.calibrate > 0 else 0
    n_total = args.warmup + 2 * args.steps + 1
    stream_q = [q[0].contiguous() for q in W.query_stream(w, q0, n_cal + n_total, dev)]
    # warm-up queries, then the calibration's, then the timed ones: one continuous drifting stream
    q_cal = stream_q[args.warmup:args.warmup + n_cal]
    queries = stream_q[:args.warmup] + stream_q[args.warmup + n_cal:]
    out = torch.empty((B, w.n_q_heads, D), dtype=torch.float32, device=dev)
    torch.cuda.synchronize()
    t_setup = time.perf_counter() - t_setup

    stream = torch.cuda.current_stream()
    t, base = 0, 0
    calibration = None
    for _ in range(args.warmup):
        step_fn(0, base + t, queries[t], out, stream=stream)
        t += 1
    torch.cuda.synchronize()
    if tier is not None:
        tier.reset_stats()
    if args.calibrate > 0:                       # on the warmed-up cache; its steps continue the query stream
        chosen, ms = ctx.calibrate_step_form(0, t, torch.stack(q_cal).contiguous(), args.calibrate, out, stream=stream)
        calibration = {"chosen_form": chosen, "ms_per_step": {str(f): v for f, v in ms.items()}}
        base = n_cal                             # step indices go on after the calibration's
    ctx.reset_stats()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step_fn(0, base + t, queries[t], out, stream=stream)
        t += 1
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    st = ctx.stats()
    ms_per_step = 1e3 * elapsed / args.steps
    hit_rate = st.hits / max(1, st.hits + st.misses)
    gathered_per_step = st.gathered_bytes / args.steps

    # index bytes a step must read: the page summaries, or the centroids plus the cluster lists
    summary_bytes = U * NP * D * 2 if w.index_centroids == 0 else U * (w.index_centroids * D * 2 + (w.index_centroids + 1 + NP) * 4)
    selected_bytes = U * k * w.page_bytes
    io_bytes = B * w.n_q_heads * D * (2 + 4)
    result = {
        "metric": "decode layer-steps/sec",
        "value": args.steps / elapsed,
        "unit": "layer-steps/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": {"workload": describe(w), "micro_batches": args.micro_batches, "setup_s": round(t_setup, 1)},
        "cache": {"hit_rate": hit_rate, "host_bytes_per_step": gathered_per_step,
                  "host_link_GBps_if_fetch_bound": gathered_per_step / (elapsed / args.steps) / 1e9},
    }

    if tier is not None:
        ts = tier.stats()
        seq = tier.sequential_read_gbps()                      # drops the pool; the file read front to back, same readers
        read_gbps = ts.bytes_read / max(ts.ms_io, 1e-9) / 1e6
        result["config"]["workload"] += f" + third tier (backing file, extents of {args.tier_extent_pages} pages, {args.tier_layout} order)"
        result["cache"]["host_bytes_per_step"] = ts.pages_requested * w.page_bytes / args.steps
        result["cache"].pop("host_link_GBps_if_fetch_bound")
        result["tier"] = {
            "extent_pages": args.tier_extent_pages, "extent_bytes": args.tier_extent_pages * w.page_bytes,
            "pool_extents": pool_extents, "pool_frac_of_file": pool_extents / n_ext, "queue_depth": args.tier_queue_depth,
            "max_run_extents": args.tier_max_run, "layout": args.tier_layout,
            "direct_io_mode": ts.direct_io, "file_GiB": n_ext * args.tier_extent_pages * w.page_bytes / 2**30, "file_write_s": round(t_write, 2),
            "missed_pages_per_step": ts.pages_requested / args.steps, "extents_needed_per_step": ts.extents_needed / args.steps,
            "pool_hit_rate": ts.extent_hits / max(1, ts.extents_needed), "extents_read_per_step": ts.extent_reads / args.steps,
            "read_calls_per_step": ts.reads_issued / args.steps, "file_bytes_per_step": ts.bytes_read / args.steps,
            "read_amplification": ts.bytes_read / max(1, ts.pages_requested * w.page_bytes),
            "ms_plan_per_step": ts.ms_plan / args.steps, "ms_io_per_step": ts.ms_io / args.steps,
            "ms_rest_per_step": ms_per_step - (ts.ms_plan + ts.ms_io) / args.steps,
            "read_GBps": read_gbps, "sequential_read_GBps": seq, "frac_of_sequential": read_gbps / seq if seq > 0 else None,
        }
        ctx.bind_tier(None)
        tier.close()
        os.unlink(args.tier)
    props = torch.cuda.get_device_properties(0)
    result["config"]["device"] = {"name": props.name, "arch": getattr(props, "gcnArchName", ""),
                                  "compute_units": props.multi_processor_count,
                                  "hbm_GiB": round(props.total_memory / 2**30, 1), "max_clock_MHz": _max_clock_mhz()}
    if w.index_centroids > 0:
        result["config"]["index"] = {"centroids": w.index_centroids, "kmeans_rounds": w.index_iterations,
                                     "build_s": round(t_index, 3)}
    if calibration is not None:
        result["config"]["calibration"] = calibration
    single = ctx.step_form() == -1
    result["config"]["step_form"] = "one launch (step_kernel)" if single else f"chain of kernels x {ctx.step_form()} group(s)"
    gpu_bytes = summary_bytes + selected_bytes + io_bytes
    if not args.no_profile_pass:
        # pass 2: the same workload continued as a chain of stand-alone kernels, every kernel
        # bracketed by HIP events on its stream: the stage breakdown
        ctx.set_profiling(1)
        ctx.reset_stats()
        for _ in range(args.steps):
            ctx.step(0, base + t, queries[t], out, stream=stream)
            t += 1
        torch.cuda.synchronize()
        ps = ctx.stats()
        n = max(1, ps.profiled_steps)
        ms_score, ms_attend = ps.ms_score / n, ps.ms_attend / n
        result["kernels_ms"] = {"what": "stage breakdown: the step run as a chain of stand-alone kernels, HIP events around each",
                                "score": ms_score, "select_resolve_fetch": ps.ms_select_resolve / n,
                                "fetch_separate": ps.ms_gather / n, "attend": ms_attend, "merge": ps.ms_merge / n,
                                "score_GBps": summary_bytes / (ms_score * 1e-3) / 1e9,
                                "attend_GBps": selected_bytes / (ms_attend * 1e-3) / 1e9}
        fetch_ms = (ps.ms_select_resolve + ps.ms_gather) / n
        link = ps.gathered_bytes / n / (fetch_ms * 1e-3) / 1e9
        # what a plain copy engine transfer of 1 GiB of the same pinned store reaches on this machine
        flat = store.view(-1)[: (1 << 30) // store.element_size()]
        dst = torch.empty_like(flat, device=dev)
        memcpy_gbps = 0.0
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            dst.copy_(flat, non_blocking=True)
            e1.record(stream)
            torch.cuda.synchronize()
            memcpy_gbps = max(memcpy_gbps, flat.numel() * flat.element_size() / (e0.elapsed_time(e1) * 1e-3) / 1e9)
        del dst
        result["host_link"] = {"what": "fetch of missed pages from pinned host memory inside the selection/fetch kernel (chain pass)",
                               "bytes_per_step": ps.gathered_bytes / n, "GBps_over_select_resolve_fetch": link,
                               "peak_GBps": HOST_LINK_PEAK_GBPS, "frac": link / HOST_LINK_PEAK_GBPS,
                               "pinned_memcpy_GBps": memcpy_gbps, "frac_of_pinned_memcpy": link / memcpy_gbps}

        # pass 3: the GPU-resident path alone, in the form the timed region used.  The last query is
        # replayed, so every selected page is a hit and nothing crosses the host link: time per
        # step = GPU time of score -> select -> resolve -> attend -> merge, taken with HIP events
        # on the stream around the K launches.  Bytes = summaries + selected K/V + q/out.
        ctx.set_profiling(0)
        q_last = queries[t - 1]
        for _ in range(3):
            ctx.step(0, base + t, q_last, out, stream=stream)
            t += 1
        torch.cuda.synchronize()
        ctx.reset_stats()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record(stream)
        for _ in range(args.steps):
            ctx.step(0, base + t, q_last, out, stream=stream)
            t += 1
        ev1.record(stream)
        torch.cuda.synchronize()
        res_ms = ev0.elapsed_time(ev1) / args.steps
        rs = ctx.stats()
        result["gpu_resident"] = {
            "what": "all-hit replay of one query: time per layer-step of score+select+resolve+attend+merge",
            "ms_per_step": res_ms, "layer_steps_per_s": 1e3 / res_ms, "misses": int(rs.misses), "bytes": gpu_bytes,
            "GBps": gpu_bytes / (res_ms * 1e-3) / 1e9, "frac_of_hbm_peak": gpu_bytes / (res_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        }
        if single:
            # the step is one kernel: its launch is bound by the host link while pages are missed
            # and by HBM once they are resident; the roofline is taken on the resident launches
            result["roofline"] = {"kernel": "step_kernel", "bound": "hbm", "achieved": gpu_bytes / (res_ms * 1e-3) / 1e9,
                                  "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": gpu_bytes / (res_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                                  "traffic": PMC_TRAFFIC_BYTES.get((w.name, "step")), "algorithmic_bytes_per_launch": gpu_bytes,
                                  "avg_launch_ms": res_ms,
                                  "launches": "the all-hit launches (selected pages resident); the timed region's launches "
                                              "also wait for the host-link fetch, see host_link"}
        else:
            name, ms, alg = ("attend", ms_attend, selected_bytes) if ms_attend >= ms_score else ("score", ms_score, summary_bytes)
            achieved = alg / (ms * 1e-3) / 1e9
            result["roofline"] = {"kernel": {"attend": "attend_mfma_kernel", "score": "score_kernel"}[name], "bound": "hbm",
                                  "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS,
                                  "traffic": PMC_TRAFFIC_BYTES.get((w.name, name)), "algorithmic_bytes_per_launch": alg,
                                  "avg_launch_ms": ms}

    if args.timeline and single and not args.no_profile_pass:
        result["timeline"] = step_timeline(ctx, base + t, q_last, out, stream)

    if args.layers > 1:
        result["layers_in_flight"] = layers_in_flight(args, cfg_w, K, W, torch, dev)

    if args.cpu_seconds > 0:
        q_cpu = [q.cpu() for q in queries[:16]]
        result["cpu_baseline"] = cpu_baseline(w, store, q_cpu, args.cpu_seconds)

    # one plain device copy of known size so that a counter run of this command has a calibration kernel
    a = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
    b = torch.empty_like(a)
    b.copy_(a)
    torch.cuda.synchronize()
    ctx.close()
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
