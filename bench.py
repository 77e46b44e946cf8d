#!/usr/bin/env python3
"""Benchmark of the offloaded sparse-decode layer-step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 3]

A "step" is one kvd_step: score -> select -> resolve -> fetch -> attend for one
layer over the whole batch.  The headline workload is the benchmark definition's
configuration 3 (1 layer, batch 16, 131072-token context, page 16, 32 q / 8 kv
heads, bf16, budget 4096 tokens, GPU cache 25 % of the pages, the rest in pinned
host memory) with synthetic Zipf-importance K/V; the drifting query stream is
continued past the configuration's 32 steps when more steps are asked for.

Prints one JSON line:

* `value`: end-to-end layer-steps/s of the K timed steps from a cold cache (fetch
  of missed pages from pinned host memory included; index, cache and queries
  resident in HBM).
* `gpu_resident`: the same step with every selected page already resident, so
  that nothing crosses the host link and wall time is GPU time, two ways:
  `replay_one_query` (the last query replayed) and `rotating` (the library's
  pre-run calibration of the launch shape aside, the launches rotate over
  several layers, each with its own index and slot pool, and over a cycle of
  drifting queries per layer, so that no launch touches what the launches just
  before it touched and the working set is several times the memory-side
  cache).  Each is the median of several repeats of a batch of launches between
  two HIP events on the launch stream, with the spread.
* `roofline`: the dominant kernel against the HBM roofline: the one-launch
  `step_kernel` on the rotating resident launches when the step runs as one
  launch (the timed region's launches of the same kernel also wait for the
  host link); else the larger of the scoring / attention kernels of the chain.
* `configs`: the other four configurations of the benchmark definition at one
  layer's worth of state of their full per-layer shape, each with end-to-end
  layer-steps/s, hit rate, host-link rate and the GPU-resident time and HBM
  fraction, and for the multi-layer configurations also with the layers of a
  decode step overlapped (kvd_step_layers).
* `kernels_ms`, `host_link`: the stage breakdown of the chain of stand-alone
  kernels and the host-link rate inside the fetch.
* `cpu_baseline`: the CPU oracle as it stands, timed on a bounded sample of the
  headline workload by worker processes on the host cores.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import math
import multiprocessing
import os
import sys
import tempfile
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
HOST_LINK_PEAK_GBPS = 63.0      # PCIe Gen5 x16, one direction: 32 GT/s x 16 lanes x 128/130
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "pmc_traffic.json")
CSRC = os.path.join(ROOT, "paper_2605_18071_amd", "csrc")


def describe(w) -> str:
    return (f"{w.name}: L={w.n_layers} B={w.batch} ctx={w.ctx} page={w.page} heads={w.n_q_heads}q/{w.n_kv_heads}kv "
            f"D={w.head_dim} {w.dtype} k={w.topk_pages} pages ({w.topk_pages * w.page} tokens) "
            f"{'flat index' if w.index_centroids == 0 else str(w.index_centroids) + ' centroids'} cache={w.capacity} pages/unit ({100.0 * w.capacity / w.n_pages:.0f}%, {w.policy}{' pool ' + str(w.lookahead_pool) if w.lookahead_pool else ''}) "
            f"{w.importance} importance, rho={w.rho}")


def kernel_source_hash() -> str:
    """Hash of the HIP sources the library is built from: ties stored counter readings to a build."""
    h = hashlib.sha256()
    for name in sorted(os.listdir(CSRC)):
        if name.endswith((".hip", ".h")):
            h.update(name.encode())
            h.update(open(os.path.join(CSRC, name), "rb").read())
    return h.hexdigest()[:16]


def traffic_variant(args) -> str:
    """Suffix of a workload's name in the stored counter readings: empty for the configuration as
    defined, else the flags that change what a launch reads or writes."""
    tags = []
    if args.centroids:
        tags.append(f"centroids{args.centroids}")
    if args.policy != "lru":
        tags.append(args.policy + (f"{args.lookahead_pool:g}" if args.lookahead_pool else ""))
    if args.window:
        tags.append(f"window{args.window:g}")
    if args.batch:
        tags.append(f"batch{args.batch}")
    if args.page_size:
        tags.append(f"page{args.page_size}")
    if args.ctx:
        tags.append(f"ctx{args.ctx}")
    if args.tier:
        tags.append("tier")
    return "".join("+" + t for t in tags)


def stored_traffic(workload: str, kernel: str):
    """HBM bytes per launch of `kernel` on `workload` (a configuration's name plus traffic_variant)
    from the stored rocprofv3 counter readings (profiles/pmc_traffic.json), or (None, reason) when
    there are none for this build."""
    try:
        rec = json.load(open(TRAFFIC_FILE))
    except (OSError, ValueError):
        return None, "no stored counter readings"
    have = kernel_source_hash()
    if rec.get("kernel_source_hash") != have:
        return None, (f"the stored counter readings were taken on kernel sources {rec.get('kernel_source_hash')}, "
                      f"this build is {have}")
    e = rec.get("kernels", {}).get(f"{workload}:{kernel}")
    if e is None:
        return None, f"no counter reading stored for {kernel} on {workload}"
    return int(e["hbm_bytes_per_launch"]), None


# ---------------------------------------------------------------------------------------------
# the oracle on the host cores
# ---------------------------------------------------------------------------------------------
def _oracle_worker(task):
    """One worker process: the oracle, as it stands, over the decode steps of one unit for about
    `seconds`.  Returns (unit-steps done, seconds spent in them)."""
    import numpy as np
    try:
        from threadpoolctl import threadpool_limits
        limit = threadpool_limits(limits=1)             # one core per worker
    except Exception:
        limit = None
    from oracle import kvd_oracle as orc
    path, meta, seconds = task
    z = np.load(path)
    code = orc.F16 if meta["dtype"] == "f16" else orc.BF16
    keys = orc.bits_to_f64(z["k"], code).reshape(-1, meta["D"])
    vals = orc.bits_to_f64(z["v"], code).reshape(-1, meta["D"])
    qs = orc.bits_to_f64(z["q"], code)                   # [steps, G, D]
    summ = orc.page_summaries(keys, meta["page"], meta["ctx"], code)         # set-up, not timed
    cent = members = None
    if meta["centroids"] > 0:                                                 # index build: set-up, not timed
        cent, assign, _ = orc.kmeans_centroids(summ, meta["centroids"], meta["iterations"], code)
        members = orc.cluster_members(assign, meta["centroids"])
    win = (orc.LookaheadWindow if meta["policy"] == "lookahead" else orc.LruWindow)(meta["capacity"])
    scale = 1.0 / math.sqrt(meta["D"])
    done, spent, t = 0, 0.0, 0
    while spent < seconds and t < 64 * len(qs):
        t0 = time.perf_counter()
        orc.decode_unit_step(qs[t % len(qs)], summ, keys, vals, win, t, k=meta["k"], page_size=meta["page"],
                             seq_len=meta["ctx"], scale=scale, sink_pages=meta["sink"], recent_pages=meta["recent"], centroids=cent,
                             members=members)
        spent += time.perf_counter() - t0
        done += 1
        t += 1
    del limit
    return done, spent


class OraclePool:
    """Worker processes for the oracle's timing, forked before anything touches the GPU."""

    def __init__(self, workers: int):
        self.workers = workers
        self.pool = multiprocessing.get_context("fork").Pool(workers) if workers > 0 else None

    def run(self, w, store, q_list, seconds: float):
        import numpy as np
        import torch
        n = min(self.workers, w.units)
        tmp = tempfile.mkdtemp(prefix="kvd_oracle_", dir="/dev/shm" if os.path.isdir("/dev/shm") else None)
        tasks = []
        meta = dict(dtype=w.dtype, D=w.head_dim, page=w.page, ctx=w.ctx, policy=w.policy, capacity=w.capacity,
                    k=w.topk_pages, sink=w.sink_pages, recent=w.recent_pages, centroids=w.index_centroids,
                    iterations=w.index_iterations)
        try:
            for i in range(n):
                u = (i * w.units) // n
                b, h = divmod(u, w.n_kv_heads)
                kv = store[0, b, h]
                raw = lambda t: t.contiguous().view(torch.int16).numpy().view(np.uint16)
                q = torch.stack([x[b, h * w.group:(h + 1) * w.group] for x in q_list])
                path = os.path.join(tmp, f"unit{u}.npz")
                np.savez(path, k=raw(kv[:, 0]), v=raw(kv[:, 1]), q=raw(q))
                tasks.append((path, meta, seconds))
            t0 = time.perf_counter()
            res = self.pool.map(_oracle_worker, tasks, chunksize=1)
            wall = time.perf_counter() - t0
        finally:
            for f in os.listdir(tmp):
                os.unlink(os.path.join(tmp, f))
            os.rmdir(tmp)
        done = sum(r[0] for r in res)
        busy = sum(r[1] for r in res)
        rate = sum(r[0] / r[1] for r in res if r[1] > 0)           # unit-steps per second of the n workers together
        return {
            "value": rate / w.units,
            "unit": "layer-steps/s",
            "cores": n,
            "kind": "oracle",
            "sample": f"{done} unit-steps ({n} of {w.units} units, one worker process and one core each, {len(q_list)} drifting "
                      f"queries taken in turn) in {busy / n:.1f} s per worker ({wall:.1f} s with loading), scaled to one "
                      f"layer-step = {w.units} units",
        }

    def close(self):
        if self.pool is not None:
            self.pool.close()
            self.pool.join()


# ---------------------------------------------------------------------------------------------
# one configuration on the GPU
# ---------------------------------------------------------------------------------------------
def _stats(xs):
    xs = sorted(xs)
    n = len(xs)
    med = xs[n // 2] if n % 2 else 0.5 * (xs[n // 2 - 1] + xs[n // 2])
    return med, xs[0], xs[-1]


class Bench:
    """One workload on the device: `rot_layers` layers, each with its own index, directory and
    slot pool, over one stored layer.  Layer 0 carries the end-to-end run; all layers carry the
    GPU-resident launches."""

    def __init__(self, w, args, torch, K, W, rot_layers: int):
        self.torch, self.K, self.W, self.args = torch, K, W, args
        dev = "cuda:0"
        self.w1 = w                                                      # the configuration at one layer
        L = max(1, rot_layers)
        self.w = w.replace(n_layers=L, physical_layers=1)
        w = self.w
        B, Hkv, NP, P, D, U, k = w.batch, w.n_kv_heads, w.n_pages, w.page, w.head_dim, w.units, w.topk_pages
        t0 = time.perf_counter()
        q0 = W.initial_queries(w.replace(n_layers=1), dev)              # every layer starts from the stored layer's query
        self.q0 = q0.expand(L, -1, -1, -1).contiguous()
        self.store = W.make_kv_store(w.replace(n_layers=1), q0, dev)
        self.summ = torch.zeros((L, B, Hkv, NP, D), dtype=w.torch_dtype, device=dev)
        self.pool = torch.zeros((L, B, Hkv, w.capacity, 2, P, D), dtype=w.torch_dtype, device=dev)
        self.ctx = K.Kvd(n_layers=L, batch=B, n_q_heads=w.n_q_heads, n_kv_heads=Hkv, page_size=P, max_pages=NP, topk_pages=k,
                         capacity_max=w.capacity, kv_dtype=w.torch_dtype, sink_pages=w.sink_pages, recent_pages=w.recent_pages,
                         physical_layers=1, micro_batches=args.micro_batches, policy=w.policy,
                         index_centroids=w.index_centroids, lookahead_pool=w.lookahead_pool)
        self.ctx.bind_summaries(self.summ)
        self.ctx.bind_host_store(self.store)
        self.ctx.bind_slot_pool(self.pool)
        for l in range(L):
            self.ctx.build_summaries(l)
        self.index_build_s = None
        if w.index_centroids > 0:
            self.centroids = torch.zeros((L, B, Hkv, w.index_centroids, D), dtype=w.torch_dtype, device=dev)
            self.cluster_start = torch.zeros((L, U, w.index_centroids + 1), dtype=torch.int32, device=dev)
            self.cluster_pages = torch.zeros((L, U, NP), dtype=torch.int32, device=dev)
            self.ctx.bind_centroids(self.centroids, self.cluster_start, self.cluster_pages)
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for l in range(L):
                self.ctx.build_centroids(l, w.index_iterations)
            torch.cuda.synchronize()
            self.index_build_s = (time.perf_counter() - t1) / L
        self.warm_cache()
        self.out = torch.empty((L, B, w.n_q_heads, D), dtype=torch.float32, device=dev)
        self.stream = torch.cuda.current_stream()
        torch.cuda.synchronize()
        self.setup_s = time.perf_counter() - t0
        self.L, self.U = L, U
        self.summary_bytes = (U * NP * D * 2 if w.index_centroids == 0 else
                              U * (w.index_centroids * D * 2 + (w.index_centroids + 1 + NP) * 4))
        self.selected_bytes = U * k * w.page_bytes
        self.gpu_bytes = self.summary_bytes + self.selected_bytes + B * w.n_q_heads * D * (2 + 4)
        self.t = 0                                                      # next step index (all layers)
        self.calibration = None

    def warm_cache(self):
        pages = self.W.warm_pages(self.w)
        if pages is not None:
            for l in range(self.w.n_layers):
                self.ctx.cache_warm(l, pages.tolist() * self.w.units, [len(pages)] * self.w.units)

    def queries(self, n):
        """n steps of the drifting per-layer query streams, [L, B, Hq, D] each."""
        return [q.contiguous() for q in self.W.query_stream(self.w, self.q0, n, "cuda:0")]

    def close(self):
        self.ctx.close()

    # -- pre-run calibration of the launch shape, on the last layer (layer 0's cache stays as it is)
    def calibrate_shape(self, q_layers, multi_layer=False):
        if self.ctx.step_form() != -1 or self.args.no_shape_calibration:
            return
        l = self.L - 1
        rule = self.ctx.step_shape()
        shape, us, us_rule = self.ctx.calibrate_step_shape(l, 0, q_layers[l], self.out[l], 16, stream=self.stream)
        self.calibration = {"what": "kvd_calibrate_step_shape before the run: (passes per scoring chunk, scoring workgroups, "
                                    "attention splits per unit, groups of units), microseconds per resident launch",
                            "rule": list(rule), "rule_us": us_rule, "chosen": list(shape), "chosen_us": us}
        if l == 0:                                                      # a context of one layer: start again from a cold cache
            self.ctx.cache_reset()
            self.warm_cache()
        elif multi_layer and self.L >= 3:
            # launches of several layers have a shape of their own: calibrated on layers 1.. (layer 0 stays cold)
            rule = self.ctx.step_shape(multi_layer=True)
            shape, us, us_rule = self.ctx.calibrate_step_shape(1, 0, q_layers[1:], self.out[1:], 8, n_layers=self.L - 1,
                                                               stream=self.stream)
            self.calibration["several_layers_per_launch"] = {"rule": list(rule), "rule_us_per_layer_step": us_rule,
                                                             "chosen": list(shape), "chosen_us_per_layer_step": us}

    # -- the end-to-end run on layer 0
    def end_to_end(self, qs, warmup, steps, step_fn=None):
        torch = self.torch
        step_fn = step_fn or self.ctx.step
        for i in range(warmup):
            step_fn(0, self.t, qs[i][0], self.out[0], stream=self.stream)
            self.t += 1
        torch.cuda.synchronize()
        self.ctx.reset_stats()
        t0 = time.perf_counter()
        for i in range(steps):
            step_fn(0, self.t, qs[warmup + i][0], self.out[0], stream=self.stream)
            self.t += 1
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        st = self.ctx.stats()
        return {"elapsed": elapsed, "ms_per_step": 1e3 * elapsed / steps, "hit_rate": st.hits / max(1, st.hits + st.misses),
                "host_bytes_per_step": st.gathered_bytes / steps,
                "host_link_GBps": st.gathered_bytes / elapsed / 1e9}

    # -- GPU-resident launches
    def _timed_batches(self, launch_batch, n_launches, repeats):
        """`repeats` batches of launches, each between two HIP events on the launch stream."""
        torch = self.torch
        launch_batch()                                                  # untimed: brings code, TLBs and (first time) pages in
        torch.cuda.synchronize()
        self.ctx.reset_stats()
        us = []
        for _ in range(repeats):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(self.stream)
            launch_batch()
            e1.record(self.stream)
            torch.cuda.synchronize()
            us.append(1e3 * e0.elapsed_time(e1) / n_launches)
        misses = int(self.ctx.stats().misses)
        med, lo, hi = _stats(us)
        return {"us_per_launch_median": med, "us_min": lo, "us_max": hi, "repeats": repeats, "launches_per_repeat": n_launches,
                "misses": misses, "bytes_per_launch": self.gpu_bytes, "GBps": self.gpu_bytes / (med * 1e-6) / 1e9,
                "frac_of_hbm_peak": self.gpu_bytes / (med * 1e-6) / 1e9 / HBM_PEAK_GBPS}

    def resident_replay(self, q_layer0, n_launches=20, repeats=5):
        def batch():
            for _ in range(n_launches):
                self.ctx.step(0, self.t, q_layer0, self.out[0], stream=self.stream)
        r = self._timed_batches(batch, n_launches, repeats)
        r["what"] = "the last query replayed on one layer: every launch reads the same index and the same selected pages"
        return r

    def resident_rotating(self, cycle, repeats=5, in_flight=False):
        """cycle: M steps of per-layer queries.  Launch order: query-major, layer-minor, so that
        consecutive launches belong to different layers.  The cycle is run twice untimed first: all
        the pages its queries select are then resident (the window holds several times what the
        cycle touches), and the timed launches fetch nothing."""
        L, M = self.L, len(cycle)

        def batch():
            for m in range(M):
                if in_flight:
                    self.ctx.step_layers(0, L, self.t, cycle[m], self.out, stream=self.stream)
                else:
                    for l in range(L):
                        self.ctx.step(l, self.t, cycle[m][l], self.out[l], stream=self.stream)
        batch()
        r = self._timed_batches(batch, M * L, repeats)
        r["what"] = (f"{L} layers (own index, directory and slot pool each) x a cycle of {M} drifting queries per layer, "
                     f"consecutive launches on different layers" + (", all layers of a cycle step in one kvd_step_layers call" if in_flight else ""))
        r["working_set_bytes"] = L * self.summary_bytes + L * self.selected_bytes
        return r


def brief_config(cfg_id, args, torch, K, W):
    """One of the other configurations: end to end from its initial cache state, then GPU-resident."""
    w = W.CONFIGS[cfg_id]
    multi = w.n_layers > 1
    w1 = w.replace(n_layers=1, physical_layers=1)
    b = Bench(w1, args, torch, K, W, rot_layers=2 * args.rot_layers if multi else args.rot_layers)
    steps = min(w.steps, 32) if w.steps > 1 else 8                     # cfg1 is one step by definition: a few more for a stable time
    warmup = 2 if w.warm == "cold" else 1
    cyc = 8
    qs = b.queries(warmup + steps + cyc)
    b.calibrate_shape(qs[0], multi_layer=multi)
    e2e = b.end_to_end(qs, warmup, steps)
    res = {"workload": describe(w1), "layers_of_state": 1, "steps": steps, "warmup": warmup,
           "step_form": "one launch (step_kernel)" if b.ctx.step_form() == -1 else f"chain of kernels x {b.ctx.step_form()} group(s)",
           "layer_steps_per_s": steps / e2e["elapsed"], "ms_per_step": e2e["ms_per_step"], "hit_rate": e2e["hit_rate"],
           "host_bytes_per_step": e2e["host_bytes_per_step"], "host_link_GBps": e2e["host_link_GBps"],
           "setup_s": round(b.setup_s, 1)}
    if b.calibration:
        res["launch_shape"] = b.calibration
    cycle = qs[warmup + steps:]
    rot = b.resident_rotating(cycle)
    res["gpu_resident"] = {k: rot[k] for k in ("what", "us_per_launch_median", "us_min", "us_max", "misses", "bytes_per_launch", "GBps",
                                               "frac_of_hbm_peak", "working_set_bytes")}
    if multi and b.L >= 2:
        fl = b.resident_rotating(cycle, in_flight=True)
        res["gpu_resident_layers_overlapped"] = {k: fl[k] for k in ("what", "us_per_launch_median", "us_min", "us_max", "misses",
                                                                      "GBps", "frac_of_hbm_peak")}
    b.close()
    del b
    torch.cuda.empty_cache()
    if multi:
        # the configuration's decode step goes through many layers: 8 of them per decode step, end to end with
        # the real miss stream, stepped one by one and with the layers sharing launches
        import copy
        a8 = copy.copy(args)
        a8.layers, a8.steps, a8.warmup = 8, 64, 4
        res["decode_step_of_8_layers"] = layers_in_flight(a8, w, K, W, torch, "cuda:0")
        torch.cuda.empty_cache()
    return res


def layers_in_flight(args, cfg_w, K, W, torch, dev):
    """The configuration's layer-step over `--layers` layers of one decode step, layers one by one
    (kvd_step per layer) against the layers overlapped (kvd_step_layers: one launch per 8 layers, or
    two chains of kernels in flight): end-to-end ms per layer-step including the fetch of missed
    pages, cold start, the first `warmup` decode steps untimed."""
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
    for mode in ("one_by_one", "overlapped"):
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


def record_traffic(args) -> int:
    """Writes profiles/pmc_traffic.json from two rocprofv3 --pmc runs of this command (one with
    FETCH_SIZE, one with WRITE_SIZE; `--record-traffic FETCH.csv WRITE.csv`, the counter_collection
    CSVs): per kernel, the counter's mean per dispatch (KiB), scaled by what the same counter reads
    for the plain copy of known size that every run of this command ends with."""
    import csv
    import re
    from paper_2605_18071_amd import workloads as W
    w = W.CONFIGS[args.config]
    copy_bytes = 256 << 20                                        # the calibration copy: reads and writes this much

    def per_kernel(path, counter):
        acc = {}
        for row in csv.DictReader(open(path)):
            if row.get("Counter_Name") != counter:
                continue
            name = row["Kernel_Name"]
            acc.setdefault(name, []).append(float(row["Counter_Value"]))
        return acc

    fetch, write = per_kernel(args.record_traffic[0], "FETCH_SIZE"), per_kernel(args.record_traffic[1], "WRITE_SIZE")

    def pick(acc, pattern):
        for name, vals in acc.items():
            if re.search(pattern, name):
                return vals
        return None

    def copy_reading(acc):
        # the calibration copy is the run's last device-to-device buffer copy (256 MiB)
        for name, vals in acc.items():
            if "copyBuffer" in name:
                return vals[-1]
        return None

    cal_f, cal_w = copy_reading(fetch), copy_reading(write)
    if not cal_f or not cal_w:
        print("record-traffic: the calibration copy kernel was not found in the CSVs", file=sys.stderr)
        return 2
    scale_f, scale_w = copy_bytes / (cal_f * 1024.0), copy_bytes / (cal_w * 1024.0)
    kernels = {}
    for key, pattern in (("step", r"step_kernel"), ("score", r"score_kernel"), ("attend", r"attend_mfma_kernel")):
        f, wv = pick(fetch, pattern), pick(write, pattern)
        if not f or not wv:
            continue
        # resident launches are the cheap majority: the median dispatch leaves the first, fetching launches out
        fm, wm = sorted(f)[len(f) // 2], sorted(wv)[len(wv) // 2]
        kernels[f"{w.name}{traffic_variant(args)}:{key}"] = {"fetch_KiB_median": fm, "write_KiB_median": wm, "dispatches": len(f),
                                      "hbm_bytes_per_launch": int(fm * 1024 * scale_f + wm * 1024 * scale_w)}
    rec = {"what": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (KiB per dispatch, median over a kernel's dispatches) of `python3 bench.py "
                   "--config N --no-other-configs --cpu-seconds 0`, scaled by the same counter's reading for a plain 256 MiB device copy",
           "kernel_source_hash": kernel_source_hash(), "fetch_scale": scale_f, "write_scale": scale_w,
           "copy_fetch_KiB": cal_f, "copy_write_KiB": cal_w, "kernels": kernels}
    old = {}
    try:
        old = json.load(open(TRAFFIC_FILE))
    except (OSError, ValueError):
        pass
    if old.get("kernel_source_hash") == rec["kernel_source_hash"]:
        merged = dict(old.get("kernels", {}))
        merged.update(kernels)
        rec["kernels"] = merged
    json.dump(rec, open(TRAFFIC_FILE, "w"), indent=1)
    print(json.dumps(rec, indent=1))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=62)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=3)
    ap.add_argument("--micro-batches", type=int, default=0, help="kvd_config.micro_batches (0 = library chooses, 1 = chain of kernels, -1 = one launch)")
    ap.add_argument("--policy", choices=["lru", "lookahead"], default="lru", help="cache replacement policy")
    ap.add_argument("--lookahead-pool", type=float, default=0.0, metavar="X",
                    help="with --policy lookahead: look-ahead candidate pool of X times the per-step budget k (0 = every page)")
    ap.add_argument("--centroids", type=int, default=0,
                    help="hierarchical index with this many centroids per unit (0 = flat page index)")
    ap.add_argument("--index-iterations", type=int, default=4, help="k-means rounds of the hierarchical index build")
    ap.add_argument("--window", type=float, default=0.0,
                    help="cache capacity as a multiple of the per-step budget k (the paper's window size); "
                         "0 keeps the configuration's capacity")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="0 skips the oracle baseline")
    ap.add_argument("--cpu-workers", type=int, default=0, help="worker processes of the oracle baseline (0 = the host's cores, 16 at most)")
    ap.add_argument("--no-profile-pass", action="store_true", help="skip the per-kernel HIP-event pass and the GPU-resident passes")
    ap.add_argument("--no-other-configs", action="store_true", help="skip the brief runs of the other configurations")
    ap.add_argument("--no-shape-calibration", action="store_true", help="keep the library's rule for the one-launch step's launch shape")
    ap.add_argument("--rot-layers", type=int, default=4, help="layers the GPU-resident launches rotate over")
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
    ap.add_argument("--page-size", type=int, default=0, metavar="P",
                    help="P > 0: the configuration with pages of P tokens (4, 8 or a multiple of 16); budget and cache keep their tokens")
    ap.add_argument("--ctx", type=int, default=0, metavar="T", help="T > 0: the configuration with a context of T tokens")
    ap.add_argument("--layers", type=int, default=1, metavar="N",
                    help="N > 1: add a leg that steps N layers per decode step, one by one and overlapped (kvd_step_layers)")
    ap.add_argument("--timeline", action="store_true",
                    help="when the step runs as one launch: add the per-workgroup timeline of one all-hit step")
    ap.add_argument("--record-traffic", nargs=2, metavar=("FETCH_CSV", "WRITE_CSV"), default=None,
                    help="no GPU work: write profiles/pmc_traffic.json from two rocprofv3 --pmc counter CSVs of this command")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this path is built and measured on one GPU only (no collectives, no sharding); "
              "run with --gpus 1", file=sys.stderr)
        return 2
    if args.record_traffic:
        return record_traffic(args)

    # the oracle's worker processes are forked first, before anything in this process touches the GPU
    workers = 0
    if args.cpu_seconds > 0:
        workers = args.cpu_workers if args.cpu_workers > 0 else min(16, os.cpu_count() or 1)
    oracle_pool = OraclePool(workers)

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
        w = w.replace(batch=args.batch)
    if args.ctx > 0:
        # another context length: the cache keeps its share of the pages, the budget its tokens
        w = w.replace(ctx=args.ctx, capacity=max(w.topk_pages, w.capacity * args.ctx // w.ctx))
    if args.page_size > 0 and args.page_size != w.page:
        # another page size: the token budget, the cache's tokens and the forced windows stay what they are
        P0, P1 = w.page, args.page_size
        rescale = lambda n: n * P0 // P1
        w = w.replace(page=P1, topk_pages=rescale(w.topk_pages), capacity=rescale(w.capacity), heavy_count=rescale(w.heavy_count),
                      sink_pages=rescale(w.sink_pages), recent_pages=rescale(w.recent_pages))
    cfg_w = w
    if w.n_layers != 1:
        # multi-layer configurations are benchmarked on one layer's worth of state at full per-layer shape
        w = w.replace(n_layers=1, physical_layers=1)
    if args.window > 0:
        w = w.replace(capacity=max(w.topk_pages, int(round(args.window * w.topk_pages))))
    w = w.replace(policy=args.policy, index_centroids=args.centroids, index_iterations=args.index_iterations,
                  lookahead_pool=int(round(args.lookahead_pool * w.topk_pages)))
    plain = not args.tier
    multi = cfg_w.n_layers > 1                  # a multi-layer configuration: its layers can share a launch (kvd_step_layers)
    rot_layers = (2 * args.rot_layers if multi else args.rot_layers) if (plain and not args.no_profile_pass) else 1

    b = Bench(w, args, torch, K, W, rot_layers)
    ctx, stream, out = b.ctx, b.stream, b.out
    U, NP, k = w.units, w.n_pages, w.topk_pages
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
        tier.write_layer(0, b.store[0])
        t_write = time.perf_counter() - t_write
        ctx.bind_tier(tier)
    step_fn = ctx.step_tiered if tier is not None else None
    n_cal = args.calibrate + 1 if args.calibrate > 0 else 0
    cyc = 8
    stream_q = b.queries(n_cal + args.warmup + 2 * args.steps + 1 + cyc)
    # warm-up queries, then the calibration's, then the timed ones: one continuous drifting stream
    q_cal = stream_q[args.warmup:args.warmup + n_cal]
    queries = stream_q[:args.warmup] + stream_q[args.warmup + n_cal:]
    if tier is None:
        b.calibrate_shape(stream_q[0], multi_layer=multi)

    calibration = None
    if args.calibrate > 0:                       # kvd_calibrate_step_form on the warmed-up cache; its steps continue the query stream
        for i in range(args.warmup):
            (step_fn or ctx.step)(0, b.t, queries[i][0], out[0], stream=stream)
            b.t += 1
        torch.cuda.synchronize()
        chosen, ms = ctx.calibrate_step_form(0, b.t, torch.stack([q[0] for q in q_cal]).contiguous(), args.calibrate, out[0],
                                             stream=stream)
        calibration = {"chosen_form": chosen, "ms_per_step": {str(f): v for f, v in ms.items()}}
        b.t += n_cal
        e2e = b.end_to_end(queries[args.warmup:], 0, args.steps, step_fn)
    else:
        if tier is not None:
            tier.reset_stats()
        e2e = b.end_to_end(queries, args.warmup, args.steps, step_fn)
    elapsed, ms_per_step = e2e["elapsed"], e2e["ms_per_step"]
    used = args.warmup + args.steps                                   # queries consumed from `queries`

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
        "config": {"workload": describe(w), "micro_batches": args.micro_batches, "setup_s": round(b.setup_s, 1)},
        "cache": {"hit_rate": e2e["hit_rate"], "host_bytes_per_step": e2e["host_bytes_per_step"],
                  "host_link_GBps_if_fetch_bound": e2e["host_link_GBps"]},
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
                                     "build_s": round(b.index_build_s, 3)}
    if calibration is not None:
        result["config"]["calibration"] = calibration
    if b.calibration is not None:
        result["config"]["launch_shape"] = b.calibration
    single = ctx.step_form() == -1
    result["config"]["step_form"] = "one launch (step_kernel)" if single else f"chain of kernels x {ctx.step_form()} group(s)"
    q_last = queries[used - 1][0]
    if not args.no_profile_pass:
        # pass 2: the same workload continued as a chain of stand-alone kernels, every kernel
        # bracketed by HIP events on its stream: the stage breakdown
        ctx.set_profiling(1)
        ctx.reset_stats()
        for i in range(args.steps):
            ctx.step(0, b.t, queries[used + i][0], out[0], stream=stream)
            b.t += 1
        torch.cuda.synchronize()
        used += args.steps
        q_last = queries[used - 1][0]
        ps = ctx.stats()
        n = max(1, ps.profiled_steps)
        ms_score, ms_attend = ps.ms_score / n, ps.ms_attend / n
        result["kernels_ms"] = {"what": "stage breakdown: the step run as a chain of stand-alone kernels, HIP events around each",
                                "score": ms_score, "select_resolve_fetch": ps.ms_select_resolve / n,
                                "fetch_separate": ps.ms_gather / n, "attend": ms_attend, "merge": ps.ms_merge / n,
                                "score_GBps": b.summary_bytes / (ms_score * 1e-3) / 1e9,
                                "attend_GBps": b.selected_bytes / (ms_attend * 1e-3) / 1e9}
        fetch_ms = (ps.ms_select_resolve + ps.ms_gather) / n
        link = ps.gathered_bytes / n / (fetch_ms * 1e-3) / 1e9
        # what a plain copy engine transfer of 1 GiB of the same pinned store reaches on this machine
        flat = b.store.view(-1)[: (1 << 30) // b.store.element_size()]
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

        # pass 3: the GPU-resident path alone, in the form the timed region used: nothing crosses
        # the host link, so wall time = GPU time of score -> select -> resolve -> attend -> merge.
        # Bytes = index + selected K/V + q/out.
        ctx.set_profiling(0)
        replay = b.resident_replay(q_last)
        cycle = queries[used:used + cyc]
        rotating = b.resident_rotating(cycle)
        result["gpu_resident"] = {"replay_one_query": replay, "rotating": rotating,
                                  "rotating_over_replay": rotating["us_per_launch_median"] / replay["us_per_launch_median"]}
        if multi and b.L >= 2:
            result["gpu_resident"]["layers_overlapped"] = b.resident_rotating(cycle, in_flight=True)
        if single:
            # the step is one kernel: its launch is bound by the host link while pages are missed
            # and by HBM once they are resident; the roofline is taken on the resident launches
            traffic, why = stored_traffic(w.name + traffic_variant(args), "step")
            med = rotating["us_per_launch_median"]
            result["roofline"] = {"kernel": "step_kernel", "bound": "hbm", "achieved": rotating["GBps"], "peak": HBM_PEAK_GBPS,
                                  "unit": "GB/s", "frac": rotating["GBps"] / HBM_PEAK_GBPS, "traffic": traffic,
                                  "algorithmic_bytes_per_launch": b.gpu_bytes, "avg_launch_ms": med * 1e-3,
                                  "launch_us_median_min_max": [med, rotating["us_min"], rotating["us_max"]],
                                  "frac_replay_one_query": replay["frac_of_hbm_peak"],
                                  "launches": "the resident launches rotating over layers and drifting queries (gpu_resident.rotating); "
                                              "the timed region's launches of the same kernel also wait for the host-link fetch, see host_link"}
            if why:
                result["roofline"]["traffic_note"] = why
        else:
            name, ms, alg = ("attend", ms_attend, b.selected_bytes) if ms_attend >= ms_score else ("score", ms_score, b.summary_bytes)
            achieved = alg / (ms * 1e-3) / 1e9
            traffic, why = stored_traffic(w.name + traffic_variant(args), name)
            result["roofline"] = {"kernel": {"attend": "attend_mfma_kernel", "score": "score_kernel"}[name], "bound": "hbm",
                                  "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS,
                                  "traffic": traffic, "algorithmic_bytes_per_launch": alg, "avg_launch_ms": ms}
            if why:
                result["roofline"]["traffic_note"] = why

    if args.timeline and single and not args.no_profile_pass:
        result["timeline"] = step_timeline(ctx, b.t, q_last, out[0], stream)

    if args.layers > 1:
        result["layers_in_flight"] = layers_in_flight(args, cfg_w, K, W, torch, dev)

    if args.cpu_seconds > 0:
        q_cpu = [q[0].cpu() for q in queries[:16]]
        result["cpu_baseline"] = oracle_pool.run(w, b.store, q_cpu, args.cpu_seconds)
    oracle_pool.close()
    b.close()
    del b, ctx, out
    torch.cuda.empty_cache()

    if plain and not args.no_other_configs and not args.no_profile_pass and args.batch == 0:
        result["configs"] = {}
        for c in (1, 2, 4, 5, 3):
            if c != args.config:
                result["configs"][f"cfg{c}"] = brief_config(c, args, torch, K, W)

    # one plain device copy of known size so that a counter run of this command has a calibration kernel
    a = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
    c2 = torch.empty_like(a)
    c2.copy_(a)
    torch.cuda.synchronize()
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
