"""ctypes binding of libkvd (see include/kvd.h).  Argument marshalling only: every
stage of the decode step runs in the HIP kernels of the library.  Tensors are
passed as raw device / pinned-host pointers; torch is used for memory and streams.

Loading fails loudly (ImportError) if the library has not been built:
    python -m paper_2605_18071_amd.build
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libkvd.so")

KVD_F16, KVD_BF16 = 0, 1
KVD_EVICT_LRU, KVD_EVICT_LOOKAHEAD = 0, 1
OK, ERR_ARG, ERR_SHAPE, ERR_CAPACITY, ERR_DTYPE, ERR_HIP, ERR_STATE = 0, -1, -2, -3, -4, -5, -6


class KvdConfig(C.Structure):
    _fields_ = [
        ("n_layers", C.c_int32), ("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
        ("head_dim", C.c_int32), ("page_size", C.c_int32), ("max_pages", C.c_int32), ("topk_pages", C.c_int32),
        ("sink_pages", C.c_int32), ("recent_pages", C.c_int32), ("kv_dtype", C.c_int32), ("policy", C.c_int32),
        ("softmax_scale", C.c_float), ("capacity_max", C.c_int32), ("capacity", C.POINTER(C.c_int32)),
        ("physical_layers", C.c_int32), ("micro_batches", C.c_int32), ("attn_splits", C.c_int32),
        ("index_centroids", C.c_int32), ("lookahead_pool", C.c_int32),
    ]


class KvdTierConfig(C.Structure):
    _fields_ = [
        ("n_layers", C.c_int32), ("n_units", C.c_int32), ("max_pages", C.c_int32), ("extent_pages", C.c_int32),
        ("page_bytes", C.c_int64), ("pool_extents", C.c_int64), ("queue_depth", C.c_int32),
        ("max_run_extents", C.c_int32), ("direct_io", C.c_int32),
    ]


class KvdTierStats(C.Structure):
    _fields_ = [
        ("steps", C.c_uint64), ("pages_requested", C.c_uint64), ("extents_needed", C.c_uint64),
        ("extent_hits", C.c_uint64), ("extent_reads", C.c_uint64), ("extent_evictions", C.c_uint64),
        ("reads_issued", C.c_uint64), ("bytes_read", C.c_uint64), ("ms_plan", C.c_double), ("ms_io", C.c_double),
        ("direct_io", C.c_int32),
    ]


class KvdStats(C.Structure):
    _fields_ = [
        ("steps", C.c_uint64), ("hits", C.c_uint64), ("misses", C.c_uint64), ("evictions", C.c_uint64),
        ("gathered_bytes", C.c_uint64),
        ("ms_score", C.c_double), ("ms_select_resolve", C.c_double), ("ms_gather", C.c_double),
        ("ms_attend", C.c_double), ("ms_merge", C.c_double), ("ms_total", C.c_double),
        ("profiled_steps", C.c_uint64),
    ]


EXPORTS = [
    "kvd_create", "kvd_destroy", "kvd_strerror", "kvd_last_hip_error", "kvd_abi_version",
    "kvd_bind_summaries", "kvd_bind_host_store", "kvd_bind_slot_pool", "kvd_set_seq_lens",
    "kvd_build_summaries", "kvd_cache_reset", "kvd_cache_warm", "kvd_cache_export", "kvd_cache_import",
    "kvd_bind_centroids", "kvd_build_centroids", "kvd_refresh_clusters", "kvd_append_kv", "kvd_advance", "kvd_score_select", "kvd_cache_resolve", "kvd_sparse_decode_attn", "kvd_step", "kvd_step_trace",
    "kvd_set_profiling", "kvd_step_form", "kvd_set_step_form", "kvd_calibrate_step_form", "kvd_set_wait_limit_us", "kvd_step_timeline", "kvd_get_stats", "kvd_reset_stats",
    "kvd_tier_open", "kvd_tier_close", "kvd_tier_last_errno", "kvd_tier_set_layout", "kvd_tier_write_layer",
    "kvd_tier_patch_page", "kvd_tier_fetch", "kvd_tier_trace", "kvd_tier_pooled", "kvd_tier_drop_pool", "kvd_tier_get_stats",
    "kvd_tier_reset_stats", "kvd_tier_sequential_read_gbps", "kvd_layout_from_clusters", "kvd_bind_tier",
    "kvd_step_tiered", "kvd_step_layers", "kvd_sparse_decode_attn_noalloc",
    "kvd_set_step_shape", "kvd_get_step_shape", "kvd_calibrate_step_shape",
]

_lib = None


def load() -> C.CDLL:
    """Loads libkvd.so once and declares the prototypes."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2605_18071_amd.build`")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i32p, f32p = C.c_void_p, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_float)
    protos = {
        "kvd_create": [C.POINTER(KvdConfig), C.POINTER(vp)],
        "kvd_destroy": [vp],
        "kvd_last_hip_error": [vp],
        "kvd_abi_version": [],
        "kvd_bind_summaries": [vp, vp],
        "kvd_bind_host_store": [vp, vp],
        "kvd_bind_slot_pool": [vp, vp],
        "kvd_set_seq_lens": [vp, i32p],
        "kvd_build_summaries": [vp, i32, vp],
        "kvd_cache_reset": [vp],
        "kvd_cache_warm": [vp, i32, i32p, i32p],
        "kvd_cache_export": [vp, i32, i32p, i32p],
        "kvd_cache_import": [vp, i32, i32p, i32p],
        "kvd_bind_centroids": [vp, vp, vp, vp],
        "kvd_build_centroids": [vp, i32, i32, vp, vp],
        "kvd_refresh_clusters": [vp, i32, vp],
        "kvd_append_kv": [vp, i32, vp, vp, vp],
        "kvd_advance": [vp, vp],
        "kvd_score_select": [vp, i32, vp, vp, vp, vp],
        "kvd_cache_resolve": [vp, i32, i32, vp, vp, vp, vp, vp, i32, vp],
        "kvd_sparse_decode_attn": [vp, i32, vp, vp, vp, vp, vp, vp],
        "kvd_step": [vp, i32, i32, vp, vp, vp, vp],
        "kvd_step_layers": [vp, i32, i32, i32, vp, vp, vp, vp],
        "kvd_step_trace": [vp, vp, vp, vp, vp, vp, vp, vp],
        "kvd_set_profiling": [vp, i32],
        "kvd_step_timeline": [vp, C.POINTER(C.c_int64), i32, i32p],
        "kvd_set_wait_limit_us": [vp, C.c_int64],
        "kvd_step_form": [vp],
        "kvd_set_step_form": [vp, i32],
        "kvd_calibrate_step_form": [vp, i32, i32, vp, i32, i32, vp, vp, i32p, f32p],
        "kvd_get_stats": [vp, C.POINTER(KvdStats)],
        "kvd_reset_stats": [vp],
        "kvd_tier_open": [C.POINTER(KvdTierConfig), C.c_char_p, vp, C.POINTER(vp)],
        "kvd_tier_close": [vp],
        "kvd_tier_last_errno": [vp],
        "kvd_tier_set_layout": [vp, i32, vp],
        "kvd_tier_write_layer": [vp, i32, vp],
        "kvd_tier_patch_page": [vp, i32, i32, i32, C.c_int64, vp, C.c_int64],
        "kvd_tier_fetch": [vp, i32, i32, vp, vp, i32, vp],
        "kvd_tier_trace": [vp, vp, vp, C.c_int64, vp, C.c_int64],
        "kvd_tier_pooled": [vp, vp, C.c_int64, C.POINTER(C.c_int64)],
        "kvd_tier_drop_pool": [vp],
        "kvd_tier_get_stats": [vp, C.POINTER(KvdTierStats)],
        "kvd_tier_reset_stats": [vp],
        "kvd_tier_sequential_read_gbps": [vp, C.POINTER(C.c_double)],
        "kvd_layout_from_clusters": [vp, i32, vp],
        "kvd_bind_tier": [vp, vp],
        "kvd_step_tiered": [vp, i32, i32, vp, vp, vp, vp],
        "kvd_set_step_shape": [vp, i32, i32, i32, i32, i32],
        "kvd_get_step_shape": [vp, i32, i32p],
        "kvd_calibrate_step_shape": [vp, i32, i32, i32, vp, vp, vp, i32, i32p, f32p, f32p],
        "kvd_sparse_decode_attn_noalloc": [vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, C.c_float, i32, vp],
    }
    for name, args in protos.items():
        fn = getattr(lib, name)
        fn.argtypes = args
        fn.restype = C.c_int
    lib.kvd_strerror.argtypes = [C.c_int]
    lib.kvd_strerror.restype = C.c_char_p
    _lib = lib
    return lib


class KvdError(RuntimeError):
    def __init__(self, status: int, where: str, hip: int = 0):
        self.status = status
        msg = load().kvd_strerror(status).decode()
        super().__init__(f"{where}: {msg} (status {status}" + (f", hip error {hip})" if hip else ")"))


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _i32_array(values: Sequence[int]):
    arr = (C.c_int32 * len(values))(*[int(v) for v in values])
    return arr


def _stream_handle(stream: Optional[torch.cuda.Stream]) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def sparse_decode_attn_noalloc(q, slot_pool, sel_pages, sel_slots, seq_len, out, lse=None, *, batch, n_q_heads,
                               n_kv_heads, page_size, topk_pages, capacity_max, kv_dtype, softmax_scale=0.0,
                               attn_splits=0, stream=None):
    """kvd_sparse_decode_attn_noalloc: the attention stage without a context and without any allocation."""
    lib = load()
    dt = {torch.float16: KVD_F16, torch.bfloat16: KVD_BF16}.get(kv_dtype, kv_dtype)
    st = lib.kvd_sparse_decode_attn_noalloc(q.data_ptr(), slot_pool.data_ptr(), sel_pages.data_ptr(), sel_slots.data_ptr(),
                                            seq_len.data_ptr(), out.data_ptr(), _ptr(lse), batch, n_q_heads, n_kv_heads,
                                            page_size, topk_pages, capacity_max, dt, softmax_scale, attn_splits,
                                            _stream_handle(stream))
    if st != OK:
        raise KvdError(st, "kvd_sparse_decode_attn_noalloc")


class Kvd:
    """One kvd_ctx.  Methods mirror the C entry points one to one."""

    def __init__(self, *, n_layers, batch, n_q_heads, n_kv_heads, page_size, max_pages, topk_pages, capacity_max,
                 kv_dtype, head_dim=128, sink_pages=0, recent_pages=0, softmax_scale=0.0, capacity=None,
                 physical_layers=0, micro_batches=0, attn_splits=0, policy=KVD_EVICT_LRU, index_centroids=0,
                 lookahead_pool=0):
        self.lib = load()
        self._cap = None
        cfg = KvdConfig()
        cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads = n_layers, batch, n_q_heads, n_kv_heads
        cfg.head_dim, cfg.page_size, cfg.max_pages, cfg.topk_pages = head_dim, page_size, max_pages, topk_pages
        cfg.sink_pages, cfg.recent_pages = sink_pages, recent_pages
        cfg.kv_dtype = {torch.float16: KVD_F16, torch.bfloat16: KVD_BF16}.get(kv_dtype, kv_dtype)
        cfg.policy = {"lru": KVD_EVICT_LRU, "lookahead": KVD_EVICT_LOOKAHEAD}.get(policy, policy)
        cfg.softmax_scale = softmax_scale
        cfg.capacity_max = capacity_max
        if capacity is not None:
            self._cap = _i32_array(list(capacity))
            cfg.capacity = C.cast(self._cap, C.POINTER(C.c_int32))
        cfg.physical_layers, cfg.micro_batches, cfg.attn_splits = physical_layers, micro_batches, attn_splits
        cfg.index_centroids = index_centroids
        cfg.lookahead_pool = lookahead_pool
        self.cfg = cfg
        self.ctx = C.c_void_p()
        st = self.lib.kvd_create(C.byref(cfg), C.byref(self.ctx))
        if st != OK:
            self.ctx = C.c_void_p()
            raise KvdError(st, "kvd_create")
        self.units = batch * n_kv_heads
        self._keep = []

    def _check(self, st: int, where: str):
        if st != OK:
            raise KvdError(st, where, self.lib.kvd_last_hip_error(self.ctx))

    def close(self):
        if self.ctx:
            self.lib.kvd_destroy(self.ctx)
            self.ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- buffers
    def bind_summaries(self, t: torch.Tensor):
        self._keep.append(t)
        self._check(self.lib.kvd_bind_summaries(self.ctx, t.data_ptr()), "kvd_bind_summaries")

    def bind_host_store(self, t: torch.Tensor):
        self._keep.append(t)
        self._check(self.lib.kvd_bind_host_store(self.ctx, t.data_ptr()), "kvd_bind_host_store")

    def bind_slot_pool(self, t: torch.Tensor):
        self._keep.append(t)
        self._check(self.lib.kvd_bind_slot_pool(self.ctx, t.data_ptr()), "kvd_bind_slot_pool")

    def set_seq_lens(self, seq_lens: Sequence[int]):
        self._check(self.lib.kvd_set_seq_lens(self.ctx, _i32_array(list(seq_lens))), "kvd_set_seq_lens")

    # ---- set-up helpers
    def build_summaries(self, layer: int, stream=None):
        self._check(self.lib.kvd_build_summaries(self.ctx, layer, _stream_handle(stream)), "kvd_build_summaries")

    def cache_reset(self):
        self._check(self.lib.kvd_cache_reset(self.ctx), "kvd_cache_reset")

    def cache_warm(self, layer: int, pages: Sequence[int], counts: Sequence[int]):
        self._check(self.lib.kvd_cache_warm(self.ctx, layer, _i32_array(list(pages)), _i32_array(list(counts))),
                    "kvd_cache_warm")

    def cache_export(self, layer: int):
        n = self.units * self.cfg.capacity_max
        page = torch.empty(n, dtype=torch.int32)
        stamp = torch.empty(n, dtype=torch.int32)
        self._check(self.lib.kvd_cache_export(self.ctx, layer, C.cast(page.data_ptr(), C.POINTER(C.c_int32)),
                                              C.cast(stamp.data_ptr(), C.POINTER(C.c_int32))), "kvd_cache_export")
        shape = (self.units, self.cfg.capacity_max)
        return page.view(shape), stamp.view(shape)

    def cache_import(self, layer: int, slot_page: torch.Tensor, slot_stamp: torch.Tensor):
        sp = slot_page.to(torch.int32).contiguous()
        ss = slot_stamp.to(torch.int32).contiguous()
        self._check(self.lib.kvd_cache_import(self.ctx, layer, C.cast(sp.data_ptr(), C.POINTER(C.c_int32)),
                                              C.cast(ss.data_ptr(), C.POINTER(C.c_int32))), "kvd_cache_import")

    # ---- hierarchical index
    def bind_centroids(self, centroids: torch.Tensor, cluster_start: torch.Tensor, cluster_pages: torch.Tensor):
        self._keep += [centroids, cluster_start, cluster_pages]
        self._check(self.lib.kvd_bind_centroids(self.ctx, centroids.data_ptr(), cluster_start.data_ptr(),
                                                cluster_pages.data_ptr()), "kvd_bind_centroids")

    def build_centroids(self, layer: int, iterations: int, assign_trace: Optional[torch.Tensor] = None, stream=None):
        self._check(self.lib.kvd_build_centroids(self.ctx, layer, iterations, _ptr(assign_trace), _stream_handle(stream)),
                    "kvd_build_centroids")

    def refresh_clusters(self, layer: int, stream=None):
        self._check(self.lib.kvd_refresh_clusters(self.ctx, layer, _stream_handle(stream)), "kvd_refresh_clusters")

    # ---- growth of the store
    def append_kv(self, layer: int, k_new: torch.Tensor, v_new: torch.Tensor, stream=None):
        self._check(self.lib.kvd_append_kv(self.ctx, layer, k_new.data_ptr(), v_new.data_ptr(), _stream_handle(stream)),
                    "kvd_append_kv")

    def advance(self, stream=None):
        self._check(self.lib.kvd_advance(self.ctx, _stream_handle(stream)), "kvd_advance")

    # ---- hot path
    def score_select(self, layer: int, q: torch.Tensor, sel_pages: torch.Tensor, scores: Optional[torch.Tensor] = None,
                     stream=None):
        self._check(self.lib.kvd_score_select(self.ctx, layer, q.data_ptr(), sel_pages.data_ptr(), _ptr(scores),
                                              _stream_handle(stream)), "kvd_score_select")

    def cache_resolve(self, layer: int, step: int, sel_pages, sel_slots, hit_mask=None, evicted=None, counts=None,
                      do_gather: bool = True, stream=None):
        self._check(self.lib.kvd_cache_resolve(self.ctx, layer, step, sel_pages.data_ptr(), sel_slots.data_ptr(),
                                               _ptr(hit_mask), _ptr(evicted), _ptr(counts), 1 if do_gather else 0,
                                               _stream_handle(stream)), "kvd_cache_resolve")

    def sparse_decode_attn(self, layer: int, q, sel_pages, sel_slots, out, lse=None, stream=None):
        self._check(self.lib.kvd_sparse_decode_attn(self.ctx, layer, q.data_ptr(), sel_pages.data_ptr(),
                                                    sel_slots.data_ptr(), out.data_ptr(), _ptr(lse),
                                                    _stream_handle(stream)), "kvd_sparse_decode_attn")

    def step(self, layer: int, step: int, q, out, lse=None, stream=None):
        self._check(self.lib.kvd_step(self.ctx, layer, step, q.data_ptr(), out.data_ptr(), _ptr(lse),
                                      _stream_handle(stream)), "kvd_step")

    def step_layers(self, layer0: int, n_layers: int, step: int, q_layers, out_layers, lse_layers=None, stream=None):
        self._check(self.lib.kvd_step_layers(self.ctx, layer0, n_layers, step, q_layers.data_ptr(), out_layers.data_ptr(),
                                             _ptr(lse_layers), _stream_handle(stream)), "kvd_step_layers")

    def step_trace(self, sel_pages=None, sel_slots=None, hit_mask=None, evicted=None, counts=None, scores=None,
                   stream=None):
        self._check(self.lib.kvd_step_trace(self.ctx, _ptr(sel_pages), _ptr(sel_slots), _ptr(hit_mask), _ptr(evicted),
                                            _ptr(counts), _ptr(scores), _stream_handle(stream)), "kvd_step_trace")

    # ---- third tier
    def layout_from_clusters(self, layer: int) -> torch.Tensor:
        pos = torch.empty((self.units, self.cfg.max_pages), dtype=torch.int32)
        self._check(self.lib.kvd_layout_from_clusters(self.ctx, layer, pos.data_ptr()), "kvd_layout_from_clusters")
        return pos

    def bind_tier(self, tier: Optional["KvdTier"]):
        self._keep.append(tier)
        self._check(self.lib.kvd_bind_tier(self.ctx, tier.handle if tier is not None else None), "kvd_bind_tier")

    def step_tiered(self, layer: int, step: int, q, out, lse=None, stream=None):
        self._check(self.lib.kvd_step_tiered(self.ctx, layer, step, q.data_ptr(), out.data_ptr(), _ptr(lse),
                                             _stream_handle(stream)), "kvd_step_tiered")

    # ---- counters
    def set_profiling(self, mode):
        self._check(self.lib.kvd_set_profiling(self.ctx, int(mode)), "kvd_set_profiling")

    def step_form(self) -> int:
        return int(self.lib.kvd_step_form(self.ctx))

    def set_step_form(self, form: int):
        self._check(self.lib.kvd_set_step_form(self.ctx, int(form)), "kvd_set_step_form")

    def calibrate_step_form(self, layer: int, first_step: int, q_steps: torch.Tensor, steps_per_form: int,
                            out: torch.Tensor, stream=None):
        """Returns (chosen form, {form: ms per step}) — see kvd_calibrate_step_form."""
        chosen = C.c_int32()
        ms = (C.c_float * 4)()
        self._check(self.lib.kvd_calibrate_step_form(self.ctx, layer, first_step, q_steps.data_ptr(), q_steps.shape[0],
                                                     steps_per_form, out.data_ptr(), _stream_handle(stream),
                                                     C.byref(chosen), ms), "kvd_calibrate_step_form")
        return chosen.value, {f: ms[i] for i, f in enumerate((1, 2, 4, -1)) if ms[i] >= 0}

    def set_step_shape(self, passes: int = 0, scoring_workgroups: int = 0, attn_splits: int = 0, groups: int = 0,
                       multi_layer: bool = False):
        self._check(self.lib.kvd_set_step_shape(self.ctx, 1 if multi_layer else 0, passes, scoring_workgroups, attn_splits,
                                                groups), "kvd_set_step_shape")

    def step_shape(self, multi_layer: bool = False):
        """(passes, scoring workgroups, attention splits, groups) a launch of the one-launch step would take."""
        shape = (C.c_int32 * 4)()
        self._check(self.lib.kvd_get_step_shape(self.ctx, 1 if multi_layer else 0, shape), "kvd_get_step_shape")
        return tuple(shape)

    def calibrate_step_shape(self, layer: int, step: int, q: torch.Tensor, out: torch.Tensor, launches_per_shape: int = 16,
                             n_layers: int = 1, stream=None):
        """Returns ((passes, scoring workgroups, splits, groups), us per layer-step of it, us per layer-step of the rule's shape)."""
        shape = (C.c_int32 * 4)()
        us, us_rule = C.c_float(), C.c_float()
        self._check(self.lib.kvd_calibrate_step_shape(self.ctx, layer, n_layers, step, q.data_ptr(), out.data_ptr(),
                                                      _stream_handle(stream), launches_per_shape, shape, C.byref(us),
                                                      C.byref(us_rule)), "kvd_calibrate_step_shape")
        return tuple(shape), us.value, us_rule.value

    def set_wait_limit_us(self, microseconds: int):
        self._check(self.lib.kvd_set_wait_limit_us(self.ctx, int(microseconds)), "kvd_set_wait_limit_us")

    def step_timeline(self) -> torch.Tensor:
        """[workgroups, 5] int64 records of the last single-launch step run under profiling mode 2:
        ticks (100 MHz) at start / inputs ready / work done / exit, and the tag (see kvd.h)."""
        n = C.c_int32()
        probe = (C.c_int64 * 5)()
        self._check(self.lib.kvd_step_timeline(self.ctx, probe, 0, C.byref(n)), "kvd_step_timeline")
        buf = (C.c_int64 * (5 * n.value))()
        self._check(self.lib.kvd_step_timeline(self.ctx, buf, n.value, C.byref(n)), "kvd_step_timeline")
        return torch.tensor(list(buf), dtype=torch.int64).reshape(-1, 5)

    def stats(self) -> KvdStats:
        st = KvdStats()
        self._check(self.lib.kvd_get_stats(self.ctx, C.byref(st)), "kvd_get_stats")
        return st

    def reset_stats(self):
        self._check(self.lib.kvd_reset_stats(self.ctx), "kvd_reset_stats")


class KvdTier:
    """One kvd_tier (host code only; needs no GPU).  `pool` is a uint8 CPU tensor of pool_extents *
    extent_pages * page_bytes bytes, 4096-byte aligned; pinned if a GPU is to read it."""

    def __init__(self, path: str, pool: torch.Tensor, *, n_layers, n_units, max_pages, extent_pages, page_bytes,
                 pool_extents, queue_depth=8, max_run_extents=8, direct_io=False):
        self.lib = load()
        cfg = KvdTierConfig()
        cfg.n_layers, cfg.n_units, cfg.max_pages, cfg.extent_pages = n_layers, n_units, max_pages, extent_pages
        cfg.page_bytes, cfg.pool_extents = page_bytes, pool_extents
        cfg.queue_depth, cfg.max_run_extents, cfg.direct_io = queue_depth, max_run_extents, 1 if direct_io else 0
        if pool.device.type != "cpu" or pool.numel() * pool.element_size() < pool_extents * extent_pages * page_bytes:
            raise ValueError("the pool must be CPU memory of pool_extents * extent_pages * page_bytes bytes")
        self.cfg, self.pool, self.path = cfg, pool, path
        self.handle = C.c_void_p()
        st = self.lib.kvd_tier_open(C.byref(cfg), path.encode(), pool.data_ptr(), C.byref(self.handle))
        if st != OK:
            self.handle = C.c_void_p()
            raise KvdError(st, "kvd_tier_open")

    def _check(self, st: int, where: str):
        if st != OK:
            raise KvdError(st, f"{where} (errno {self.lib.kvd_tier_last_errno(self.handle)})")

    def close(self):
        if self.handle:
            self.lib.kvd_tier_close(self.handle)
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_layout(self, layer: int, position: torch.Tensor):
        pos = position.to(torch.int32).contiguous()
        self._check(self.lib.kvd_tier_set_layout(self.handle, layer, pos.data_ptr()), "kvd_tier_set_layout")

    def write_layer(self, layer: int, host_pages: torch.Tensor):
        self._check(self.lib.kvd_tier_write_layer(self.handle, layer, host_pages.data_ptr()), "kvd_tier_write_layer")

    def patch_page(self, layer: int, unit: int, page: int, offset_in_page: int, src: torch.Tensor):
        src = src.contiguous()
        self._check(self.lib.kvd_tier_patch_page(self.handle, layer, unit, page, offset_in_page, src.data_ptr(),
                                                 src.numel() * src.element_size()), "kvd_tier_patch_page")

    def fetch(self, layer: int, step: int, miss_list: torch.Tensor, miss_count: torch.Tensor) -> torch.Tensor:
        """miss_list [U, k, 2] int32, miss_count [U] int32 (CPU) -> byte offsets into the pool, [U, k] int64."""
        k = miss_list.shape[1]
        off = torch.empty((self.cfg.n_units, k), dtype=torch.int64)
        self._check(self.lib.kvd_tier_fetch(self.handle, layer, step, miss_list.data_ptr(), miss_count.data_ptr(), k,
                                            off.data_ptr()), "kvd_tier_fetch")
        return off

    def trace(self):
        """dict(needed, hits, reads, evictions, read_calls, runs [(first, count)], evicted [extents]) of the last fetch."""
        counts = torch.zeros(5, dtype=torch.int64)
        self._check(self.lib.kvd_tier_trace(self.handle, counts.data_ptr(), None, 0, None, 0), "kvd_tier_trace")
        runs = torch.zeros((int(counts[4]), 2), dtype=torch.int64)
        evicted = torch.zeros(int(counts[3]), dtype=torch.int64)
        self._check(self.lib.kvd_tier_trace(self.handle, counts.data_ptr(), runs.data_ptr(), runs.shape[0],
                                            evicted.data_ptr(), evicted.shape[0]), "kvd_tier_trace")
        names = ("needed", "hits", "reads", "evictions", "read_calls")
        out = {n: int(counts[i]) for i, n in enumerate(names)}
        out["runs"] = [(int(a), int(b)) for a, b in runs.tolist()]
        out["evicted"] = evicted.tolist()
        return out

    def pooled(self):
        n = C.c_int64()
        self._check(self.lib.kvd_tier_pooled(self.handle, None, 0, C.byref(n)), "kvd_tier_pooled")
        ext = torch.zeros(n.value, dtype=torch.int64)
        self._check(self.lib.kvd_tier_pooled(self.handle, ext.data_ptr(), n.value, C.byref(n)), "kvd_tier_pooled")
        return ext.tolist()

    def drop_pool(self):
        self._check(self.lib.kvd_tier_drop_pool(self.handle), "kvd_tier_drop_pool")

    def stats(self) -> KvdTierStats:
        st = KvdTierStats()
        self._check(self.lib.kvd_tier_get_stats(self.handle, C.byref(st)), "kvd_tier_get_stats")
        return st

    def reset_stats(self):
        self._check(self.lib.kvd_tier_reset_stats(self.handle), "kvd_tier_reset_stats")

    def sequential_read_gbps(self) -> float:
        g = C.c_double()
        self._check(self.lib.kvd_tier_sequential_read_gbps(self.handle, C.byref(g)), "kvd_tier_sequential_read_gbps")
        return g.value
