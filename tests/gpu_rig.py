"""GPU test rig: builds a workload on the device, a kvd context bound to it, and
per-unit oracle mirrors, and compares the two after every step.

The HIP path is driven only through the C-ABI binding; the oracle only through
oracle/kvd_oracle.py; the inputs come from paper_2605_18071_amd/workloads.py.
"""
from __future__ import annotations

import math
from typing import Iterable, List, Optional, Sequence, Tuple

import numpy as np
import torch

from oracle import kvd_oracle as orc
from paper_2605_18071_amd import kvd as K
from paper_2605_18071_amd import workloads as W
from tests import helpers as H

DEV = "cuda"


class Rig:
    def __init__(self, w: W.Workload, *, seq_lens: Optional[Sequence[int]] = None, capacity: Optional[Sequence[int]] = None,
                 micro_batches: int = 0, attn_splits: int = 0, build_index: bool = True):
        self.w = w
        self.q0 = W.initial_queries(w, DEV)
        self.store = W.make_kv_store(w, self.q0, DEV)                      # pinned host
        L, B, Hkv, NP, P, D = w.n_layers, w.batch, w.n_kv_heads, w.n_pages, w.page, w.head_dim
        self.summaries = torch.zeros((L, B, Hkv, NP, D), dtype=w.torch_dtype, device=DEV)
        self.pool = torch.zeros((L, B, Hkv, w.capacity, 2, P, D), dtype=w.torch_dtype, device=DEV)
        self.kvd = K.Kvd(n_layers=L, batch=B, n_q_heads=w.n_q_heads, n_kv_heads=Hkv, page_size=P, max_pages=NP,
                         topk_pages=w.topk_pages, capacity_max=w.capacity, kv_dtype=w.torch_dtype,
                         sink_pages=w.sink_pages, recent_pages=w.recent_pages, capacity=capacity,
                         physical_layers=w.physical_layers, micro_batches=micro_batches, attn_splits=attn_splits,
                         policy=w.policy, index_centroids=w.index_centroids, lookahead_pool=w.lookahead_pool)
        self.kvd.bind_summaries(self.summaries)
        self.kvd.bind_host_store(self.store)
        self.kvd.bind_slot_pool(self.pool)
        self.seq_lens = list(seq_lens) if seq_lens is not None else [w.ctx] * B
        self.kvd.set_seq_lens(self.seq_lens)
        self.capacity = capacity
        self.hier = w.index_centroids > 0
        if self.hier:
            Nc = w.index_centroids
            self.centroids = torch.zeros((L, B, Hkv, Nc, D), dtype=w.torch_dtype, device=DEV)
            self.cluster_start = torch.zeros((L, B * Hkv, Nc + 1), dtype=torch.int32, device=DEV)
            self.cluster_pages = torch.zeros((L, B * Hkv, NP), dtype=torch.int32, device=DEV)
            self.assign_trace = torch.zeros((L, w.index_iterations, B * Hkv, NP), dtype=torch.int32, device=DEV)
            self.kvd.bind_centroids(self.centroids, self.cluster_start, self.cluster_pages)
        if build_index:
            for l in range(L):
                self.kvd.build_summaries(l)
            torch.cuda.synchronize()
            if self.hier:
                for l in range(L):
                    self.kvd.build_centroids(l, w.index_iterations, self.assign_trace[l])
                torch.cuda.synchronize()
                self.n_assign_trace = self.assign_trace.cpu().numpy()
        self.warm()
        U, k = w.units, w.topk_pages
        i32 = dict(dtype=torch.int32, device=DEV)
        self.sel_pages = torch.empty((U, k), **i32)
        self.sel_slots = torch.empty((U, k), **i32)
        self.hit_mask = torch.empty((U, k), **i32)
        self.evicted = torch.empty((U, k), **i32)
        self.counts = torch.empty((U, 3), **i32)
        self.scores = torch.empty((U, NP), dtype=torch.float32, device=DEV)
        self.out = torch.empty((B, w.n_q_heads, D), dtype=torch.float32, device=DEV)
        self.lse = torch.empty((B, w.n_q_heads), dtype=torch.float32, device=DEV)

    def warm_list(self, b: int) -> List[int]:
        pages = W.warm_pages(self.w)
        if pages is None:
            return []
        if self.w.warm == "recent":
            n_valid = -(-self.seq_lens[b] // self.w.page)
            return list(range(n_valid - self.w.recent_pages, n_valid))
        return pages.tolist()

    def warm(self):
        w = self.w
        self.kvd.cache_reset()
        if w.warm == "cold":
            return
        for l in range(w.n_layers):
            pages, counts = [], []
            for u in range(w.units):
                lst = self.warm_list(u // w.n_kv_heads)
                pages.extend(lst)
                counts.append(len(lst))
            self.kvd.cache_warm(l, pages, counts)

    def cap(self, layer: int, u: int) -> int:
        if self.capacity is None:
            return self.w.capacity
        return int(self.capacity[layer * self.w.units + u])

    def attach_tier(self, path: str, *, extent_pages: int, pool_extents: int, max_run_extents: int = 8,
                    queue_depth: int = 4, direct_io: bool = False, semantic: bool = False):
        """Puts the third tier behind the window: the backing file is written from the host store,
        kvd_step_tiered is used from now on, and the context's host store is replaced by one full
        of NaNs, so that a page taken from there instead of the file cannot go unnoticed."""
        w = self.w
        pool = torch.zeros(pool_extents * extent_pages * w.page_bytes, dtype=torch.uint8).pin_memory()
        self.tier = K.KvdTier(path, pool, n_layers=w.phys_layers, n_units=w.units, max_pages=w.n_pages,
                              extent_pages=extent_pages, page_bytes=w.page_bytes, pool_extents=pool_extents,
                              queue_depth=queue_depth, max_run_extents=max_run_extents, direct_io=direct_io)
        self.tier_pool = pool
        self.positions = []
        for lp in range(w.phys_layers):
            if semantic:
                pos = self.kvd.layout_from_clusters(lp)
                self.tier.set_layout(lp, pos)
            else:
                pos = torch.arange(w.n_pages, dtype=torch.int32).repeat(w.units, 1)
            self.positions.append(pos.numpy())
            self.tier.write_layer(lp, self.store[lp])
        self.kvd.bind_tier(self.tier)
        self.poison = torch.full(self.store.shape, float("nan"), dtype=self.store.dtype).pin_memory()
        self.kvd.bind_host_store(self.poison)
        self.tiered = True

    def step(self, layer: int, t: int, q_layer: torch.Tensor):
        """One fused layer-step through kvd_step (kvd_step_tiered once a tier is attached); trace
        copied into the rig's buffers."""
        if getattr(self, "tiered", False):
            try:
                self.kvd.step_tiered(layer, t, q_layer, self.out, self.lse)
            except K.KvdError as e:
                raise AssertionError(f"{e}; tier errno {self.tier.lib.kvd_tier_last_errno(self.tier.handle)}, "
                                     f"direct I/O mode {self.tier.stats().direct_io}") from e
        else:
            self.kvd.step(layer, t, q_layer, self.out, self.lse)
        self.kvd.step_trace(self.sel_pages, self.sel_slots, self.hit_mask, self.evicted, self.counts, self.scores)
        torch.cuda.synchronize()
        self.n_sel_pages = self.sel_pages.cpu().numpy()
        self.n_sel_slots = self.sel_slots.cpu().numpy()
        self.n_hit_mask = self.hit_mask.cpu().numpy()
        self.n_evicted = self.evicted.cpu().numpy()
        self.n_counts = self.counts.cpu().numpy()
        self.n_scores = self.scores.cpu().numpy()
        if self.hier:                                              # the library packs the cluster scores as [U][Nc]
            Nc = self.w.index_centroids
            self.n_scores = self.n_scores.reshape(-1)[: self.w.units * Nc].reshape(self.w.units, Nc)
        self.n_out = self.out.cpu().numpy()
        self.n_lse = self.lse.cpu().numpy()

    def close(self):
        self.kvd.close()
        if getattr(self, "tiered", False):
            self.tier.close()


class StoreRows:
    """The K (which = 0) or V (1) rows of one unit of the host store, [tokens, D], widened to
    float64 only where they are read: rows[token indices] -> float64 [n, D].  Lets the oracle
    follow every unit of a full-size configuration without a float64 copy of the whole store."""

    def __init__(self, unit_store: torch.Tensor, which: int):
        self.kv, self.which = unit_store, which                             # [NP, 2, P, D] in the KV dtype
        self.page = unit_store.shape[2]
        self.shape = (unit_store.shape[0] * self.page, unit_store.shape[3])

    def __getitem__(self, tokens) -> np.ndarray:
        t = torch.as_tensor(np.asarray(tokens, dtype=np.int64))
        return H.f64(self.kv[t // self.page, self.which, t % self.page])

    def all(self) -> np.ndarray:
        return H.f64(self.kv[:, self.which]).reshape(self.shape)


class OracleUnit:
    """The oracle's view of one (layer, b, h): its slice of the host store, its own
    summaries, and its LRU window carried across steps."""

    def __init__(self, rig: Rig, layer: int, b: int, h: int, summaries: Optional[np.ndarray] = None, lazy: bool = False):
        """lazy: keep no float64 copy of the unit's K and V (full-size configurations: 256 MiB per
        unit and more); rows are widened where the oracle reads them."""
        w = rig.w
        self.rig, self.layer, self.b, self.h = rig, layer, b, h
        self.u = b * w.n_kv_heads + h
        lp = layer % w.phys_layers
        kv = rig.store[lp, b, h]                                            # [NP, 2, P, D]
        self.seq_len = rig.seq_lens[b]
        self.code = H.dtype_code(w.torch_dtype)
        if lazy:
            self.keys, self.values = StoreRows(kv, 0), StoreRows(kv, 1)
            self.summ = orc.page_summaries(self.keys.all(), w.page, self.seq_len, self.code)
        else:
            self.keys = H.f64(kv[:, 0]).reshape(-1, w.head_dim)
            self.values = H.f64(kv[:, 1]).reshape(-1, w.head_dim)
            self.summ = orc.page_summaries(self.keys, w.page, self.seq_len, self.code)
        if summaries is not None:                                  # a test planted its own index
            self.summ = summaries[: self.summ.shape[0]]
        if w.policy == "lookahead":
            self.window = orc.LookaheadWindow(rig.cap(layer, self.u), pool=w.lookahead_pool)
        else:
            self.window = orc.LruWindow(rig.cap(layer, self.u))
        self.window.warm(rig.warm_list(b), stamp=-1)
        self.scale = 1.0 / math.sqrt(w.head_dim)
        self.centroids = self.members = None
        self.kmeans_divergences = 0
        if rig.hier:
            self.build_hier_index()

    def build_hier_index(self):
        """The oracle's k-means, round by round beside the GPU's recorded assignments: a GPU
        assignment that differs is accepted only if its centroid is as near as the nearest one to
        within rounding of the fp64 distance, and the oracle then continues from it.  Centroids
        and cluster lists must then agree exactly."""
        rig, w = self.rig, self.rig.w
        Nc = w.index_centroids
        n = self.summ.shape[0]
        cent = orc.kmeans_init(self.summ, Nc)
        forced = []
        for it in range(w.index_iterations):
            own = orc.kmeans_assign(self.summ, cent)
            gpu = rig.n_assign_trace[self.layer, it, self.u, :n].astype(np.int32)
            if not np.array_equal(own, gpu):
                d = orc.kmeans_distances(self.summ, cent)
                rows = np.nonzero(own != gpu)[0]
                assert np.all(gpu[rows] >= 0) and np.all(gpu[rows] < Nc)
                dmin = d[rows].min(axis=1)
                assert np.all(d[rows, gpu[rows]] <= dmin + 1e-9 * (1.0 + np.abs(dmin))), \
                    f"k-means assignment differs outside rounding at unit {self.u} round {it}"
                self.kmeans_divergences += len(rows)
            forced.append(gpu)
            cent = orc.kmeans_update(self.summ, gpu, cent)
        self.centroids, assign, _ = orc.kmeans_centroids(self.summ, Nc, w.index_iterations, self.code, forced_assign=forced)
        self.members = orc.cluster_members(assign, Nc)
        got = rig.centroids[self.layer, self.b, self.h].cpu()
        assert np.array_equal(H.bits(got), orc.f64_to_bits(self.centroids, self.code)), f"centroids differ at unit {self.u}"
        start = rig.cluster_start[self.layer, self.u].cpu().numpy()
        pages = rig.cluster_pages[self.layer, self.u].cpu().numpy()
        assert start[0] == 0 and start[-1] == n and np.all(np.diff(start) >= 0)
        for c in range(Nc):
            assert np.array_equal(pages[start[c]:start[c + 1]], self.members[c]), f"cluster {c} of unit {self.u}"

    def step(self, t: int, q_layer: torch.Tensor, forced_sel=None, forced_evicted=None):
        w = self.rig.w
        qg = H.f64(q_layer[self.b, self.h * w.group:(self.h + 1) * w.group])
        return orc.decode_unit_step(qg, self.summ, self.keys, self.values, self.window, t, k=w.topk_pages,
                                    page_size=w.page, seq_len=self.seq_len, scale=self.scale,
                                    sink_pages=w.sink_pages, recent_pages=w.recent_pages, forced_sel=forced_sel,
                                    forced_evicted=forced_evicted, centroids=self.centroids, members=self.members)


class StepReport:
    def __init__(self):
        self.tie_divergences = 0
        self.victim_tie_divergences = 0
        self.max_attn_err = 0.0
        self.max_lse_err = 0.0
        self.max_score_err = 0.0
        self.hits = 0
        self.misses = 0
        self.unit_steps = 0


def score_bound(ou: OracleUnit, q_layer: torch.Tensor) -> np.ndarray:
    """fp32 forward-error bound of the kernel's score per page:
    (8 sequential fma + 4 tree adds + pooled-query rounding) ~ 20 eps * scale * sum_d |qbar_d s_pd|."""
    w = ou.rig.w
    qbar = orc.pooled_query(H.f64(q_layer[ou.b, ou.h * w.group:(ou.h + 1) * w.group]))
    index = ou.centroids if ou.centroids is not None else ou.summ
    return 20.0 * 2.0 ** -24 * ou.scale * (np.abs(index) @ np.abs(qbar)) + 1e-12


def compare_unit(rig: Rig, ou: OracleUnit, t: int, q_layer: torch.Tensor, rep: StepReport, check_scores: bool = True):
    """Compare what kvd_step left in the rig's buffers for unit `ou` with the oracle's
    step.  A GPU selection that differs from the oracle's only inside the tie band is
    adopted by the oracle for this step (and counted), so that traces stay comparable."""
    w = rig.w
    u, k = ou.u, w.topk_pages
    g_sel = rig.n_sel_pages[u]
    hier = ou.centroids is not None
    # the oracle's own step first; where the GPU's selection differs from it inside the tie band
    # the step is taken again from the same window with the GPU's selection
    before = dict(ou.window.stamp)
    want = ou.step(t, q_layer)
    o_scores, o_sel = want["scores"], want["sel"]
    n_valid = o_scores.shape[0]
    if check_scores:
        g_scores = rig.n_scores[u, :n_valid].astype(np.float64)
        err = np.abs(g_scores - o_scores)
        bound = score_bound(ou, q_layer)
        assert np.all(err <= bound), f"score error {err.max():.3e} above fp32 bound at unit {u} step {t}"
        rep.max_score_err = max(rep.max_score_err, float(err.max()))
    forced = None
    if not np.array_equal(g_sel, o_sel):
        if hier:
            ok, msg = H.hier_selection_is_valid(o_scores, ou.members, g_sel, k, ou.summ.shape[0], w.sink_pages, w.recent_pages)
        else:
            ok, msg = H.selection_is_valid(o_scores, g_sel, k, w.sink_pages, w.recent_pages)
        assert ok, f"selection differs outside the tie band at unit {u} step {t}: {msg}"
        rep.tie_divergences += 1
        forced = g_sel
        ou.window.stamp = dict(before)
        want = ou.step(t, q_layer, forced_sel=forced)

    # cache trace: hit / miss / evicted sets, bit-exact
    hm = rig.n_hit_mask[u]
    valid = g_sel >= 0
    g_hits = sorted(g_sel[valid & (hm == 1)].tolist())
    g_miss = sorted(g_sel[valid & (hm == 0)].tolist())
    ev = rig.n_evicted[u]
    g_ev = sorted(ev[ev >= 0].tolist())
    if w.policy == "lookahead" and g_ev != want["evicted"]:
        # victims are chosen by score: a different set is accepted only inside the tie band, and
        # the oracle then continues from the GPU's choice
        used = set(int(p) for p in want["used"] if p >= 0)
        cands = [p for p in before if p not in used]
        if w.lookahead_pool > 0:
            ok, msg = H.pooled_eviction_is_valid(want["evict_scores"], before, cands, g_ev, len(want["evicted"]), w.lookahead_pool)
        else:
            ok, msg = H.eviction_is_valid(want["evict_scores"], cands, g_ev, len(want["evicted"]))
        assert ok, f"victims differ outside the tie band at unit {u} step {t}: {msg}"
        rep.victim_tie_divergences += 1
        ou.window.stamp = before
        want = ou.step(t, q_layer, forced_sel=forced, forced_evicted=g_ev)
    assert g_hits == want["hits"], f"hit set differs at unit {u} step {t}"
    assert g_miss == want["misses"], f"miss set differs at unit {u} step {t}"
    assert g_ev == want["evicted"], f"evicted set differs at unit {u} step {t}"
    cnt = rig.n_counts[u].tolist()
    assert cnt == [len(g_hits), len(g_miss), len(g_ev)], f"counts differ at unit {u} step {t}: {cnt}"
    slots = rig.n_sel_slots[u]
    assert np.all(slots[valid] >= 0) and np.all(slots[~valid] == -1)
    assert len(set(slots[valid].tolist())) == int(valid.sum()), "two selected pages share a slot"
    assert slots[valid].max(initial=0) < rig.cap(ou.layer, u)

    # attention output
    G = w.group
    g_out = rig.n_out[ou.b, ou.h * G:(ou.h + 1) * G]
    g_lse = rig.n_lse[ou.b, ou.h * G:(ou.h + 1) * G]
    e = H.attn_rel_err(g_out, want["out"])
    assert e <= H.ATTN_RTOL, f"attention rel err {e:.3e} at unit {u} step {t}"
    le = float(np.abs(g_lse - want["lse"]).max())
    # lse is computed and returned in fp32 (q.k accumulated over 128 products, the scaling, the log):
    # a few fp32 steps of its own size, which beyond |lse| ~ 500 is more than 1e-3
    lse_tol = max(1e-3, 16.0 * float(np.spacing(np.abs(want["lse"]).astype(np.float32)).max()))
    assert le <= lse_tol, f"lse abs err {le:.3e} at unit {u} step {t}"
    rep.max_attn_err = max(rep.max_attn_err, e)
    rep.max_lse_err = max(rep.max_lse_err, le)
    rep.hits += len(g_hits)
    rep.misses += len(g_miss)
    rep.unit_steps += 1
    return want


def check_directory(rig: Rig, layer: int, units: Iterable[OracleUnit], check_data: bool = True):
    """Directory invariants and contents after a step: every unit's resident set and
    stamps equal the oracle's, pages are unique, slots stay below the capacity, and
    (check_data) each occupied slot holds the bytes of its page in the host store."""
    w = rig.w
    slot_page, slot_stamp = rig.kvd.cache_export(layer)
    for ou in units:
        sp = slot_page[ou.u].numpy()
        st = slot_stamp[ou.u].numpy()
        occ = sp >= 0
        assert not occ[rig.cap(layer, ou.u):].any()
        pages = sp[occ].tolist()
        assert len(pages) == len(set(pages))
        got = {int(p): int(s) for p, s in zip(sp[occ], st[occ])}
        assert got == ou.window.stamp, f"resident set / stamps differ at unit {ou.u}"
        if check_data:
            lp = layer % w.phys_layers
            for s in np.nonzero(occ)[0][:64]:
                a = rig.pool[layer, ou.b, ou.h, int(s)].cpu().view(torch.int16).reshape(-1)
                b = H.slot_image(rig.store[lp, ou.b, ou.h, int(sp[s])])
                assert torch.equal(a, b), f"slot {s} of unit {ou.u} != page {sp[s]}"


def run_steps(rig: Rig, units: List[OracleUnit], steps: int, *, layers: Optional[Sequence[int]] = None,
              check_dir_every: int = 0, progress: str = "") -> StepReport:
    """Drives `steps` decode steps over the given layers and compares every oracle unit
    after each layer-step."""
    w = rig.w
    rep = StepReport()
    layers = list(range(w.n_layers)) if layers is None else list(layers)
    by_layer = {l: [ou for ou in units if ou.layer == l] for l in layers}
    for t, q in enumerate(W.query_stream(w, rig.q0, steps, DEV)):
        for l in layers:
            rig.step(l, t, q[l])
            for ou in by_layer[l]:
                compare_unit(rig, ou, t, q[l], rep)
            if check_dir_every and (t % check_dir_every == 0 or t == steps - 1):
                check_directory(rig, l, by_layer[l])
        if progress:
            print(f"[{progress}] step {t} ok: units {rep.unit_steps} ties {rep.tie_divergences}+{rep.victim_tie_divergences} "
                  f"attn_err {rep.max_attn_err:.2e} hit_rate {rep.hits / max(1, rep.hits + rep.misses):.3f}", flush=True)
    return rep
