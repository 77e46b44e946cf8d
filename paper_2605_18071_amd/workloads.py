"""Seeded synthetic workloads shaped like the paper's long-context decode runs.

This module only *draws inputs*: the paged K/V store, the initial queries and
the drifting query stream.  It contains none of the method's arithmetic (no
summaries, scores, selection, cache logic or attention), so both the HIP path
and the CPU oracle can be fed from it without sharing any computation.

The paper evaluates on public long-context suites with real checkpoints
(Experiment section: 8B/14B-class GQA models, contexts of 60k-360k tokens,
budgets of 2048 tokens or 1.56 % / 6.25 %).  Neither the suites nor the weights
are used here; the five workloads below stand in for them with the same tensor
shapes (32 q / 8 kv heads or 28 q / 4 kv heads, head_dim 128, fp16/bf16) and a
planted importance structure:

  * K, V ~ N(0,1) i.i.d.;  q0 ~ N(0,1) per (layer, sequence, query head);
  * the "query direction" of a unit is u = normalize(mean_g q0[group]);
  * planted heavy pages: every key of the page gets  K += shift * u;
  * Zipf importance: a random permutation ranks the pages of a unit and the page
    of rank r gets  K += amp * r^(-alpha) * u;
  * drift: q_t = rho * q_{t-1} + (1 - rho) * N(0,1)  (fp32 state, rounded to the
    KV dtype when handed out).

Host-store layout: [physical_layers][B][Hkv][NP][2][P][D]  (K page then V page,
contiguous), pinned when a GPU is present.  `physical_layers` < `n_layers`
aliases logical layer l onto store layer l % physical_layers so the larger
workloads fit host memory; every logical layer still has its own queries,
cache directory and slot pool.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Iterator, Optional

import torch


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    n_layers: int
    batch: int
    ctx: int                 # tokens per sequence
    page: int                # tokens per page
    n_q_heads: int
    n_kv_heads: int
    dtype: str               # "f16" | "bf16"
    topk_pages: int          # token budget / page
    capacity: int            # cache pages per (layer, sequence, kv head)
    steps: int
    rho: float = 0.9
    head_dim: int = 128
    importance: str = "planted"   # "planted" | "zipf" | "none"
    heavy_count: int = 0          # planted: pages per unit
    heavy_shift: float = 3.0
    zipf_alpha: float = 1.1
    zipf_amp: float = 6.0
    sink_pages: int = 0
    recent_pages: int = 0
    physical_layers: int = 0      # 0 -> n_layers
    warm: str = "cold"            # "cold" | "full" | "recent"
    policy: str = "lru"           # cache replacement: "lru" | "lookahead"
    lookahead_pool: int = 0       # lookahead: look-ahead candidate pool in pages, 0 = every page
    index_centroids: int = 0      # > 0: hierarchical index with this many centroids per unit
    index_iterations: int = 4     # k-means rounds of its build
    seed: int = 0

    @property
    def n_pages(self) -> int:
        return -(-self.ctx // self.page)

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def units(self) -> int:
        return self.batch * self.n_kv_heads

    @property
    def phys_layers(self) -> int:
        return self.physical_layers or self.n_layers

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float16 if self.dtype == "f16" else torch.bfloat16

    @property
    def page_bytes(self) -> int:
        return 2 * self.page * self.head_dim * 2

    def replace(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)


def _cfg(i: int, **kw) -> Workload:
    return Workload(name=f"cfg{i}", seed=1000 * i + 17, **kw)


# The five configurations of the benchmark definition (1-based, as it numbers them).
CONFIGS = {
    1: _cfg(1, n_layers=1, batch=1, ctx=4096, page=16, n_q_heads=32, n_kv_heads=8, dtype="f16",
            topk_pages=64, capacity=256, steps=1, importance="planted", heavy_count=8, warm="full"),
    2: _cfg(2, n_layers=32, batch=8, ctx=32768, page=16, n_q_heads=32, n_kv_heads=8, dtype="bf16",
            topk_pages=128, capacity=1024, steps=64, importance="planted",
            heavy_count=math.ceil(0.02 * 2048), physical_layers=8),
    3: _cfg(3, n_layers=1, batch=16, ctx=131072, page=16, n_q_heads=32, n_kv_heads=8, dtype="bf16",
            topk_pages=256, capacity=2048, steps=32, importance="zipf", zipf_alpha=1.1),
    4: _cfg(4, n_layers=28, batch=32, ctx=65536, page=32, n_q_heads=28, n_kv_heads=4, dtype="f16",
            topk_pages=64, capacity=(int(0.2 * 32 * 4 * 2048) // 32) // 4, steps=16, rho=0.95,
            importance="planted", heavy_count=math.ceil(0.01 * 2048), physical_layers=4),
    5: _cfg(5, n_layers=1, batch=4, ctx=1048576, page=64, n_q_heads=32, n_kv_heads=8, dtype="bf16",
            topk_pages=128, capacity=int(0.05 * 16384), steps=16, importance="zipf", zipf_alpha=1.2,
            recent_pages=64, warm="recent"),
}


def _gen(w: Workload, stream: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(w.seed * 16 + stream)
    return g


def initial_queries(w: Workload, device="cpu") -> torch.Tensor:
    """q0 [L, B, Hq, D] fp32 on `device`."""
    g = _gen(w, 1, device)
    return torch.randn(w.n_layers, w.batch, w.n_q_heads, w.head_dim, generator=g,
                       device=device, dtype=torch.float32)


def query_direction(w: Workload, q0: torch.Tensor) -> torch.Tensor:
    """u [L, B, Hkv, D]: unit vector along the group-mean of q0."""
    qg = q0.reshape(w.n_layers, w.batch, w.n_kv_heads, w.group, w.head_dim).mean(dim=3)
    return qg / qg.norm(dim=-1, keepdim=True)


def make_kv_store(w: Workload, q0: torch.Tensor, device="cpu", pin: Optional[bool] = None) -> torch.Tensor:
    """The paged K/V store [Lp, B, Hkv, NP, 2, P, D] in the KV dtype, on the host
    (pinned if `pin`, default: pinned when `device` is a GPU).  Drawn on `device`."""
    dev = torch.device(device)
    if pin is None:
        pin = dev.type == "cuda"
    Lp, B, H, NP, P, D = w.phys_layers, w.batch, w.n_kv_heads, w.n_pages, w.page, w.head_dim
    store = torch.empty((Lp, B, H, NP, 2, P, D), dtype=w.torch_dtype, pin_memory=pin)
    u = query_direction(w, q0.to(dev))                                  # [L, B, H, D]
    g_kv = _gen(w, 2, dev)
    g_imp = _gen(w, 3, dev)
    for lp in range(Lp):
        for b in range(B):
            kv = torch.randn(H, NP, 2, P, D, generator=g_kv, device=dev, dtype=torch.float32)
            shift = torch.zeros(H, NP, device=dev, dtype=torch.float32)
            if w.importance == "planted" and w.heavy_count > 0:
                for h in range(H):
                    idx = torch.randperm(NP, generator=g_imp, device=dev)[: w.heavy_count]
                    shift[h, idx] = w.heavy_shift
            elif w.importance == "zipf":
                for h in range(H):
                    perm = torch.randperm(NP, generator=g_imp, device=dev)
                    rank = torch.empty(NP, device=dev, dtype=torch.float32)
                    rank[perm] = torch.arange(1, NP + 1, device=dev, dtype=torch.float32)
                    shift[h] = w.zipf_amp * rank.pow(-w.zipf_alpha)
            # K (index 0 of the K/V axis) += shift * u, every token of the page
            kv[:, :, 0] += shift[:, :, None, None] * u[lp, b][:, None, None, :]
            store[lp, b].copy_(kv.to(w.torch_dtype))
            del kv
    return store


def query_stream(w: Workload, q0: torch.Tensor, steps: int, device="cpu") -> Iterator[torch.Tensor]:
    """Yields q_t [L, B, Hq, D] in the KV dtype on `device`, t = 0 .. steps-1.
    q_0 is q0; afterwards q_t = rho q_{t-1} + (1-rho) N(0,1) in fp32."""
    dev = torch.device(device)
    g = _gen(w, 4, dev)
    q = q0.to(dev, copy=True)
    for t in range(steps):
        if t > 0:
            noise = torch.randn(q.shape, generator=g, device=dev, dtype=torch.float32)
            q = w.rho * q + (1.0 - w.rho) * noise
        yield q.to(w.torch_dtype)


def warm_pages(w: Workload) -> Optional[torch.Tensor]:
    """Pages resident before step 0, identical for every unit: int32 [n] or None.
    "full": all pages (capacity covers the store); "recent": the forced recent
    window; "cold": nothing."""
    if w.warm == "full":
        return torch.arange(w.n_pages, dtype=torch.int32)
    if w.warm == "recent":
        return torch.arange(w.n_pages - w.recent_pages, w.n_pages, dtype=torch.int32)
    return None


def seq_lens(w: Workload) -> torch.Tensor:
    return torch.full((w.batch,), w.ctx, dtype=torch.int32)
