"""The seeded input generators (paper_2605_18071_amd/workloads.py): the five benchmark
configurations carry the sizes of the benchmark definition, and the generators are reproducible
and shaped as described.  No GPU needed."""
import math

import numpy as np
import pytest
import torch

from paper_2605_18071_amd import workloads as W


# (layers, batch, context, page, pages, q heads, kv heads, dtype, k, capacity per unit, units, page bytes, steps)
TABLE = {
    1: (1, 1, 4096, 16, 256, 32, 8, "f16", 64, 256, 8, 8192, 1),
    2: (32, 8, 32768, 16, 2048, 32, 8, "bf16", 128, 1024, 64, 8192, 64),
    3: (1, 16, 131072, 16, 8192, 32, 8, "bf16", 256, 2048, 128, 8192, 32),
    4: (28, 32, 65536, 32, 2048, 28, 4, "f16", 64, 409, 128, 16384, 16),
    5: (1, 4, 1048576, 64, 16384, 32, 8, "bf16", 128, 819, 32, 32768, 16),
}


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_configurations_carry_the_benchmark_definition(cfg):
    w = W.CONFIGS[cfg]
    got = (w.n_layers, w.batch, w.ctx, w.page, w.n_pages, w.n_q_heads, w.n_kv_heads, w.dtype, w.topk_pages, w.capacity,
           w.units, w.page_bytes, w.steps)
    assert got == TABLE[cfg]
    assert w.seed == 1000 * cfg + 17 and w.head_dim == 128 and w.policy == "lru"
    # token budgets 1024 / 2048 / 4096 / 2048 / 8192 tokens
    assert w.topk_pages * w.page == {1: 1024, 2: 2048, 3: 4096, 4: 2048, 5: 8192}[cfg]
    # window sizes: everything / 50 % / 25 % / a fifth of all pages shared out evenly / 5 %
    want_cap = {1: w.n_pages, 2: w.n_pages // 2, 3: w.n_pages // 4,
                4: (int(0.2 * w.batch * w.n_kv_heads * w.n_pages) // w.batch) // w.n_kv_heads, 5: int(0.05 * w.n_pages)}[cfg]
    assert w.capacity == want_cap
    assert w.rho == (0.95 if cfg == 4 else 0.9)
    assert (w.importance, w.warm) == {1: ("planted", "full"), 2: ("planted", "cold"), 3: ("zipf", "cold"),
                                      4: ("planted", "cold"), 5: ("zipf", "recent")}[cfg]
    if cfg == 5:
        assert w.recent_pages == 4096 // w.page and w.zipf_alpha == 1.2
    if cfg == 3:
        assert w.zipf_alpha == 1.1
    assert w.heavy_count == {1: 8, 2: math.ceil(0.02 * 2048), 3: 0, 4: math.ceil(0.01 * 2048), 5: 0}[cfg] or w.importance == "zipf"


def _small(**kw):
    base = dict(name="t", n_layers=2, batch=2, ctx=16 * 40, page=16, n_q_heads=8, n_kv_heads=2, dtype="bf16", topk_pages=8,
                capacity=16, steps=5, importance="planted", heavy_count=3, seed=99)
    base.update(kw)
    return W.Workload(**base)


def test_generators_are_reproducible_and_independent_per_tensor_kind():
    w = _small()
    q0a, q0b = W.initial_queries(w), W.initial_queries(w)
    assert torch.equal(q0a, q0b) and q0a.shape == (2, 2, 8, 128) and q0a.dtype == torch.float32
    sa, sb = W.make_kv_store(w, q0a), W.make_kv_store(w, q0a)
    assert torch.equal(sa.view(torch.int16), sb.view(torch.int16))
    assert sa.shape == (2, 2, 2, 40, 2, 16, 128) and sa.dtype == torch.bfloat16
    qa = [q.clone() for q in W.query_stream(w, q0a, 4)]
    qb = [q.clone() for q in W.query_stream(w, q0a, 4)]
    assert all(torch.equal(x.view(torch.int16), y.view(torch.int16)) for x, y in zip(qa, qb))
    # another seed: other tensors; drawing the store does not disturb the query stream
    w2 = w.replace(seed=100)
    assert not torch.equal(W.initial_queries(w2), q0a)
    assert torch.equal(qa[3].view(torch.int16), [q for q in W.query_stream(w, q0a, 4)][3].view(torch.int16))


def test_query_stream_drifts_as_stated():
    """q_0 is the initial query rounded to the KV dtype; q_t = rho q_{t-1} + (1 - rho) noise keeps a
    correlation of about rho with its predecessor and shrinks toward sqrt((1-rho)/(1+rho)) of its norm."""
    w = _small(rho=0.9, n_layers=1, batch=8, dtype="f16")
    q0 = W.initial_queries(w)
    qs = [q.float() for q in W.query_stream(w, q0, 60)]
    assert torch.equal(qs[0], q0.to(torch.float16).float())
    a, b = qs[10].flatten(), qs[11].flatten()
    corr = float((a @ b) / (a.norm() * b.norm()))
    assert 0.93 < corr < 0.999                                          # rho |q| dominates the (1 - rho) noise
    ratio = float(qs[59].norm() / qs[0].norm())
    assert abs(ratio - math.sqrt(0.1 / 1.9)) < 0.05                     # stationary norm of the AR(1) recursion


def test_planted_and_zipf_pages_are_shifted_along_the_query_direction():
    w = _small(n_layers=1, batch=1, heavy_count=4, heavy_shift=3.0)
    q0 = W.initial_queries(w)
    u = W.query_direction(w, q0)                                        # [L, B, Hkv, D]
    assert torch.allclose(u.norm(dim=-1), torch.ones(1, 1, 2), atol=1e-6)
    store = W.make_kv_store(w, q0).float()
    # mean over a page's tokens of K . u: about 3 for the planted pages, about 0 (+- 1/4) elsewhere
    proj = torch.einsum("hptd,hd->hp", store[0, 0, :, :, 0], u[0, 0]) / w.page
    for h in range(w.n_kv_heads):
        heavy = torch.nonzero(proj[h] > 1.5).flatten()
        assert len(heavy) == 4 and torch.all((proj[h][heavy] - 3.0).abs() < 1.0)
    v_proj = torch.einsum("hptd,hd->hp", store[0, 0, :, :, 1], u[0, 0]) / w.page
    assert float(v_proj.abs().max()) < 1.5                              # the values are not shifted
    wz = _small(n_layers=1, batch=1, importance="zipf", zipf_amp=6.0, zipf_alpha=1.1, heavy_count=0)
    sz = W.make_kv_store(wz, q0).float()
    pz = torch.einsum("hptd,hd->hp", sz[0, 0, :, :, 0], u[0, 0]) / wz.page
    top = torch.sort(pz, dim=1, descending=True).values
    assert torch.all((top[:, 0] - 6.0).abs() < 1.0) and torch.all((top[:, 1] - 6.0 * 2 ** -1.1).abs() < 1.0)


def test_warm_lists_and_physical_layers():
    assert W.warm_pages(_small()) is None
    assert W.warm_pages(_small(warm="full")).tolist() == list(range(40))
    assert W.warm_pages(_small(warm="recent", recent_pages=3)).tolist() == [37, 38, 39]
    w = _small(n_layers=4, physical_layers=2)
    assert w.phys_layers == 2 and W.make_kv_store(w, W.initial_queries(w)).shape[0] == 2
    assert W.initial_queries(w).shape[0] == 4                           # every logical layer has its own queries
    assert W.seq_lens(w).tolist() == [w.ctx, w.ctx]
