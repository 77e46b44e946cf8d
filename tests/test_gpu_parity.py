"""Parity of the HIP path (through the C ABI) against the CPU oracle, element by
element, on seeded inputs small enough for the oracle to finish in seconds but
spanning several tiles, ragged tails and the degenerate cases.  Runs on a GPU machine.
"""
import math

import numpy as np
import pytest
import torch

from oracle import kvd_oracle as orc
from paper_2605_18071_amd import workloads as W
from tests import helpers as H

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from paper_2605_18071_amd import kvd as K
    from tests import gpu_rig as R


def small(name, **kw):
    base = dict(name=name, n_layers=1, batch=2, ctx=16 * 300, page=16, n_q_heads=8, n_kv_heads=2, dtype="bf16",
                topk_pages=24, capacity=60, steps=6, importance="planted", heavy_count=5, seed=4242)
    base.update(kw)
    return W.Workload(**base)


def all_units(rig, layers=None):
    w = rig.w
    layers = range(w.n_layers) if layers is None else layers
    return [R.OracleUnit(rig, l, b, h) for l in layers for b in range(w.batch) for h in range(w.n_kv_heads)]


# --------------------------------------------------------------------------- #
# index build
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("dtype,page", [("bf16", 16), ("f16", 16), ("bf16", 64), ("f16", 20)])
def test_summaries_bit_exact(dtype, page):
    w = small("summ", dtype=dtype, page=page, ctx=page * 37, batch=2)
    rig = R.Rig(w, seq_lens=[w.ctx, w.ctx - page - 3])              # second sequence: ragged last page
    got = rig.summaries.cpu()
    for ou in all_units(rig):
        n = ou.summ.shape[0]
        want_bits = orc.f64_to_bits(ou.summ, ou.code)
        assert np.array_equal(H.bits(got[0, ou.b, ou.h, :n]), want_bits), (ou.b, ou.h)
    rig.close()


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_summaries_and_step_with_tiny_and_huge_keys(dtype):
    """Keys at the edges of the format: one sequence's keys scaled into the subnormal range of
    fp16 (bf16: 2^-125), the other's 4096 times the usual size (fp16: up to a quarter of the largest
    finite value).  The index must
    still be the correctly rounded mean (halves of the smallest subnormal round to even), and the
    step must still agree with the oracle."""
    w = small("edges", dtype=dtype, ctx=16 * 40, topk_pages=6, capacity=12, batch=2, steps=3)
    rig = R.Rig(w, build_index=False)
    tiny, huge = (2.0 ** -20 if dtype == "f16" else 2.0 ** -125), 2.0 ** 12      # (logits of some ten thousands)
    rig.store[0, 0, :, :, 0] = (rig.store[0, 0, :, :, 0].float() * tiny).to(w.torch_dtype)
    rig.store[0, 1, :, :, 0] = (rig.store[0, 1, :, :, 0].float() * huge).to(w.torch_dtype)
    rig.kvd.build_summaries(0)
    torch.cuda.synchronize()
    got = rig.summaries.cpu()
    units = all_units(rig)
    for ou in units:
        assert np.array_equal(H.bits(got[0, ou.b, ou.h]), orc.f64_to_bits(ou.summ, ou.code)), (ou.b, ou.h)
    sub = np.abs(units[0].summ)
    smallest_normal = 2.0 ** -14 if dtype == "f16" else 2.0 ** -126
    assert sub.max() < smallest_normal * 64 and (sub[sub > 0] < smallest_normal).any()   # (subnormal summaries do occur)
    rep = R.run_steps(rig, units, w.steps, check_dir_every=1, progress=f"edges-{dtype}")
    assert rep.unit_steps == w.steps * w.units
    rig.close()


# --------------------------------------------------------------------------- #
# stage 1: scores and selection
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("kw", [
    dict(),                                                         # 300 pages: one full 256-page block + tail
    dict(dtype="f16", n_q_heads=14, n_kv_heads=2, topk_pages=17),   # G = 7
    dict(ctx=16 * 1031, topk_pages=128, capacity=128),              # five blocks, ragged
    dict(ctx=16 * 40, topk_pages=64, capacity=64),                  # fewer valid pages than k -> padding
    dict(sink_pages=2, recent_pages=5),                             # forced pages
    dict(n_q_heads=2, n_kv_heads=2, topk_pages=1, capacity=4),      # G = 1, k = 1 -> argmax
])
def test_score_select_parity(kw):
    w = small("sel", **kw)
    seq = [w.ctx, w.ctx - 21] if w.ctx > 16 * 64 or "sink_pages" in kw else None
    rig = R.Rig(w, seq_lens=seq)
    rep = R.StepReport()
    for t, q in enumerate(W.query_stream(w, rig.q0, 3, R.DEV)):
        rig.kvd.score_select(0, q[0], rig.sel_pages, rig.scores)
        torch.cuda.synchronize()
        sel = rig.sel_pages.cpu().numpy()
        scores = rig.scores.cpu().numpy()
        for ou in all_units(rig):
            qg = H.f64(q[0][ou.b, ou.h * w.group:(ou.h + 1) * w.group])
            o_scores = orc.page_scores(orc.pooled_query(qg), ou.summ, ou.scale)
            o_sel = orc.select_pages(o_scores, w.topk_pages, w.sink_pages, w.recent_pages)
            n = o_scores.shape[0]
            err = np.abs(scores[ou.u, :n] - o_scores)
            assert np.all(err <= R.score_bound(ou, q[0])), err.max()
            if not np.array_equal(sel[ou.u], o_sel):
                ok, msg = H.selection_is_valid(o_scores, sel[ou.u], w.topk_pages, w.sink_pages, w.recent_pages)
                assert ok, msg
                rep.tie_divergences += 1
    assert rep.tie_divergences <= 1
    rig.close()


def test_select_exact_ties_go_to_lower_page():
    """Identical summary rows give bit-identical scores on both sides; the choice among
    them is then decided only by the tie rule."""
    w = small("ties", ctx=16 * 200, topk_pages=16, capacity=32, heavy_count=0)
    rig = R.Rig(w, build_index=False)
    g = torch.Generator(device=R.DEV)
    g.manual_seed(770_010)
    base = torch.randn(w.units, 10, w.head_dim, device=R.DEV, generator=g)
    idx = torch.randint(0, 10, (w.units, w.n_pages), device=R.DEV, generator=g)
    summ = torch.gather(base, 1, idx[:, :, None].expand(-1, -1, w.head_dim)).to(w.torch_dtype)
    rig.summaries.copy_(summ.view(rig.summaries.shape))
    q = next(W.query_stream(w, rig.q0, 1, R.DEV))
    rig.kvd.score_select(0, q[0], rig.sel_pages, rig.scores)
    torch.cuda.synchronize()
    sel = rig.sel_pages.cpu().numpy()
    summ64 = H.f64(summ)
    cls = idx.cpu().numpy()
    for b in range(w.batch):
        for h in range(w.n_kv_heads):
            u = b * w.n_kv_heads + h
            qg = H.f64(q[0][b, h * w.group:(h + 1) * w.group])
            sc = orc.page_scores(orc.pooled_query(qg), summ64[u], 1.0 / math.sqrt(w.head_dim))
            ok, msg = H.selection_is_valid(sc, sel[u], w.topk_pages)
            assert ok, msg
            # pages with the same summary row tie exactly on both sides: inside such a class the
            # selected pages must be the lowest-numbered ones
            chosen = set(sel[u].tolist())
            for c in range(10):
                members = np.nonzero(cls[u] == c)[0]
                flags = [int(p) in chosen for p in members]
                assert flags == sorted(flags, reverse=True), (u, c)
    # all scores equal: the k lowest pages win
    rig.summaries.zero_()
    rig.kvd.score_select(0, q[0], rig.sel_pages, None)
    torch.cuda.synchronize()
    assert np.array_equal(rig.sel_pages.cpu().numpy(), np.tile(np.arange(w.topk_pages), (w.units, 1)))
    rig.close()


# --------------------------------------------------------------------------- #
# stage 2: directory + fetch
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("n_pages,k,cap", [(120, 8, 8), (120, 8, 19), (700, 33, 70), (64, 16, 64), (3000, 200, 333)])
def test_resolve_trace_parity(n_pages, k, cap):
    """Random, locality-biased selection traces straight into kvd_cache_resolve."""
    w = small("lru", ctx=16 * n_pages, topk_pages=k, capacity=cap, batch=2, n_kv_heads=2, n_q_heads=4)
    rig = R.Rig(w, build_index=False)
    rng = np.random.default_rng(n_pages * 1000 + k)
    wins = [orc.LruWindow(cap) for _ in range(w.units)]
    for t in range(40):
        sel = np.zeros((w.units, k), dtype=np.int32)
        for u in range(w.units):
            centre = (t * 3 + 17 * u) % n_pages
            p = np.exp(-np.abs(np.arange(n_pages) - centre) / (2.0 * k)) + 1e-3
            sel[u] = np.sort(rng.choice(n_pages, size=k, replace=False, p=p / p.sum()))
        rig.sel_pages.copy_(torch.from_numpy(sel))
        rig.kvd.cache_resolve(0, t, rig.sel_pages, rig.sel_slots, rig.hit_mask, rig.evicted, rig.counts, do_gather=True)
        torch.cuda.synchronize()
        hm = rig.hit_mask.cpu().numpy()
        ev = rig.evicted.cpu().numpy()
        cnt = rig.counts.cpu().numpy()
        slots = rig.sel_slots.cpu().numpy()
        for u in range(w.units):
            hits, misses, evicted = wins[u].resolve(sel[u], t)
            assert sorted(sel[u][hm[u] == 1].tolist()) == hits, (t, u)
            assert sorted(sel[u][hm[u] == 0].tolist()) == misses, (t, u)
            assert sorted(ev[u][ev[u] >= 0].tolist()) == evicted, (t, u)
            assert cnt[u].tolist() == [len(hits), len(misses), len(evicted)]
            assert len(set(slots[u].tolist())) == k and slots[u].min() >= 0 and slots[u].max() < cap
        if t % 13 == 0 or t == 39:
            sp, st = rig.kvd.cache_export(0)
            for u in range(w.units):
                occ = sp[u] >= 0
                got = {int(p): int(s) for p, s in zip(sp[u][occ], st[u][occ])}
                assert got == wins[u].stamp, (t, u)
                b, h = divmod(u, w.n_kv_heads)
                for s in np.nonzero(occ.numpy())[0]:
                    a = rig.pool[0, b, h, int(s)].cpu().view(torch.int16).reshape(-1)
                    assert torch.equal(a, H.slot_image(rig.store[0, b, h, int(sp[u][s])])), (t, u, s)
    st = rig.kvd.stats()
    assert st.hits + st.misses == 40 * w.units * k
    assert st.gathered_bytes == st.misses * w.page_bytes
    rig.close()


@pytest.mark.parametrize("page", [16, 4], ids=["page16", "page4-packed"])
@pytest.mark.parametrize("generic", [False, True], ids=["fused", "size-agnostic"])
def test_resolve_and_attention_skip_padding_and_made_up_pages(generic, page, monkeypatch):
    """A caller's selection may hold -1 anywhere and pages that do not exist: both count as
    padding (no slot, no hit, no miss, no tokens), in the directory update and in the attention
    (with pages of 4 tokens the holes fall inside MFMA tiles)."""
    if generic:
        monkeypatch.setenv("KVD_GENERIC_SELECT", "1")
    w = small("holes", ctx=page * 90, page=page, topk_pages=10, capacity=14, batch=2, n_kv_heads=2, n_q_heads=8)
    rig = R.Rig(w, build_index=False)
    units = all_units(rig)
    rng = np.random.default_rng(606)
    q = next(W.query_stream(w, rig.q0, 1, R.DEV))[0]
    for t in range(6):
        sel = np.full((w.units, w.topk_pages), -1, dtype=np.int32)
        for u in range(w.units):
            real = np.sort(rng.choice(w.n_pages, size=6, replace=False))
            sel[u, [0, 2, 3, 5, 6, 9]] = real                          # ascending, with holes between
            sel[u, 4] = w.n_pages + 5                                  # pages that do not exist
            sel[u, 7] = 2 ** 30
        rig.sel_pages.copy_(torch.from_numpy(sel))
        rig.kvd.cache_resolve(0, t, rig.sel_pages, rig.sel_slots, rig.hit_mask, rig.evicted, rig.counts, do_gather=True)
        rig.kvd.sparse_decode_attn(0, q, rig.sel_pages, rig.sel_slots, rig.out, rig.lse)
        torch.cuda.synchronize()
        slots, hm, cnt = rig.sel_slots.cpu().numpy(), rig.hit_mask.cpu().numpy(), rig.counts.cpu().numpy()
        out, lse = rig.out.cpu().numpy(), rig.lse.cpu().numpy()
        for ou in units:
            u = ou.u
            valid = (sel[u] >= 0) & (sel[u] < w.n_pages)
            real = sel[u][valid]
            hits, misses, evicted = ou.window.resolve(real, t)
            assert np.all(slots[u][~valid] == -1) and np.all(hm[u][~valid] == 0)
            assert np.all(slots[u][valid] >= 0) and len(set(slots[u][valid].tolist())) == 6
            assert sorted(real[hm[u][valid] == 1].tolist()) == hits and cnt[u].tolist() == [len(hits), len(misses), len(evicted)]
            toks = orc.selected_tokens(real, w.page, ou.seq_len)
            G = w.group
            want, want_lse = orc.attend(H.f64(q[ou.b, ou.h * G:(ou.h + 1) * G]), ou.keys[toks], ou.values[toks], ou.scale)
            assert H.attn_rel_err(out[ou.b, ou.h * G:(ou.h + 1) * G], want) <= H.ATTN_RTOL, (t, u)
            assert np.abs(lse[ou.b, ou.h * G:(ou.h + 1) * G] - want_lse).max() <= 1e-3
    assert rig.kvd.stats().evictions > 0
    R.check_directory(rig, 0, units)
    rig.close()


@pytest.mark.parametrize("policy", ["lru", "lookahead"])
@pytest.mark.parametrize("mb", [-1, 1], ids=["single-launch", "kernel-chain"])
def test_cache_survives_export_reset_import_in_mid_run(mb, policy):
    """After some steps the directory is exported, the cache emptied (and the slot pool wiped) and
    the directory imported again: the slots are refilled from the host store and decoding goes on
    exactly as if nothing had happened."""
    w = small("export", topk_pages=20, capacity=30, steps=9, policy=policy)
    rig = R.Rig(w, micro_batches=mb)
    units = all_units(rig)
    rep = R.StepReport()
    for t, q in enumerate(W.query_stream(w, rig.q0, w.steps, R.DEV)):
        if t in (4, 7):
            sp, st = rig.kvd.cache_export(0)
            rig.kvd.cache_reset()
            rig.pool.fill_(float("nan"))
            empty, _ = rig.kvd.cache_export(0)
            assert bool((empty == -1).all())
            rig.kvd.cache_import(0, sp, st)
            R.check_directory(rig, 0, units)
        rig.step(0, t, q[0])
        for ou in units:
            R.compare_unit(rig, ou, t, q[0], rep)
    assert rep.unit_steps == w.steps * w.units and rig.kvd.stats().evictions > 0
    R.check_directory(rig, 0, units)
    rig.close()


def test_cache_export_import_and_warm_errors():
    w = small("imp", ctx=16 * 100, topk_pages=4, capacity=10, batch=1, n_kv_heads=2, n_q_heads=4)
    rig = R.Rig(w, build_index=False)
    rig.kvd.cache_warm(0, [5, 6, 7, 9, 8], [3, 2])
    sp, st = rig.kvd.cache_export(0)
    assert sp[0].tolist() == [5, 6, 7] + [-1] * 7 and sp[1].tolist() == [9, 8] + [-1] * 8
    assert st.max() == -1
    assert torch.equal(rig.pool[0, 0, 1, 0].cpu().view(torch.int16).reshape(-1), H.slot_image(rig.store[0, 0, 1, 9]))
    sp2 = sp.clone(); sp2[0, 4] = 42; st2 = st.clone(); st2[0, 4] = 3
    rig.kvd.cache_import(0, sp2, st2)
    a, b = rig.kvd.cache_export(0)
    assert torch.equal(a, sp2) and torch.equal(b, st2)
    assert torch.equal(rig.pool[0, 0, 0, 4].cpu().view(torch.int16).reshape(-1), H.slot_image(rig.store[0, 0, 0, 42]))
    bad = sp2.clone(); bad[1, 3] = 9                                # page 9 twice in unit 1
    with pytest.raises(K.KvdError) as e:
        rig.kvd.cache_import(0, bad, st2)
    assert e.value.status == K.ERR_STATE
    bad = sp2.clone(); bad[0, 2] = 100                              # page out of range
    with pytest.raises(K.KvdError):
        rig.kvd.cache_import(0, bad, st2)
    a, b = rig.kvd.cache_export(0)                                  # rejected imports leave the cache unchanged
    assert torch.equal(a, sp2) and torch.equal(b, st2)
    with pytest.raises(K.KvdError) as e:
        rig.kvd.cache_warm(0, list(range(11)) + [1], [11, 1])
    assert e.value.status == K.ERR_CAPACITY
    with pytest.raises(K.KvdError) as e:
        rig.kvd.cache_warm(0, [1, 1, 2], [2, 1])
    assert e.value.status == K.ERR_ARG
    rig.close()


def test_unbound_buffers_and_unpinned_store_are_rejected():
    k = K.Kvd(n_layers=1, batch=1, n_q_heads=4, n_kv_heads=1, page_size=16, max_pages=32, topk_pages=4,
              capacity_max=8, kv_dtype=torch.float16)
    q = torch.zeros(1, 4, 128, dtype=torch.float16, device=R.DEV)
    out = torch.zeros(1, 4, 128, dtype=torch.float32, device=R.DEV)
    with pytest.raises(K.KvdError) as e:
        k.step(0, 0, q, out)
    assert e.value.status == K.ERR_STATE
    pageable = torch.zeros(1, 1, 1, 32, 2, 16, 128, dtype=torch.float16)
    with pytest.raises(K.KvdError) as e:
        k.bind_host_store(pageable)
    assert e.value.status == K.ERR_ARG
    with pytest.raises(K.KvdError):
        k.set_seq_lens([16 * 32 + 1])
    k.close()


# --------------------------------------------------------------------------- #
# stage 3: attention
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("kw,splits", [
    (dict(), 0),
    (dict(), 1),
    (dict(dtype="f16"), 5),
    (dict(n_q_heads=2, n_kv_heads=2), 0),                            # G = 1
    (dict(n_q_heads=14, n_kv_heads=2, dtype="f16", page=32, ctx=32 * 150), 3),   # G = 7, two tiles per page
    (dict(n_q_heads=16, n_kv_heads=2, page=64, ctx=64 * 90), 0),     # G = 8, four tiles per page
    (dict(page=20, ctx=20 * 111, n_q_heads=6, n_kv_heads=2), 4),     # G = 3, page not a multiple of the tile
    (dict(ctx=16 * 30, topk_pages=40, capacity=40), 0),              # k > valid pages -> padded selection
    (dict(page=4, ctx=4 * 1000, topk_pages=50, capacity=120), 0),    # four pages per tile, a ragged last tile (50 pages)
    (dict(page=8, ctx=8 * 600, topk_pages=33, capacity=80, dtype="f16", n_q_heads=14, n_kv_heads=2), 3),   # two pages per tile, G = 7
    (dict(page=4, ctx=4 * 40, topk_pages=64, capacity=64), 0),       # k > valid pages with packed pages
])
def test_attention_parity(kw, splits):
    w = small("attn", **kw)
    seq = [w.ctx - 5, w.ctx - w.page - 1]                            # ragged last pages
    rig = R.Rig(w, seq_lens=seq, attn_splits=splits)
    units = all_units(rig)
    rng = np.random.default_rng(11)
    q = next(W.query_stream(w, rig.q0, 1, R.DEV))[0]
    k = w.topk_pages
    sel = np.full((w.units, k), -1, dtype=np.int32)
    for ou in units:
        n_valid = ou.summ.shape[0]
        kk = min(k, n_valid)
        pages = rng.choice(n_valid - 1, size=kk - 1, replace=False).tolist() + [n_valid - 1]   # ragged last page included
        sel[ou.u, :kk] = np.sort(np.asarray(pages, dtype=np.int32))
    rig.sel_pages.copy_(torch.from_numpy(sel))
    rig.kvd.cache_resolve(0, 0, rig.sel_pages, rig.sel_slots)
    rig.kvd.sparse_decode_attn(0, q, rig.sel_pages, rig.sel_slots, rig.out, rig.lse)
    torch.cuda.synchronize()
    out, lse = rig.out.cpu().numpy(), rig.lse.cpu().numpy()
    G = w.group
    for ou in units:
        toks = orc.selected_tokens(sel[ou.u], w.page, ou.seq_len)
        qg = H.f64(q[ou.b, ou.h * G:(ou.h + 1) * G])
        o, l = orc.attend(qg, ou.keys[toks], ou.values[toks], ou.scale)
        e = H.attn_rel_err(out[ou.b, ou.h * G:(ou.h + 1) * G], o)
        assert e <= H.ATTN_RTOL, (ou.b, ou.h, e)
        assert np.abs(lse[ou.b, ou.h * G:(ou.h + 1) * G] - l).max() <= 1e-3
    rig.close()


def test_attention_with_all_pages_equals_dense_and_ignores_cache_state():
    w = small("dense", ctx=16 * 48, topk_pages=48, capacity=48, dtype="f16")
    rig = R.Rig(w, seq_lens=[w.ctx, w.ctx - 7])
    q = next(W.query_stream(w, rig.q0, 1, R.DEV))[0]
    rig.step(0, 0, q)                                                 # cold: everything is fetched
    cold = rig.n_out.copy()
    assert rig.n_counts[:, 1].sum() > 0
    rig.step(0, 1, q)                                                 # warm: everything hits
    assert rig.n_counts[:, 1].sum() == 0
    assert np.array_equal(cold, rig.n_out)
    G = w.group
    for ou in all_units(rig):
        T = ou.seq_len
        qg = H.f64(q[ou.b, ou.h * G:(ou.h + 1) * G])
        logits = ou.scale * (qg @ ou.keys[:T].T)
        p = np.exp(logits - logits.max(axis=1, keepdims=True))
        dense = (p / p.sum(axis=1, keepdims=True)) @ ou.values[:T]
        assert H.attn_rel_err(cold[ou.b, ou.h * G:(ou.h + 1) * G], dense) <= H.ATTN_RTOL
    rig.close()


# --------------------------------------------------------------------------- #
# the whole step, several steps, scaled-down versions of the five configurations
# --------------------------------------------------------------------------- #
SCALED = {
    1: W.CONFIGS[1],                                                                    # full size already
    2: W.CONFIGS[2].replace(n_layers=3, physical_layers=2, batch=2, ctx=16 * 520, topk_pages=32, capacity=260,
                            heavy_count=11, steps=8),
    3: W.CONFIGS[3].replace(batch=2, ctx=16 * 1100, topk_pages=48, capacity=275, steps=8),
    4: W.CONFIGS[4].replace(n_layers=2, physical_layers=1, batch=3, ctx=32 * 300, topk_pages=16, capacity=60,
                            heavy_count=3, steps=6),
    5: W.CONFIGS[5].replace(batch=1, ctx=64 * 700, topk_pages=24, recent_pages=8, capacity=35, steps=6),
}


@pytest.mark.parametrize("mb", [-1, 1], ids=["single-launch", "kernel-chain"])
@pytest.mark.parametrize("n_pages", [77, 1031, 2050])
def test_step_parity_page_counts_off_the_load_width(n_pages, mb):
    """Page counts that are not a multiple of the selection's 4-page loads (77, 1031) or of a
    wave's 256-page block (2050), with ragged sequences: every thread's last pages are padding."""
    w = small("odd", ctx=16 * n_pages, topk_pages=min(40, n_pages // 2), capacity=max(48, n_pages // 8), steps=5,
              sink_pages=1, recent_pages=3)
    rig = R.Rig(w, seq_lens=[w.ctx - 7, w.ctx - 16 * 5 - 1], micro_batches=mb)
    units = all_units(rig)
    rep = R.run_steps(rig, units, w.steps, check_dir_every=2, progress=f"np{n_pages}-mb{mb}")
    assert rep.unit_steps == w.steps * w.units
    assert rep.tie_divergences <= 2
    rig.close()


@pytest.mark.parametrize("mb", [-1, 1], ids=["single-launch", "kernel-chain"])
@pytest.mark.parametrize("page,dtype,poison", [(16, "bf16", "nan"), (32, "f16", "inf"), (64, "bf16", "nan"), (8, "bf16", "nan"),
                                               (4, "f16", "inf"), (5, "bf16", "nan")])
def test_rows_beyond_the_sequence_end_may_hold_anything(page, dtype, poison, mb):
    """A store whose rows beyond every sequence's end hold NaNs or infinities (a caller's
    uninitialised memory): pages are copied whole into their slots, so the attention kernels
    have to keep those rows out themselves; the ragged last page is selected at every step."""
    w = small("poisoned-tail", page=page, dtype=dtype, ctx=page * 120, topk_pages=20, capacity=44, steps=4,
              recent_pages=2)
    seq_lens = [w.ctx - page - 5, w.ctx - 1]
    rig = R.Rig(w, seq_lens=seq_lens, micro_batches=mb, build_index=False)
    bad = float("nan") if poison == "nan" else float("inf")
    for b, n in enumerate(seq_lens):
        p0, r = divmod(n, page)
        rig.store[:, b, :, p0, :, r:, :] = bad
        rig.store[:, b, :, p0 + 1:] = -bad if poison == "inf" else bad
    rig.kvd.build_summaries(0)
    torch.cuda.synchronize()
    units = all_units(rig)
    rep = R.run_steps(rig, units, w.steps, check_dir_every=2, progress=f"poisoned-p{page}-mb{mb}")
    assert rep.unit_steps == w.steps * w.units
    assert rep.tie_divergences <= 2
    rig.close()


@pytest.mark.parametrize("kw", [
    dict(ctx=16 * 8200, topk_pages=48, capacity=300),                 # 8200 pages: 9 per thread, ragged wave blocks
    dict(ctx=32 * 8192, page=32, dtype="f16", n_q_heads=14, n_kv_heads=2, topk_pages=40, capacity=128, policy="lookahead"),
    dict(ctx=64 * 16384, page=64, topk_pages=64, capacity=96, recent_pages=6, batch=1),   # the largest unit the form takes
], ids=["8200-pages", "8192-pages-f16-g7-lookahead", "16384-pages"])
def test_step_parity_units_of_8192_pages_and_more(kw):
    """Units of 8192 pages and more run the one-launch step with 1024-thread workgroups."""
    w = small("wide", steps=4, **kw)
    rig = R.Rig(w, seq_lens=[w.ctx - 5, w.ctx - 3 * w.page - 1][:w.batch], micro_batches=-1)
    assert rig.kvd.step_form() == -1
    units = all_units(rig)
    rep = R.run_steps(rig, units, w.steps, check_dir_every=2, progress="wide")
    assert rep.unit_steps == w.steps * w.units
    assert rep.tie_divergences <= 2 and rep.victim_tie_divergences <= 2
    rig.close()


@pytest.mark.parametrize("mb,policy", [(-1, "lru"), (1, "lookahead"), (-1, "lookahead")],
                         ids=["single-launch-lru", "kernel-chain-lookahead", "single-launch-lookahead"])
def test_step_parity_at_the_largest_sizes_of_the_fused_kernels(mb, policy):
    """The limits of the register-resident kernels all at once: 16384 pages, 2048 selected pages,
    a window of 4096 slots, 8 query heads per KV head; the second sequence a little shorter."""
    w = small("largest", ctx=16 * 16384, topk_pages=2048, capacity=4096, batch=2, n_kv_heads=1, n_q_heads=8,
              heavy_count=64, steps=6, policy=policy, seed=31337, rho=0.2)     # (a fast-drifting query: the window fills and evicts)
    rig = R.Rig(w, seq_lens=[w.ctx, w.ctx - 16 * 37 - 9], micro_batches=mb)
    assert rig.kvd.step_form() == mb
    units = all_units(rig)
    rep = R.run_steps(rig, units, w.steps, check_dir_every=2, progress=f"largest-mb{mb}-{policy}")
    assert rep.unit_steps == w.steps * w.units and rig.kvd.stats().evictions > 0
    assert rep.tie_divergences <= 4 and rep.victim_tie_divergences <= 4
    rig.close()


def test_step_parity_beyond_the_fused_kernels_sizes():
    """More pages (16400) and more slots (4100) than the register-resident kernels take: the
    size-agnostic select / resolve / fetch kernels run without being asked for."""
    w = small("beyond", ctx=16 * 16400, topk_pages=300, capacity=4100, batch=1, n_kv_heads=2, n_q_heads=4,
              heavy_count=32, steps=3, seed=31338)
    rig = R.Rig(w, seq_lens=[w.ctx - 21])
    assert rig.kvd.step_form() == 1                                   # (no one-launch step at these sizes)
    units = all_units(rig)
    rep = R.run_steps(rig, units, w.steps, check_dir_every=2, progress="beyond")
    assert rep.unit_steps == w.steps * w.units and rep.tie_divergences <= 2
    rig.close()


@pytest.mark.parametrize("page,n_pages,mb", [(1, 700, 0), (3, 300, 0), (255, 40, 0), (256, 48, 0), (4, 900, 0), (4, 900, 1), (8, 500, 0),
                                            (8, 500, 1)])
def test_step_parity_extreme_page_sizes_and_very_short_sequences(page, n_pages, mb):
    """Pages of one token, of an odd few, of 4 and 8 tokens (packed slots: several pages per MFMA
    tile; as one launch and as a chain of kernels) and of the largest sizes (255: not a multiple of
    the 16-token tile, 256: sixteen tiles), in a batch whose second sequence has fewer valid pages
    than the budget and whose third is a single token long."""
    w = small("pages", page=page, ctx=page * n_pages, topk_pages=12 if page not in (4, 8) else 42, capacity=20 if page not in (4, 8) else 70,
              batch=3, steps=5, heavy_count=4, seed=2718 + page)
    seq = [w.ctx - (page // 2), 5 * page + (1 if page > 1 else 0), 1]
    rig = R.Rig(w, seq_lens=seq, micro_batches=mb)
    assert (rig.kvd.step_form() == -1) == ((page % 16 == 0 or page in (4, 8)) and mb == 0)
    units = all_units(rig)
    rep = R.run_steps(rig, units, w.steps, check_dir_every=2, progress=f"page{page}")
    assert rep.unit_steps == w.steps * w.units and rep.tie_divergences <= 2
    # the single-token sequence: one page selected, the rest padding, from the first step on
    last = rig.n_sel_pages[2 * w.n_kv_heads:]
    assert np.all(last[:, 0] == 0) and np.all(last[:, 1:] == -1)
    rig.close()


@pytest.mark.parametrize("mb", [-1, 1], ids=["single-launch", "kernel-chain"])
@pytest.mark.parametrize("name,kw", [
    ("window-equals-budget", dict(topk_pages=24, capacity=24)),                       # every unselected page leaves at once
    ("window-holds-everything", dict(ctx=16 * 90, topk_pages=24, capacity=90)),       # a page misses once at most
    ("all-forced", dict(topk_pages=10, capacity=30, sink_pages=4, recent_pages=6)),   # nothing left to choose
    ("one-unit", dict(batch=1, n_kv_heads=1, n_q_heads=8)),
    ("many-units", dict(batch=80, n_kv_heads=8, n_q_heads=8, ctx=16 * 64, topk_pages=8, capacity=12, heavy_count=3)),   # 640 units
    ("lookahead-window-equals-budget", dict(topk_pages=24, capacity=24, policy="lookahead")),
])
def test_step_parity_degenerate_windows_and_unit_counts(name, kw, mb):
    w = small(name, steps=6, **kw)
    rig = R.Rig(w, micro_batches=mb)
    units = all_units(rig) if w.units <= 32 else [R.OracleUnit(rig, 0, b, h) for b, h in [(0, 0), (17, 3), (41, 7), (79, 7), (63, 0)]]
    rep = R.run_steps(rig, units, w.steps, check_dir_every=2, progress=f"{name}-mb{mb}")
    assert rep.unit_steps == w.steps * len(units) and rep.tie_divergences + rep.victim_tie_divergences <= 2
    st = rig.kvd.stats()
    if name == "window-holds-everything":
        assert st.evictions == 0 and st.misses <= w.units * w.n_pages
    if name.endswith("window-equals-budget"):
        assert st.evictions == st.misses - w.units * w.topk_pages     # after the cold step every miss displaces a page
    if name == "all-forced":
        assert st.misses == w.units * w.topk_pages                     # the same ten pages every step: cold misses only
    rig.close()


@pytest.mark.parametrize("mb", [-1, 1], ids=["single-launch", "kernel-chain"])
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_step_parity_with_extreme_queries(dtype, mb):
    """Queries that make the softmax hard: all zeros (every token weighs the same: the output is
    the mean of the selected values, the scores all tie and the lowest pages are selected), and
    queries 40 times the usual size (logits of a few hundred either way, one token taking nearly
    all the weight)."""
    w = small("extreme-q", dtype=dtype, topk_pages=16, capacity=30, steps=1)
    rig = R.Rig(w, micro_batches=mb)
    units = all_units(rig)
    rep = R.StepReport()
    q0 = next(W.query_stream(w, rig.q0, 1, R.DEV))[0]
    zero = torch.zeros_like(q0)
    rig.step(0, 0, zero)
    for ou in units:
        want = R.compare_unit(rig, ou, 0, zero, rep)
        assert rig.n_sel_pages[ou.u].tolist() == list(range(16))      # all scores 0: ties go to the lowest pages
        vals = ou.values[: 16 * w.page].mean(axis=0)
        G = w.group
        assert np.allclose(rig.n_out[ou.b, ou.h * G:(ou.h + 1) * G], vals[None, :], rtol=0, atol=2e-3 * np.abs(vals).max())
        assert np.allclose(want["lse"], math.log(16 * w.page))
    big = (q0.float() * 40.0).to(q0.dtype)
    for t in (1, 2):
        rig.step(0, t, big)
        for ou in units:
            want = R.compare_unit(rig, ou, t, big, rep)
            assert np.abs(want["lse"]).max() > 50.0                    # (the logits really are large)
    assert rep.tie_divergences == 0
    rig.close()


def test_two_contexts_step_concurrently_on_two_streams():
    """Two contexts of different shapes, forms and policies, their steps enqueued on two streams
    with no synchronisation between them: neither disturbs the other (the library keeps no state
    outside its contexts)."""
    wa = small("ctx-a", dtype="f16", topk_pages=20, capacity=30, steps=6, seed=11)
    wb = small("ctx-b", dtype="bf16", page=32, ctx=32 * 200, n_q_heads=14, n_kv_heads=2, topk_pages=12, capacity=18,
               policy="lookahead", steps=6, seed=12)
    a, b = R.Rig(wa, micro_batches=-1), R.Rig(wb, micro_batches=2)
    ua, ub = all_units(a), all_units(b)
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    rep_a, rep_b = R.StepReport(), R.StepReport()
    qa, qb = W.query_stream(wa, a.q0, wa.steps, R.DEV), W.query_stream(wb, b.q0, wb.steps, R.DEV)
    torch.cuda.synchronize()
    for t in range(6):
        q1, q2 = next(qa)[0].contiguous(), next(qb)[0].contiguous()
        torch.cuda.synchronize()                                      # (the queries are ready; the steps below overlap)
        for rig, q, st in ((a, q1, sa), (b, q2, sb)):
            rig.kvd.step(0, t, q, rig.out, rig.lse, stream=st)
            rig.kvd.step_trace(rig.sel_pages, rig.sel_slots, rig.hit_mask, rig.evicted, rig.counts, rig.scores, stream=st)
        torch.cuda.synchronize()
        for rig, units, q, rep in ((a, ua, q1, rep_a), (b, ub, q2, rep_b)):
            rig.n_sel_pages, rig.n_sel_slots = rig.sel_pages.cpu().numpy(), rig.sel_slots.cpu().numpy()
            rig.n_hit_mask, rig.n_evicted = rig.hit_mask.cpu().numpy(), rig.evicted.cpu().numpy()
            rig.n_counts, rig.n_scores = rig.counts.cpu().numpy(), rig.scores.cpu().numpy()
            rig.n_out, rig.n_lse = rig.out.cpu().numpy(), rig.lse.cpu().numpy()
            for ou in units:
                R.compare_unit(rig, ou, t, q, rep)
    R.check_directory(a, 0, ua)
    R.check_directory(b, 0, ub)
    assert rep_a.unit_steps == 6 * wa.units and rep_b.unit_steps == 6 * wb.units
    a.close()
    b.close()


@pytest.mark.parametrize("env", [dict(KVD_FUSE_MERGE="0"), dict(KVD_SCORE_BLOCKS="7"), dict(KVD_SCORE_BLOCKS="100000"),
                                 dict(KVD_FUSE_MERGE="0", KVD_GENERIC_SELECT="1")],
                         ids=["separate-merge-kernel", "seven-score-blocks", "many-score-blocks", "separate-everything"])
def test_chain_of_kernels_in_its_other_launch_shapes(env, monkeypatch):
    """The chain of kernels with the attention splits merged by a kernel of its own instead of by
    the last split, and with the scoring grid far smaller and far larger than the default."""
    for k_, v_ in env.items():
        monkeypatch.setenv(k_, v_)
    w = small("shapes", ctx=16 * 1500, topk_pages=96, capacity=150, steps=5, n_q_heads=14, n_kv_heads=2, dtype="f16")
    rig = R.Rig(w, seq_lens=[w.ctx, w.ctx - 16 * 9 - 5], micro_batches=1, attn_splits=5)
    units = all_units(rig)
    rep = R.run_steps(rig, units, w.steps, check_dir_every=2, progress="shapes")
    assert rep.unit_steps == w.steps * w.units and rep.tie_divergences <= 2
    rig.kvd.set_profiling(1)                                          # the profiled chain brackets the merge kernel too
    q = next(W.query_stream(w, rig.q0, 1, R.DEV))[0]
    rig.step(0, w.steps, q)
    for ou in units:
        R.compare_unit(rig, ou, w.steps, q, rep)
    st = rig.kvd.stats()
    assert st.profiled_steps == 1 and st.ms_attend > 0 and (st.ms_merge > 0) == (env.get("KVD_FUSE_MERGE") == "0")
    rig.close()


@pytest.mark.parametrize("mb", [-1, 1], ids=["single-launch", "kernel-chain"])
def test_step_parity_one_attention_split_per_unit(mb):
    """So few selected pages that a unit's attention is one workgroup (no partials, no merge)."""
    w = small("one-split", topk_pages=6, capacity=7, steps=8)
    rig = R.Rig(w, micro_batches=mb)
    units = all_units(rig)
    rep = R.run_steps(rig, units, w.steps, check_dir_every=2, progress=f"one-split-mb{mb}")
    assert rep.unit_steps == w.steps * w.units and rep.tie_divergences <= 2
    assert rig.kvd.stats().evictions > 0
    rig.close()


@pytest.mark.parametrize("policy", ["lru", "lookahead"])
@pytest.mark.parametrize("mb", [-1, 1, 2], ids=["single-launch", "kernel-chain", "two-groups"])
@pytest.mark.parametrize("n_layers,phys,centroids", [(4, 2, 0), (3, 3, 0), (3, 2, 48), (10, 2, 0)])
def test_layers_in_flight_equal_layers_one_by_one(n_layers, phys, centroids, mb, policy):
    """kvd_step_layers overlaps the layers: as one launch whose workgroups are ordered so that the
    layers (up to 8 per launch; 10 layers take two launches) pipeline through the compute units, in
    several launch shapes, or as chains of kernels on two streams with two scratch sets.  Every
    layer has its own directory and slots, so scores, traces, directories and slot contents must be
    those of the layers stepped one by one, and the outputs too (bit for bit with the chain of
    kernels; up to the order in which the splits are merged in one launch).  The one-by-one run is
    compared with the oracle at every layer-step."""
    if n_layers == 10 and (mb == 2 or policy == "lookahead"):
        pytest.skip("ten layers: the launch that covers eight of them is what is new there")
    w = small("layers", n_layers=n_layers, physical_layers=phys, ctx=16 * 700, topk_pages=40, capacity=46, steps=7,
              policy=policy, batch=3, n_kv_heads=2, n_q_heads=8, index_centroids=centroids)
    a = R.Rig(w, micro_batches=mb)
    b = R.Rig(w, micro_batches=mb, build_index=False)
    b.summaries.copy_(a.summaries)
    if centroids:
        b.centroids.copy_(a.centroids)
        b.cluster_start.copy_(a.cluster_start)
        b.cluster_pages.copy_(a.cluster_pages)
        for l in range(n_layers):
            b.kvd.refresh_clusters(l)
        torch.cuda.synchronize()
    assert a.kvd.step_form() == mb and b.kvd.step_form() == mb
    units = all_units(a)
    by_layer = {l: [ou for ou in units if ou.layer == l] for l in range(n_layers)}
    rep = R.StepReport()
    L, B, Hq, D = n_layers, w.batch, w.n_q_heads, w.head_dim
    out_l = torch.empty((L, B, Hq, D), dtype=torch.float32, device=R.DEV)
    lse_l = torch.empty((L, B, Hq), dtype=torch.float32, device=R.DEV)
    i32 = dict(dtype=torch.int32, device=R.DEV)
    tr = [torch.empty((w.units, w.topk_pages), **i32) for _ in range(4)]
    for t, q in enumerate(W.query_stream(w, a.q0, w.steps, R.DEV)):
        outs, lses, last = [], [], None
        for l in range(L):
            a.step(l, t, q[l])
            for ou in by_layer[l]:
                R.compare_unit(a, ou, t, q[l], rep)
            outs.append(a.n_out.copy())
            lses.append(a.n_lse.copy())
            last = (a.n_sel_pages.copy(), a.n_sel_slots.copy(), a.n_hit_mask.copy(), a.n_evicted.copy())
        out_l.fill_(float("nan"))
        if mb == -1:                                     # (passes, scoring workgroups, splits, groups) of the launches of several layers
            b.kvd.set_step_shape(*[(0, 0, 0, 0), (1, 7, 1, 2), (2, 30, 2, 3)][t % 3], multi_layer=True)
            b.kvd.set_step_shape(*[(0, 0, 0, 0), (2, 9, 0, 4)][t % 2])
        if t % 2 == 0:
            b.kvd.step_layers(0, L, t, q.contiguous(), out_l, lse_l)
        else:                                            # a range that starts on another layer, then the rest
            b.kvd.step(0, t, q[0], out_l[0], lse_l[0])
            b.kvd.step_layers(1, L - 1, t, q[1:].contiguous(), out_l[1:], lse_l[1:])
        b.kvd.step_trace(tr[0], tr[1], tr[2], tr[3])
        torch.cuda.synchronize()
        for l in range(L):
            got = out_l[l].cpu().numpy()
            if mb >= 1:
                assert np.array_equal(got, outs[l]) and np.array_equal(lse_l[l].cpu().numpy(), lses[l]), (t, l)
            else:
                assert H.attn_rel_err(got, outs[l]) <= 1e-5, (t, l)
                assert np.abs(lse_l[l].cpu().numpy() - lses[l]).max() <= 1e-5, (t, l)
            pa, sa = a.kvd.cache_export(l)
            pb, sb = b.kvd.cache_export(l)
            assert torch.equal(pa, pb) and torch.equal(sa, sb), (t, l)
            assert torch.equal(a.pool[l], b.pool[l]), (t, l)
        # the trace left behind is the last layer's
        assert np.array_equal(tr[0].cpu().numpy(), last[0]) and np.array_equal(tr[1].cpu().numpy(), last[1])
        assert np.array_equal(tr[2].cpu().numpy(), last[2])
        assert np.array_equal(np.sort(tr[3].cpu().numpy(), axis=1), np.sort(last[3], axis=1))
        sa_, sb_ = a.kvd.stats(), b.kvd.stats()
        assert (sa_.hits, sa_.misses, sa_.evictions) == (sb_.hits, sb_.misses, sb_.evictions)
        print(f"[layers-{n_layers}-mb{mb}-{policy}] step {t} ok", flush=True)
    assert rep.unit_steps == w.steps * w.units * L and a.kvd.stats().evictions > 0
    a.close()
    b.close()


@pytest.mark.parametrize("mb", [-1, 1], ids=["single-launch", "kernel-chain"])
def test_layers_in_flight_in_a_growing_store(mb):
    """A decode loop as a model runs it: all layers stepped (two in flight), then every layer
    appends its new token, then the sequences advance.  Outputs, directories, slot contents, index
    and host store must be those of the same loop with the layers stepped one by one."""
    w = small("layers-append", n_layers=3, physical_layers=3, ctx=16 * 300, topk_pages=24, capacity=30, recent_pages=2,
              steps=20, batch=2)
    seq = [w.ctx - 16 * 2 - 7, w.ctx - 16 * 3]
    a = R.Rig(w, seq_lens=seq, micro_batches=mb)
    b = R.Rig(w, seq_lens=seq, micro_batches=mb, build_index=False)
    b.summaries.copy_(a.summaries)
    L = w.n_layers
    shape = (L, w.batch, w.n_q_heads, w.head_dim)
    out_a = torch.empty(shape, dtype=torch.float32, device=R.DEV)
    out_b = torch.empty(shape, dtype=torch.float32, device=R.DEV)
    gen = torch.Generator(device="cpu").manual_seed(5)
    for t, q in enumerate(W.query_stream(w, a.q0, w.steps, R.DEV)):
        q = q.contiguous()
        for l in range(L):
            a.kvd.step(l, t, q[l], out_a[l])
        b.kvd.step_layers(0, L, t, q, out_b)
        for l in range(L):
            k_new = torch.randn((w.batch, w.n_kv_heads, w.head_dim), generator=gen).to(w.torch_dtype).to(R.DEV)
            v_new = torch.randn((w.batch, w.n_kv_heads, w.head_dim), generator=gen).to(w.torch_dtype).to(R.DEV)
            a.kvd.append_kv(l, k_new, v_new)
            b.kvd.append_kv(l, k_new, v_new)
        a.kvd.advance()
        b.kvd.advance()
        torch.cuda.synchronize()
        if mb == 1:
            assert torch.equal(out_a, out_b), t
        else:
            assert H.attn_rel_err(out_b.cpu().numpy(), out_a.cpu().numpy()) <= 1e-5, t
        if t % 5 == 4 or t == w.steps - 1:
            for l in range(L):
                pa, sa = a.kvd.cache_export(l)
                pb, sb = b.kvd.cache_export(l)
                assert torch.equal(pa, pb) and torch.equal(sa, sb), (t, l)
            assert torch.equal(a.pool.view(torch.int16), b.pool.view(torch.int16)), t
            assert torch.equal(a.summaries.view(torch.int16), b.summaries.view(torch.int16)), t
            assert torch.equal(a.store.view(torch.int16), b.store.view(torch.int16)), t
    sa_, sb_ = a.kvd.stats(), b.kvd.stats()
    assert (sa_.hits, sa_.misses, sa_.evictions) == (sb_.hits, sb_.misses, sb_.evictions) and sa_.evictions > 0
    a.close()
    b.close()


def test_step_layers_rejects_ranges_outside_the_context():
    w = small("layers-args", n_layers=2, physical_layers=1)
    rig = R.Rig(w)
    q = next(iter(W.query_stream(w, rig.q0, 1, R.DEV)))
    out = torch.empty((2, w.batch, w.n_q_heads, w.head_dim), dtype=torch.float32, device=R.DEV)
    for layer0, n in [(-1, 1), (0, 0), (0, 3), (1, 2), (2, 1)]:
        with pytest.raises(K.KvdError):
            rig.kvd.step_layers(layer0, n, 0, q, out)
    rig.kvd.step_layers(0, 2, 0, q, out)
    torch.cuda.synchronize()
    rig.close()


@pytest.mark.parametrize("policy", ["lru", "lookahead"])
@pytest.mark.parametrize("mb", [-1, 1], ids=["single-launch", "kernel-chain"])
def test_step_parity_with_repeated_step_indices(mb, policy):
    """A step index may repeat (a replayed step): the pages selected in a step then tie in stamp
    with unselected ones, and the victims must still come from the unselected pages only."""
    w = small("repeat", topk_pages=20, capacity=26, steps=12, policy=policy)
    rig = R.Rig(w, micro_batches=mb)
    units = all_units(rig)
    rep = R.StepReport()
    for i, q in enumerate(W.query_stream(w, rig.q0, w.steps, R.DEV)):
        t = i // 3                                                     # every index three times
        rig.step(0, t, q[0])
        for ou in units:
            R.compare_unit(rig, ou, t, q[0], rep)
        if i % 4 == 3:
            R.check_directory(rig, 0, units)
    assert rep.unit_steps == w.steps * w.units and rig.kvd.stats().evictions > 0
    rig.close()


@pytest.mark.parametrize("seed", list(range(64)))
def test_random_shapes_against_the_oracle(seed):
    """Seeded random shapes (pages, page size, heads, group, budget, window, policy, dtype, ragged
    lengths, forced pages), stepped in the form the seed picks, compared with the oracle on up to
    four units of the layer at every step: scores, selection, trace, directory, output."""
    rng = np.random.default_rng(7700 + seed)
    page = int(rng.choice([16, 32, 64, 4, 8, 16]))
    n_pages = int(rng.choice([p for p in (40, 130, 257, 1000, 2050) if p * page <= 40000]))
    hkv = int(rng.choice([1, 2, 4]))
    group = int(rng.choice([1, 2, 4, 7, 8]))
    k = int(rng.integers(1, min(n_pages // 2, 96) + 1))
    cap = int(min(n_pages, k + rng.integers(0, 2 * k + 2)))
    forced = k > 6
    kw = dict(ctx=page * n_pages, page=page, n_kv_heads=hkv, n_q_heads=hkv * group, dtype=str(rng.choice(["bf16", "f16"])),
              topk_pages=k, capacity=cap, batch=int(rng.choice([1, 2, 3])), policy=str(rng.choice(["lru", "lookahead"])),
              sink_pages=int(rng.integers(0, 3)) if forced else 0, recent_pages=int(rng.integers(0, 3)) if forced else 0,
              heavy_count=min(5, n_pages // 8), steps=5, seed=900 + seed)
    # seeds from 12 on also draw (from a generator of their own, so that the shapes above stay what
    # they were) a finite look-ahead pool, a hierarchical index and a launch shape of the one-launch step
    extra = np.random.default_rng(880000 + seed)
    if seed >= 12:
        if kw["policy"] == "lookahead" and extra.random() < 0.6:
            kw["lookahead_pool"] = int(extra.integers(k, n_pages + 1))
        if n_pages >= 130 and extra.random() < 0.35:
            kw["index_centroids"] = max(4, n_pages // int(extra.choice([2, 3, 8])))
            kw["index_iterations"] = 2
    w = small("rand-oracle", **kw)
    seq = [int(w.ctx - rng.integers(0, 3 * page)) for _ in range(w.batch)]
    mb = int(rng.choice([-1, 1, 2])) if w.batch >= 2 else int(rng.choice([-1, 1]))
    rig = R.Rig(w, seq_lens=seq, micro_batches=mb)
    if seed >= 12 and mb == -1 and rig.kvd.step_form() == -1:
        shape = (int(extra.integers(0, 5)), int(extra.choice([0, 1, 5, 64])), int(extra.integers(0, 4)), int(extra.choice([0, 1, 2, 4])))
        try:
            rig.kvd.set_step_shape(*shape)
        except K.KvdError as e:                                        # (more splits than the budget has pages, ...)
            assert e.status == K.ERR_SHAPE, (kw, shape)
        kw["shape"] = rig.kvd.step_shape()
    picks = rng.permutation(w.units)[:4]
    units = [R.OracleUnit(rig, 0, int(u) // hkv, int(u) % hkv) for u in picks]
    rep = R.run_steps(rig, units, w.steps, check_dir_every=2, progress=f"rand-oracle-{seed}")
    assert rep.unit_steps == w.steps * len(units), kw
    assert rep.tie_divergences + rep.victim_tie_divergences <= 3, kw
    rig.close()


@pytest.mark.parametrize("seed", list(range(32)))
def test_one_launch_equals_chain_on_random_shapes(seed):
    """Seeded random shapes (pages, page size, heads, budget, window, policy, ragged lengths): the
    one-launch step and the chain of kernels, fed the same queries from the same cold start, must
    give the same scores, selections, traces and slots at every step, and the same outputs up to
    the fp32 summation order of the attention.  (Either form is checked against the oracle
    elsewhere; this one covers many shapes quickly.)"""
    rng = np.random.default_rng(9100 + seed)
    page = int(rng.choice([16, 32, 64, 4, 8, 16]))
    n_pages = int(rng.choice([40, 257, 1000, 2048, 4100, 8192, 9000]))
    hkv = int(rng.choice([1, 2, 4]))
    group = int(rng.choice([1, 2, 4, 7, 8]))
    k = int(rng.integers(1, min(n_pages // 2, 200) + 1))
    cap = int(min(n_pages, k + rng.integers(0, 3 * k + 2)))
    kw = dict(ctx=page * n_pages, page=page, n_kv_heads=hkv, n_q_heads=hkv * group, dtype=str(rng.choice(["bf16", "f16"])),
              topk_pages=k, capacity=cap, batch=int(rng.choice([1, 2, 3])), policy=str(rng.choice(["lru", "lookahead"])),
              sink_pages=int(rng.integers(0, 2)) if k > 4 else 0, recent_pages=int(rng.integers(0, 3)) if k > 4 else 0,
              heavy_count=min(5, n_pages // 8), steps=5, seed=500 + seed)
    w = small("rand", **kw)
    seq = [int(w.ctx - rng.integers(0, 3 * page)) for _ in range(w.batch)]
    a = R.Rig(w, seq_lens=seq, micro_batches=-1)
    b = R.Rig(w, seq_lens=seq, micro_batches=1, build_index=False)
    b.summaries.copy_(a.summaries)
    assert a.kvd.step_form() == -1 and b.kvd.step_form() == 1
    for t, q in enumerate(W.query_stream(w, a.q0, w.steps, R.DEV)):
        a.step(0, t, q[0])
        b.step(0, t, q[0])
        assert np.array_equal(a.n_scores, b.n_scores), (kw, t)
        assert np.array_equal(a.n_sel_pages, b.n_sel_pages), (kw, t)
        assert np.array_equal(a.n_hit_mask, b.n_hit_mask), (kw, t)
        assert np.array_equal(a.n_sel_slots, b.n_sel_slots), (kw, t)
        assert np.array_equal(np.sort(a.n_evicted, axis=1), np.sort(b.n_evicted, axis=1)), (kw, t)
        assert np.array_equal(a.n_counts, b.n_counts), (kw, t)
        # (fp16 probabilities enter the P.V product with 11 mantissa bits, rounded against each split's own running maximum)
        assert H.attn_rel_err(a.n_out, b.n_out) <= (1e-5 if w.dtype == "bf16" else 5e-4), (kw, t)
        assert np.abs(a.n_lse - b.n_lse).max() <= 1e-4, (kw, t)
    sa, _ = a.kvd.cache_export(0)
    sb, _ = b.kvd.cache_export(0)
    assert torch.equal(sa, sb), kw
    a.close()
    b.close()


@pytest.mark.parametrize("mb", [-1, 1], ids=["single-launch", "kernel-chain"])
@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_step_parity_scaled_configs(cfg, mb):
    """micro_batches=-1 runs the layer-step as one launch, 1 as a chain of separate kernels."""
    w = SCALED[cfg]
    rig = R.Rig(w, micro_batches=mb)
    units = all_units(rig)
    rep = R.run_steps(rig, units, w.steps, check_dir_every=3, progress=f"cfg{cfg}-scaled-mb{mb}")
    assert rep.unit_steps == w.steps * w.n_layers * w.units
    assert rep.tie_divergences <= 2
    if cfg == 1:
        assert rep.misses == 0                                       # the cache holds every page
    rig.close()


def test_micro_batches_and_per_unit_capacities_give_identical_results():
    w = SCALED[3].replace(batch=4, steps=5)
    rng = np.random.default_rng(5)
    caps = rng.integers(w.topk_pages, w.capacity + 1, size=w.n_layers * w.units).tolist()
    outs = []
    for mb in (-1, 1, 4):
        rig = R.Rig(w, capacity=caps, micro_batches=mb)
        units = all_units(rig) if mb == 4 else []
        trace = []
        for t, q in enumerate(W.query_stream(w, rig.q0, w.steps, R.DEV)):
            rig.step(0, t, q[0])
            rep = R.StepReport()
            for ou in units:
                R.compare_unit(rig, ou, t, q[0], rep)
            trace.append((rig.n_sel_pages.copy(), rig.n_hit_mask.copy(), np.sort(rig.n_evicted, axis=1),
                          rig.n_counts.copy(), rig.n_out.copy()))
        outs.append(trace)
        rig.close()
    # the two multi-kernel runs are the same kernels on the same units: bit-identical; the
    # single-launch step sums the tiles of a split in a different order, so its outputs agree to
    # fp32 rounding while selections and cache traces are identical
    for a, b in zip(outs[1], outs[2]):
        for x, y in zip(a, b):
            assert np.array_equal(x, y)
    for a, b in zip(outs[0], outs[1]):
        for x, y in zip(a[:4], b[:4]):
            assert np.array_equal(x, y)
        assert H.attn_rel_err(a[4], b[4]) <= 1e-5


# --------------------------------------------------------------------------- #
# growth of the store during decoding
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("kw,mb", [
    (dict(), 1),                                                      # bf16, page 16 (tile layout), chain of kernels
    (dict(), -1),                                                     # the same, one launch
    (dict(dtype="f16", page=32, ctx=32 * 120, n_q_heads=14, n_kv_heads=2), 1),
    (dict(page=20, ctx=20 * 90, n_q_heads=6, n_kv_heads=2), 1),      # natural slot layout
    (dict(page=8, ctx=8 * 200), -1),                                  # packed slot layout, one launch
    (dict(page=4, ctx=4 * 300, dtype="f16"), 1),                      # packed slot layout, chain of kernels
])
def test_append_kv_grows_store_index_and_slots(kw, mb):
    """Each decode step appends one token per sequence: host store, resident slot and index entry
    must follow, and the next steps must attend to the new tokens (the last pages are forced into
    the selection so that they are resident and attended)."""
    w = small("append", recent_pages=2, topk_pages=20, capacity=40, steps=30, **kw)
    P = w.page
    seq = [w.ctx - max(2 * P + 5, w.steps + 3), w.ctx - max(3 * P, w.steps + P)]   # room to grow, over page boundaries
    rig = R.Rig(w, seq_lens=seq, micro_batches=mb)
    units = all_units(rig)
    gen = torch.Generator(device="cpu").manual_seed(99)
    rep = R.StepReport()
    qs = W.query_stream(w, rig.q0, w.steps, R.DEV)
    for t in range(w.steps):
        q = next(qs)
        rig.step(0, t, q[0])
        for ou in units:
            R.compare_unit(rig, ou, t, q[0], rep)
        k_new = torch.randn((w.batch, w.n_kv_heads, w.head_dim), generator=gen).to(w.torch_dtype)
        v_new = torch.randn((w.batch, w.n_kv_heads, w.head_dim), generator=gen).to(w.torch_dtype)
        rig.kvd.append_kv(0, k_new.to(R.DEV), v_new.to(R.DEV))
        rig.kvd.advance()
        torch.cuda.synchronize()
        summ = rig.summaries.cpu()
        for ou in units:
            pos = ou.seq_len
            ou.keys[pos] = H.f64(k_new[ou.b, ou.h])                     # the oracle's copy of the store grows from the inputs
            ou.values[pos] = H.f64(v_new[ou.b, ou.h])
            ou.seq_len = pos + 1
            ou.summ = orc.page_summaries(ou.keys, P, ou.seq_len, ou.code)
            page, off = divmod(pos, P)
            assert torch.equal(rig.store[0, ou.b, ou.h, page, 0, off], k_new[ou.b, ou.h])
            assert torch.equal(rig.store[0, ou.b, ou.h, page, 1, off], v_new[ou.b, ou.h])
            n = ou.summ.shape[0]
            assert np.array_equal(H.bits(summ[0, ou.b, ou.h, :n]), orc.f64_to_bits(ou.summ, ou.code)), (t, ou.u)
        rig.seq_lens = [s + 1 for s in rig.seq_lens]
        if t % 7 == 0 or t == w.steps - 1:
            R.check_directory(rig, 0, units)                            # slots still equal their (grown) host pages
    assert rep.tie_divergences <= 2
    assert any((s0 + w.steps) // P > s0 // P for s0 in seq)              # a page boundary was crossed
    rig.close()


def test_append_kv_errors():
    w = small("append-err", ctx=16 * 40, topk_pages=8, capacity=16, batch=1)
    rig = R.Rig(w)                                                      # sequences already fill every page
    kv = torch.zeros((w.batch, w.n_kv_heads, w.head_dim), dtype=w.torch_dtype, device=R.DEV)
    with pytest.raises(K.KvdError) as e:
        rig.kvd.append_kv(0, kv, kv)
    assert e.value.status == K.ERR_SHAPE
    with pytest.raises(K.KvdError) as e:
        rig.kvd.advance()
    assert e.value.status == K.ERR_SHAPE
    rig.close()
    w2 = small("append-alias", n_layers=2, physical_layers=1, ctx=16 * 40, topk_pages=8, capacity=16, batch=1)
    rig = R.Rig(w2, seq_lens=[16 * 30])
    with pytest.raises(K.KvdError) as e:
        rig.kvd.append_kv(0, kv, kv)
    assert e.value.status == K.ERR_STATE                                # two layers share one stored layer
    rig.close()


@pytest.mark.parametrize("mb", [-1, 1, 2], ids=["single-launch", "kernel-chain", "two-groups"])
def test_step_replayed_from_a_hip_graph(mb):
    """kvd_step keeps no host-side state per call (the one launch's counters and published words
    return to zero by themselves; the groups fork and join with events only), so a captured step
    can be replayed: every replay must equal the eager step on the same inputs."""
    w = SCALED[3].replace(steps=8)
    eager, graphed = R.Rig(w, micro_batches=mb), R.Rig(w, micro_batches=mb)
    qs = [q[0].contiguous() for q in W.query_stream(w, eager.q0, 8, R.DEV)]
    for t in range(4):                                                # same history on both sides
        eager.step(0, t, qs[t])
        graphed.step(0, t, qs[t])
    q_static = qs[4].clone()
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        graphed.kvd.step(0, 4, q_static, graphed.out, graphed.lse, stream=s)
    torch.cuda.synchronize()
    # (capturing does not run the launch; the first replay is the first execution)
    for i, t in enumerate([4, 5, 6, 7]):
        q_static.copy_(qs[t])
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        graphed.kvd.step_trace(graphed.sel_pages, graphed.sel_slots, graphed.hit_mask, graphed.evicted, graphed.counts,
                               graphed.scores)
        torch.cuda.synchronize()
        eager.step(0, 4, qs[t])                                       # the captured launch carries step index 4
        assert torch.equal(graphed.sel_pages.cpu(), torch.from_numpy(eager.n_sel_pages)), i
        assert torch.equal(graphed.hit_mask.cpu(), torch.from_numpy(eager.n_hit_mask)), i
        assert torch.equal(graphed.counts.cpu(), torch.from_numpy(eager.n_counts)), i
        assert torch.equal(graphed.out.cpu(), torch.from_numpy(eager.n_out)), i
        assert (torch.zeros(3) + 1).sum().item() == 3.0               # unrelated eager work between replays
    assert graphed.kvd.stats().misses == eager.kvd.stats().misses
    eager.close()
    graphed.close()


@pytest.mark.parametrize("mb", [-1, 1], ids=["single-launch", "kernel-chain"])
def test_layers_in_flight_replayed_from_a_hip_graph(mb):
    """kvd_step_layers forks into and joins back from a stream of the library with events only, so
    the call can be captured from the caller's stream; every replay must equal the eager call."""
    w = small("layers-graph", n_layers=3, physical_layers=2, ctx=16 * 600, topk_pages=32, capacity=40, steps=8, batch=2)
    eager, graphed = R.Rig(w, micro_batches=mb), R.Rig(w, micro_batches=mb)
    qs = [q.contiguous() for q in W.query_stream(w, eager.q0, 8, R.DEV)]
    L = w.n_layers
    shape = (L, w.batch, w.n_q_heads, w.head_dim)
    out_e = torch.empty(shape, dtype=torch.float32, device=R.DEV)
    out_g = torch.empty(shape, dtype=torch.float32, device=R.DEV)
    for t in range(3):                                                # same history on both sides
        eager.kvd.step_layers(0, L, t, qs[t], out_e)
        graphed.kvd.step_layers(0, L, t, qs[t], out_g)
    torch.cuda.synchronize()
    q_static = qs[3].clone()
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        graphed.kvd.step_layers(0, L, 3, q_static, out_g, stream=s)
    torch.cuda.synchronize()
    for i, t in enumerate([3, 4, 5, 6, 7]):
        q_static.copy_(qs[t])
        out_g.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        eager.kvd.step_layers(0, L, 3, qs[t], out_e)                   # the captured launches carry step index 3
        torch.cuda.synchronize()
        if mb == 1:
            assert torch.equal(out_g, out_e), i
        else:
            assert H.attn_rel_err(out_g.cpu().numpy().reshape(-1, w.head_dim), out_e.cpu().numpy().reshape(-1, w.head_dim)) <= 1e-5, i
        for l in range(L):
            pa, sa = eager.kvd.cache_export(l)
            pb, sb = graphed.kvd.cache_export(l)
            assert torch.equal(pa, pb) and torch.equal(sa, sb), (i, l)
        assert (torch.zeros(3) + 1).sum().item() == 3.0               # unrelated eager work between replays
    se, sg = eager.kvd.stats(), graphed.kvd.stats()
    assert sg.misses == se.misses and se.misses > 0
    eager.close()
    graphed.close()


def test_calibration_picks_a_form_and_leaves_the_cache_consistent():
    """The pre-run calibration replays the same real steps in every form, each time from the cache
    as it was at the call; afterwards the cache must be exactly where the oracle is after taking
    those steps once, and decoding continues in the chosen form."""
    w = SCALED[3].replace(batch=4, steps=4)
    rig = R.Rig(w)
    units = all_units(rig)
    n_q, spf, t0 = 5, 6, 3
    qs = torch.stack([q[0] for q in W.query_stream(w, rig.q0, t0 + n_q + 2, R.DEV)]).contiguous()
    rep = R.StepReport()
    for t in range(t0):                                               # the calibration starts from a cache in use
        rig.step(0, t, qs[t])
        for ou in units:
            R.compare_unit(rig, ou, t, qs[t], rep)
    rig.kvd.reset_stats()
    q_cal = qs[t0:t0 + n_q]
    chosen, ms = rig.kvd.calibrate_step_form(0, t0, q_cal, spf, rig.out)
    assert set(ms) == {1, 2, 4, -1} and all(v > 0 for v in ms.values())
    assert chosen == min(ms, key=ms.get) and rig.kvd.step_form() == chosen
    n_run = spf + 1                                                   # every form replays the same 1 untimed + spf timed steps
    want_miss = 0
    for i in range(n_run):                                            # the oracle takes them once
        for ou in units:
            want_miss += len(ou.step(t0 + i, q_cal[i % n_q])["misses"])
    R.check_directory(rig, 0, units)
    st = rig.kvd.stats()
    assert st.misses == 2 * len(ms) * want_miss and want_miss > 0     # every replay saw the same misses
    for j in range(2):                                                # and decoding goes on from there
        rig.step(0, t0 + n_run + j, qs[t0 + n_q + j])
        for ou in units:
            R.compare_unit(rig, ou, t0 + n_run + j, qs[t0 + n_q + j], rep)
    for form in (1, 2, -1):
        rig.kvd.set_step_form(form)
        assert rig.kvd.step_form() == form
    rig.kvd.set_profiling(1)
    with pytest.raises(K.KvdError):                                   # profiled steps all run as one chain: nothing to compare
        rig.kvd.calibrate_step_form(0, 100, q_cal, 2, rig.out)
    rig.kvd.set_profiling(0)
    with pytest.raises(K.KvdError):
        rig.kvd.set_step_form(99)
    rig.close()


def test_one_launch_step_with_more_chunks_per_scoring_workgroup_than_it_counts_in_lds():
    """The waves of a scoring workgroup count a chunk's arrivals in LDS for the workgroup's first
    32 chunks and report later chunks wave by wave; with one or two scoring workgroups for 80
    chunks both ways are taken in one launch, and the selection must see the same totals."""
    w = SCALED[2].replace(n_layers=1, physical_layers=1, batch=5, steps=3)
    rig = R.Rig(w, micro_batches=-1)
    assert rig.kvd.step_form() == -1
    units = all_units(rig)
    qs = [q[0] for q in W.query_stream(w, rig.q0, 8, R.DEV)]
    rep = R.StepReport()
    t = 0
    for shape in [(1, 1, 1, 1), (1, 2, 0, 1), (2, 1, 0, 2), (0, 0, 0, 0)]:
        rig.kvd.set_step_shape(*shape)
        rig.step(0, t, qs[t])
        for ou in units:
            R.compare_unit(rig, ou, t, qs[t], rep)
        t += 1
    assert rep.unit_steps == 4 * w.units and rep.tie_divergences <= 2
    rig.close()


@pytest.mark.parametrize("cfg", [2, 5])
def test_one_launch_step_in_every_launch_shape_and_after_its_calibration(cfg):
    """The launch shape of the one-launch step (passes per scoring chunk, scoring workgroups,
    attention splits) decides only how the units' stages overlap: results must match the oracle
    in every shape, and the calibration must leave the cache where one step of its query takes it."""
    w = SCALED[cfg].replace(steps=4)
    rig = R.Rig(w, micro_batches=-1)
    assert rig.kvd.step_form() == -1
    units = all_units(rig, layers=[0])
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    p0, n0, s0, g0 = rig.kvd.step_shape()
    assert 1 <= p0 <= 8 and 1 <= n0 <= cus and s0 >= 1 and g0 == 1
    qs = [q[0] for q in W.query_stream(w, rig.q0, 20, R.DEV)]
    rep = R.StepReport()
    t = 0
    shapes = [(1, 1, 1, 1), (3, 5, s0, 2), (2, cus, 2 * s0, 1), (8, 40, max(1, s0 // 2), 4), (1, 3, 0, 3), (0, 0, 0, 8), (0, 0, 0, 0)]
    for shape in shapes:
        rig.kvd.set_step_shape(*shape)
        got = rig.kvd.step_shape()
        assert (shape[0] == 0 or got[0] == shape[0]) and (shape[2] == 0 or got[2] == shape[2])
        assert shape[1] == 0 or 1 <= got[1] <= shape[1]               # (scoring workgroups are capped at the number of chunks)
        assert shape[3] == 0 or 1 <= got[3] <= min(shape[3], w.units)  # (no empty group)
        for _ in range(2):
            rig.step(0, t, qs[t])
            for ou in units:
                R.compare_unit(rig, ou, t, qs[t], rep)
            t += 1
    assert rig.kvd.step_shape() == (p0, n0, s0, g0)
    for bad in [(9, 0, 0, 0), (0, cus + 1, 0, 0), (0, 0, 2 * s0 + 1, 0), (-1, 0, 0, 0), (0, 0, 0, 9)]:
        with pytest.raises(K.KvdError) as e:
            rig.kvd.set_step_shape(*bad)
        assert e.value.status == K.ERR_SHAPE
    # calibration: one real step of the query, then all-hit replays in a grid of shapes
    chosen, us, us_rule = rig.kvd.calibrate_step_shape(0, t, qs[t], rig.out, launches_per_shape=4)
    assert rig.kvd.step_shape() == chosen and 0 < us <= us_rule * 1.000001
    for ou in units:                                                  # the oracle takes that step once
        ou.step(t, qs[t])
    R.check_directory(rig, 0, units)
    t += 1
    for _ in range(2):
        rig.step(0, t, qs[t])
        for ou in units:
            R.compare_unit(rig, ou, t, qs[t], rep)
        t += 1
    print(f"cfg{cfg}-scaled: rule {(p0, n0, s0)} {us_rule:.1f} us, chosen {chosen} {us:.1f} us")
    rig.kvd.set_step_form(1)
    with pytest.raises(K.KvdError) as e:                              # nothing to shape in a chain of kernels
        rig.kvd.calibrate_step_shape(0, t, qs[t], rig.out)
    assert e.value.status == K.ERR_STATE
    rig.close()


def test_single_launch_timeline_and_wait_limit():
    """The one-launch step records one line per workgroup, in dispatch order and with consistent
    clocks; a wait limit of zero makes waiting workgroups give up (every kernel still ends
    normally), which the library reports until the cache is reset."""
    w = SCALED[3].replace(steps=4)
    rig = R.Rig(w, micro_batches=-1)
    units = all_units(rig)
    qs = [q[0] for q in W.query_stream(w, rig.q0, 4, R.DEV)]
    rig.kvd.set_profiling(2)
    rep = R.StepReport()
    for t in range(2):
        rig.step(0, t, qs[t])
        for ou in units:
            R.compare_unit(rig, ou, t, qs[t], rep)
    rec = rig.kvd.step_timeline().numpy()
    role, unit = rec[:, 4] & 0xff, (rec[:, 4] >> 8) & 0xffffff
    assert (role == 1).sum() == w.units and (role == 2).sum() % w.units == 0 and (role == 0).sum() >= 1
    assert set(unit[role != 0].tolist()) == set(range(w.units))
    t = rec[:, :4]
    assert np.all(np.diff(t, axis=1) >= 0)                           # start <= ready <= done <= exit
    first_score = t[role == 0, 0].min()
    for u in range(w.units):                                          # a unit's stages follow one another:
        sel = t[(role == 1) & (unit == u)][0]                         # a split has its entries after the unit's scores
        att = t[(role == 2) & (unit == u)]                            # were there (hits are published before the
        assert sel[1] >= first_score and att[:, 1].min() >= sel[1]    # selection workgroup is done), and the unit's
        assert att[:, 2].max() >= sel[2]                              # output after its last missed page was fetched
    rig.kvd.set_profiling(0)

    rig.kvd.set_wait_limit_us(0)
    rig.kvd.step(0, 2, qs[2], rig.out, rig.lse)                       # workgroups that have to wait give up
    torch.cuda.synchronize()
    with pytest.raises(K.KvdError) as e:
        rig.kvd.stats()
    assert e.value.status == K.ERR_STATE
    with pytest.raises(K.KvdError) as e:                              # the failed step has no trace either
        rig.kvd.step_trace(rig.sel_pages)
    assert e.value.status == K.ERR_STATE
    # the next step call reports the failure once; the library has then emptied the windows and
    # taken the chain of kernels, and goes on by itself
    assert rig.kvd.step_form() == -1
    with pytest.raises(K.KvdError) as e:
        rig.kvd.step(0, 3, qs[3], rig.out, rig.lse)
    assert e.value.status == K.ERR_STATE
    assert rig.kvd.step_form() == 1
    rig.kvd.stats()
    units = all_units(rig)                                            # cold again on both sides
    rep = R.StepReport()
    for t in range(2):
        rig.step(0, t, qs[t])
        for ou in units:
            R.compare_unit(rig, ou, t, qs[t], rep)
    R.check_directory(rig, 0, units)
    # back to the one launch with its waits in order, through kvd_cache_reset as well
    rig.kvd.set_wait_limit_us(2_000_000)
    rig.kvd.set_step_form(-1)
    rig.kvd.cache_reset()
    units = all_units(rig)
    for t in range(2):
        rig.step(0, t, qs[t])
        for ou in units:
            R.compare_unit(rig, ou, t, qs[t], rep)
    rig.close()


# --------------------------------------------------------------------------- #
# lookahead eviction
# --------------------------------------------------------------------------- #
def _tight(cfg):
    """A scaled configuration whose window is small enough to evict at nearly every step."""
    w = SCALED[cfg]
    return w.replace(policy="lookahead", capacity=w.topk_pages + w.topk_pages // 6, steps=w.steps + 6)


@pytest.mark.parametrize("mb", [-1, 1, 2], ids=["single-launch", "kernel-chain", "two-groups"])
@pytest.mark.parametrize("cfg", [2, 3, 5])
def test_lookahead_step_parity(cfg, mb):
    w = _tight(cfg)
    rig = R.Rig(w, micro_batches=mb)
    units = all_units(rig)
    rep = R.run_steps(rig, units, w.steps, check_dir_every=3, progress=f"cfg{cfg}-lookahead-mb{mb}")
    assert rep.unit_steps == w.steps * w.n_layers * w.units
    assert rep.tie_divergences <= 2 and rep.victim_tie_divergences <= 2
    st = rig.kvd.stats()
    assert st.evictions > w.n_layers * w.units                          # the policy was exercised
    rig.close()


@pytest.mark.parametrize("mb", [-1, 1], ids=["single-launch", "kernel-chain"])
@pytest.mark.parametrize("cfg,pool", [(2, 40), (3, 60), (3, 48), (3, 400), (5, 30)])
def test_lookahead_with_a_finite_pool_step_parity(cfg, pool, mb):
    """Lookahead eviction with a finite look-ahead candidate pool: 1.25 x the budget as in the
    paper's evaluation (cfg2: 32 pages -> 40, cfg3: 48 -> 60, cfg5: 24 -> 30 with forced recent pages),
    a pool that is exactly the selection (cfg3, 48: LRU order throughout) and one that covers a third
    of the pages (400: pool pages must leave too)."""
    w = _tight(cfg).replace(lookahead_pool=pool)
    rig = R.Rig(w, micro_batches=mb)
    units = all_units(rig)
    rep = R.run_steps(rig, units, w.steps, check_dir_every=3, progress=f"cfg{cfg}-pool{pool}-mb{mb}")
    assert rep.unit_steps == w.steps * w.n_layers * w.units
    assert rep.tie_divergences <= 2 and rep.victim_tie_divergences <= 2
    assert rig.kvd.stats().evictions > w.n_layers * w.units
    rig.close()


def test_lookahead_pool_equal_to_the_selection_is_lru():
    """With M = k and no forced pages every unselected resident page is outside the pool: the GPU's
    trace must then be the LRU trace, step by step."""
    w = _tight(3)
    a = R.Rig(w.replace(lookahead_pool=w.topk_pages), micro_batches=-1)
    b = R.Rig(w.replace(policy="lru"), micro_batches=-1, build_index=False)
    b.summaries.copy_(a.summaries)
    for t, q in enumerate(W.query_stream(w, a.q0, w.steps, R.DEV)):
        a.step(0, t, q[0])
        b.step(0, t, q[0])
        assert np.array_equal(a.n_sel_pages, b.n_sel_pages) and np.array_equal(a.n_hit_mask, b.n_hit_mask), t
        assert np.array_equal(np.sort(a.n_evicted, axis=1), np.sort(b.n_evicted, axis=1)), t
    assert a.kvd.stats().evictions > 0
    pa, sa = a.kvd.cache_export(0)
    pb, sb = b.kvd.cache_export(0)
    assert torch.equal(pa, pb) and torch.equal(sa, sb)
    a.close()
    b.close()


@pytest.mark.parametrize("pool", [0, 60])
def test_lookahead_size_agnostic_kernels_and_separate_entry_points(pool, monkeypatch):
    """The same policy through the size-agnostic resolve kernel, driven stage by stage:
    kvd_score_select leaves the scores that kvd_cache_resolve ranks the victims by."""
    monkeypatch.setenv("KVD_GENERIC_SELECT", "1")
    w = _tight(3).replace(lookahead_pool=pool)
    rig = R.Rig(w)
    units = all_units(rig)
    rep = R.StepReport()
    for t, q in enumerate(W.query_stream(w, rig.q0, w.steps, R.DEV)):
        rig.kvd.score_select(0, q[0], rig.sel_pages, rig.scores)
        rig.kvd.cache_resolve(0, t, rig.sel_pages, rig.sel_slots, rig.hit_mask, rig.evicted, rig.counts, do_gather=True)
        rig.kvd.sparse_decode_attn(0, q[0], rig.sel_pages, rig.sel_slots, rig.out, rig.lse)
        torch.cuda.synchronize()
        rig.n_sel_pages, rig.n_sel_slots = rig.sel_pages.cpu().numpy(), rig.sel_slots.cpu().numpy()
        rig.n_hit_mask, rig.n_evicted = rig.hit_mask.cpu().numpy(), rig.evicted.cpu().numpy()
        rig.n_counts, rig.n_scores = rig.counts.cpu().numpy(), rig.scores.cpu().numpy()
        rig.n_out, rig.n_lse = rig.out.cpu().numpy(), rig.lse.cpu().numpy()
        for ou in units:
            R.compare_unit(rig, ou, t, q[0], rep)
    R.check_directory(rig, 0, units)
    assert rep.tie_divergences <= 2 and rep.victim_tie_divergences <= 2
    assert rig.kvd.stats().evictions > 0
    rig.close()


def test_lookahead_exact_ties_drop_the_higher_page():
    """Pages with identical summary rows score bit-identically on both sides, so among them only
    the tie rule decides who leaves: GPU and oracle must agree without any tolerance."""
    w = small("la-ties", ctx=16 * 200, topk_pages=16, capacity=24, heavy_count=0, policy="lookahead", steps=10)
    rig = R.Rig(w, build_index=False)
    g = torch.Generator(device=R.DEV)
    g.manual_seed(770_011)                                            # (own generator: the outcome must not depend on what ran before)
    base = torch.randn(w.units, 24, w.head_dim, device=R.DEV, generator=g)
    idx = torch.randint(0, 24, (w.units, w.n_pages), device=R.DEV, generator=g)
    summ = torch.gather(base, 1, idx[:, :, None].expand(-1, -1, w.head_dim)).to(w.torch_dtype)
    rig.summaries.copy_(summ.view(rig.summaries.shape))
    units = all_units(rig)
    for ou in units:                                                  # the oracle scores the same index
        ou.summ = H.f64(rig.summaries[0, ou.b, ou.h])
    rep = R.run_steps(rig, units, w.steps)
    assert rep.tie_divergences == 0 and rep.victim_tie_divergences == 0
    assert rig.kvd.stats().evictions > 0
    rig.close()


# --------------------------------------------------------------------------- #
# hierarchical index
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("cfg,mb,kw", [
    (3, 1, dict()),                                                   # 1100 pages -> 550 centroids, bf16
    (3, 2, dict()),                                                   # groups on streams
    (2, 1, dict(index_iterations=2)),                                 # 3 layers, planted heavy pages
    (4, 1, dict()),                                                   # fp16, G = 7, page 32
    (5, 1, dict()),                                                   # page 64, recent pages forced and pre-warmed
    (3, -1, dict()),                                                  # the same through the one-launch step
    (4, -1, dict()),
    (5, -1, dict()),
    (2, -1, dict(index_iterations=2)),
])
def test_hierarchical_index_build_and_step_parity(cfg, mb, kw):
    """k-means build (assignments of every round, centroids, cluster lists) and decode steps whose
    selection goes through the centroids, against the oracle."""
    w = SCALED[cfg]
    w = w.replace(**{**dict(index_centroids=w.n_pages // 2, index_iterations=3), **kw})
    rig = R.Rig(w, micro_batches=mb)
    assert (rig.kvd.step_form() == -1) == (mb == -1)
    units = all_units(rig)                                            # builds and checks the index of every unit
    assert sum(ou.kmeans_divergences for ou in units) <= 4
    rep = R.run_steps(rig, units, w.steps, check_dir_every=3, progress=f"cfg{cfg}-hier-mb{mb}")
    assert rep.unit_steps == w.steps * w.n_layers * w.units
    assert rep.tie_divergences <= 2
    rig.close()


@pytest.mark.parametrize("cfg,mb,generic,pool", [(3, 1, False, 0), (3, 2, False, 0), (5, 1, False, 0), (2, 1, True, 0), (3, -1, False, 0),
                                                 (5, -1, False, 0), (2, -1, False, 0), (3, -1, False, 60), (2, 1, True, 40),
                                                 (5, 1, False, 30)])
def test_lookahead_eviction_under_the_hierarchical_index(cfg, mb, generic, pool, monkeypatch):
    """The paper's own combination: selection through the centroids, victims by the lowest
    current-step score — here the score of the page's cluster.  Small windows, so that nearly every
    step evicts; pages of one cluster tie exactly and leave higher page first."""
    if generic:
        monkeypatch.setenv("KVD_GENERIC_SELECT", "1")
    w = _tight(cfg)
    w = w.replace(index_centroids=w.n_pages // 4, index_iterations=2, lookahead_pool=pool)   # (pool > 0: a finite look-ahead pool, ranked by cluster score)
    rig = R.Rig(w, micro_batches=mb)
    units = all_units(rig)
    rep = R.run_steps(rig, units, w.steps, check_dir_every=3, progress=f"cfg{cfg}-hier-lookahead-mb{mb}")
    assert rep.unit_steps == w.steps * w.n_layers * w.units
    assert rep.tie_divergences <= 2 and rep.victim_tie_divergences <= 4
    assert rig.kvd.stats().evictions > w.n_layers * w.units
    rig.close()


def test_lookahead_with_cluster_lists_written_by_the_caller():
    """The caller plants its own index (runs of 5 neighbouring pages, centroid = the run's first
    summary; the last pages in no cluster at all) and announces it with kvd_refresh_clusters; the
    lookahead victims must follow the planted clusters' scores, and a resident page of no cluster
    must be the first to leave."""
    w = small("hier-planted", ctx=16 * 203, topk_pages=20, capacity=26, heavy_count=0, policy="lookahead",
              index_centroids=40, steps=8)
    rig = R.Rig(w, build_index=False)
    rig.kvd.build_summaries(0)
    torch.cuda.synchronize()
    NP, Nc, U = w.n_pages, w.index_centroids, w.units
    runs = [list(range(5 * c, 5 * c + 5)) for c in range(Nc)]                    # pages 200..202 belong to no cluster
    start = torch.tensor([5 * c for c in range(Nc + 1)], dtype=torch.int32)
    pages = torch.full((NP,), -1, dtype=torch.int32)
    pages[:5 * Nc] = torch.arange(5 * Nc, dtype=torch.int32)
    rig.cluster_start[0].copy_(start.repeat(U, 1))
    rig.cluster_pages[0].copy_(pages.repeat(U, 1))
    rig.centroids[0].copy_(rig.summaries[0][:, :, 0:5 * Nc:5, :])
    rig.kvd.refresh_clusters(0)
    # pages 200 and 201 start out resident: they can only leave as victims
    rig.kvd.cache_warm(0, [200, 201] * U, [2] * U)
    units = []
    for b in range(w.batch):
        for h in range(w.n_kv_heads):
            ou = R.OracleUnit.__new__(R.OracleUnit)
            rig.hier = False                                                      # (no k-means to follow)
            R.OracleUnit.__init__(ou, rig, 0, b, h)
            rig.hier = True
            ou.centroids = ou.summ[0:5 * Nc:5]
            ou.members = [np.array(r, dtype=np.int32) for r in runs]
            ou.window.warm([200, 201], stamp=-1)
            units.append(ou)
    rep = R.StepReport()
    gone = {ou.u: set() for ou in units}
    for t, q in enumerate(W.query_stream(w, rig.q0, w.steps, R.DEV)):
        rig.step(0, t, q[0])
        for ou in units:
            gone[ou.u] |= set(R.compare_unit(rig, ou, t, q[0], rep)["evicted"])
            # the clusterless pages go first: 201 with the first victim, 200 with the second
            assert len(gone[ou.u]) < 1 or 201 in gone[ou.u]
            assert len(gone[ou.u]) < 2 or 200 in gone[ou.u]
    assert all(len(g) >= 2 for g in gone.values())
    assert rep.tie_divergences <= 2 and rig.kvd.stats().evictions > 0
    R.check_directory(rig, 0, units)
    rig.close()


@pytest.mark.parametrize("mb", [-1, 1], ids=["single-launch", "kernel-chain"])
def test_hierarchical_exact_ties_go_to_the_lower_cluster(mb):
    """Every centroid is the same vector, so all clusters score exactly alike in every step: the
    clusters must then be taken in ascending cluster order.  Cluster c holds the run of pages
    5 (Nc - 1 - c) .. +4, so that cluster order is the reverse of page order and the two cannot be
    mistaken for each other; k = 22 ends inside the fifth cluster, which gives its two lowest pages."""
    w = small("hier-ties", ctx=16 * 200, topk_pages=22, capacity=40, heavy_count=0, index_centroids=40, steps=4)
    rig = R.Rig(w, micro_batches=mb, build_index=False)
    rig.kvd.build_summaries(0)
    torch.cuda.synchronize()
    NP, Nc, U = w.n_pages, w.index_centroids, w.units
    runs = [list(range(5 * (Nc - 1 - c), 5 * (Nc - 1 - c) + 5)) for c in range(Nc)]
    start = torch.tensor([5 * c for c in range(Nc + 1)], dtype=torch.int32)
    pages = torch.tensor([p for r in runs for p in r], dtype=torch.int32)
    rig.cluster_start[0].copy_(start.repeat(U, 1))
    rig.cluster_pages[0].copy_(pages.repeat(U, 1))
    rig.centroids[0].copy_(rig.summaries[0][:, :, 7:8, :].expand(-1, -1, Nc, -1))
    rig.kvd.refresh_clusters(0)
    units = []
    for b in range(w.batch):
        for h in range(w.n_kv_heads):
            ou = R.OracleUnit.__new__(R.OracleUnit)
            rig.hier = False                                                      # (no k-means to follow)
            R.OracleUnit.__init__(ou, rig, 0, b, h)
            rig.hier = True
            ou.centroids = np.repeat(ou.summ[7:8], Nc, axis=0)
            ou.members = [np.array(r, dtype=np.int32) for r in runs]
            units.append(ou)
    want = sorted(p for r in runs[:4] for p in r) + runs[4][:2]
    rep = R.StepReport()
    for t, q in enumerate(W.query_stream(w, rig.q0, w.steps, R.DEV)):
        rig.step(0, t, q[0])
        for ou in units:
            R.compare_unit(rig, ou, t, q[0], rep)
            assert rig.n_sel_pages[ou.u].tolist() == sorted(want), (t, ou.u)
    assert rep.tie_divergences == 0
    rig.close()


def test_layout_from_clusters_matches_the_oracle_with_pages_of_no_cluster():
    """Cluster lists written by the caller, clusters of scattered pages in no particular order and
    seven pages listed nowhere: the file layout derived from them must be the oracle's (clusters
    one after another in cluster order, the unlisted pages last in page order); lists that name a
    page twice are refused."""
    w = small("layout", ctx=16 * 120, topk_pages=10, capacity=20, index_centroids=9, steps=1)
    rig = R.Rig(w, build_index=False)
    NP, Nc, U = w.n_pages, w.index_centroids, w.units
    rng = np.random.default_rng(4711)
    want = []
    for u in range(U):
        listed = rng.permutation(NP)[: NP - 7]
        cluster_of = rng.integers(0, Nc, size=len(listed))
        members = [np.sort(listed[cluster_of == c]).astype(np.int32) for c in range(Nc)]
        start = np.concatenate([[0], np.cumsum([len(m) for m in members])]).astype(np.int32)
        pages = np.full(NP, -1, dtype=np.int32)
        pages[: start[-1]] = np.concatenate(members)
        rig.cluster_start[0, u].copy_(torch.from_numpy(start))
        rig.cluster_pages[0, u].copy_(torch.from_numpy(pages))
        want.append(orc.extent_positions(NP, members))
    rig.kvd.refresh_clusters(0)
    torch.cuda.synchronize()
    got = rig.kvd.layout_from_clusters(0).numpy()
    assert np.array_equal(got, np.stack(want))
    assert any(not np.array_equal(wu, np.arange(NP)) for wu in want)
    bad = rig.cluster_pages[0, 0].clone()
    bad[1] = bad[0]                                                    # one page named twice
    rig.cluster_pages[0, 0].copy_(bad)
    with pytest.raises(K.KvdError):
        rig.kvd.layout_from_clusters(0)
    rig.close()


def test_hierarchical_index_ragged_forced_and_duplicate_pages():
    """Sequences of different lengths (the index covers the valid pages only), sink and recent
    pages, more centroids than distinct summaries (exact distance ties, empty clusters), and the
    stage-by-stage entry points."""
    w = small("hier-edge", ctx=16 * 200, topk_pages=24, capacity=40, sink_pages=2, recent_pages=3, heavy_count=0,
              index_centroids=64, index_iterations=3, steps=5)
    rig = R.Rig(w, seq_lens=[w.ctx - 7, w.ctx - 16 * 90 - 3], build_index=False)
    g = torch.Generator(device=R.DEV)
    g.manual_seed(770_012)
    base = torch.randn(w.units, 20, w.head_dim, device=R.DEV, generator=g)        # 20 distinct rows < 64 centroids
    idx = torch.randint(0, 20, (w.units, w.n_pages), device=R.DEV, generator=g)
    summ = torch.gather(base, 1, idx[:, :, None].expand(-1, -1, w.head_dim)).to(w.torch_dtype)
    rig.summaries.copy_(summ.view(rig.summaries.shape))
    rig.kvd.build_centroids(0, w.index_iterations, rig.assign_trace[0])
    torch.cuda.synchronize()
    rig.n_assign_trace = rig.assign_trace.cpu().numpy()
    units = []
    for b in range(w.batch):
        for h in range(w.n_kv_heads):
            ou = R.OracleUnit.__new__(R.OracleUnit)                                # the oracle indexes the same summaries
            R.OracleUnit.__init__(ou, rig, 0, b, h, summaries=H.f64(rig.summaries[0, b, h]))
            units.append(ou)
    assert all(ou.kmeans_divergences == 0 for ou in units)                        # exact ties resolve identically
    assert any(len(m) == 0 for ou in units for m in ou.members)                   # some clusters are empty
    rep = R.StepReport()
    for t, q in enumerate(W.query_stream(w, rig.q0, w.steps, R.DEV)):
        rig.kvd.score_select(0, q[0], rig.sel_pages, rig.scores)
        rig.kvd.cache_resolve(0, t, rig.sel_pages, rig.sel_slots, rig.hit_mask, rig.evicted, rig.counts, do_gather=True)
        rig.kvd.sparse_decode_attn(0, q[0], rig.sel_pages, rig.sel_slots, rig.out, rig.lse)
        torch.cuda.synchronize()
        rig.n_sel_pages, rig.n_sel_slots = rig.sel_pages.cpu().numpy(), rig.sel_slots.cpu().numpy()
        rig.n_hit_mask, rig.n_evicted = rig.hit_mask.cpu().numpy(), rig.evicted.cpu().numpy()
        rig.n_counts = rig.counts.cpu().numpy()
        rig.n_scores = rig.scores.cpu().numpy().reshape(-1)[: w.units * 64].reshape(w.units, 64)
        rig.n_out, rig.n_lse = rig.out.cpu().numpy(), rig.lse.cpu().numpy()
        for ou in units:
            R.compare_unit(rig, ou, t, q[0], rep)
    assert rep.tie_divergences == 0
    rig.close()


def test_hierarchical_index_argument_errors():
    common = dict(n_layers=1, batch=1, n_q_heads=4, n_kv_heads=1, page_size=16, max_pages=64, topk_pages=4, capacity_max=8,
                  kv_dtype=torch.float16)
    with pytest.raises(K.KvdError) as e:
        K.Kvd(index_centroids=65, **common)                           # more centroids than pages
    assert e.value.status == K.ERR_SHAPE
    k = K.Kvd(index_centroids=16, **common)
    with pytest.raises(K.KvdError) as e:
        k.build_centroids(0, 3)                                       # nothing bound yet
    assert e.value.status == K.ERR_STATE
    with pytest.raises(K.KvdError) as e:
        k.refresh_clusters(0)
    assert e.value.status == K.ERR_STATE
    k.close()
    k = K.Kvd(**common)
    t = torch.zeros(64, dtype=torch.int32, device=R.DEV)
    with pytest.raises(K.KvdError) as e:
        k.bind_centroids(t, t, t)                                     # flat index: no centroids to bind
    assert e.value.status == K.ERR_STATE
    k.close()


@pytest.mark.parametrize("cfg", [2, 5])
def test_size_agnostic_select_resolve_kernels(cfg, monkeypatch):
    """The register-resident fused kernel covers up to 16384 pages and 4096 slots per unit; larger
    units take separate select / resolve / fetch kernels.  Force that path on a small workload."""
    monkeypatch.setenv("KVD_GENERIC_SELECT", "1")
    w = SCALED[cfg]
    rig = R.Rig(w)
    units = all_units(rig)
    rep = R.run_steps(rig, units, w.steps, check_dir_every=2, progress=f"cfg{cfg}-generic")
    assert rep.unit_steps == w.steps * w.n_layers * w.units
    assert rep.tie_divergences <= 2
    rig.close()


@pytest.mark.parametrize("generic", [False, True], ids=["fused", "size-agnostic"])
@pytest.mark.parametrize("policy", ["lru", "lookahead"])
def test_degenerate_victim_keys_take_the_radix_fallback(policy, generic, monkeypatch):
    """Three thousand resident pages that all look alike to the victim choice — warmed long ago
    (LRU: one age class) or all scoring exactly zero (lookahead: a zero query) — fall into one
    histogram bucket of more than 1024 candidates, so the choice must fall back to radix
    refinement and still take the lowest pages (LRU) or the highest (lookahead) first."""
    if generic:
        monkeypatch.setenv("KVD_GENERIC_SELECT", "1")
    w = small("degen-victims", ctx=16 * 4000, topk_pages=64, capacity=3000, heavy_count=0, batch=1, n_kv_heads=2,
              n_q_heads=4, policy=policy, steps=1)
    rig = R.Rig(w, build_index=(policy == "lookahead"))
    warm = list(range(1000, 4000))
    rig.kvd.cache_warm(0, warm * w.units, [len(warm)] * w.units)
    units = all_units(rig)
    for ou in units:
        ou.window.warm(warm, stamp=-1)
    rep = R.StepReport()
    if policy == "lookahead":
        zero = torch.zeros((w.batch, w.n_q_heads, w.head_dim), dtype=w.torch_dtype, device=R.DEV)
        rig.step(0, 100, zero)                                        # every score 0: pages 0..63 selected, all of them misses
        for ou in units:
            want = R.compare_unit(rig, ou, 100, zero, rep)
            assert want["misses"] == list(range(64)) and want["evicted"] == list(range(3936, 4000))
    else:
        sel = np.tile(np.arange(64, dtype=np.int32), (w.units, 1))
        rig.sel_pages.copy_(torch.from_numpy(sel))
        rig.kvd.cache_resolve(0, 100, rig.sel_pages, rig.sel_slots, rig.hit_mask, rig.evicted, rig.counts, do_gather=True)
        torch.cuda.synchronize()
        ev = rig.evicted.cpu().numpy()
        for ou in units:
            hits, misses, evicted = ou.window.resolve(sel[ou.u], 100)
            assert (hits, misses, evicted) == ([], list(range(64)), list(range(1000, 1064)))
            assert sorted(ev[ou.u][ev[ou.u] >= 0].tolist()) == evicted
            assert rig.counts.cpu().numpy()[ou.u].tolist() == [0, 64, 64]
    assert rep.victim_tie_divergences == 0
    R.check_directory(rig, 0, units)
    rig.close()


def test_degenerate_scores_take_the_radix_fallback():
    """More than 1024 pages with exactly the same score land in one histogram bucket: the fused
    kernel must fall back to radix refinement and still pick the lowest pages among the ties."""
    w = small("degen", ctx=16 * 3000, topk_pages=40, capacity=64, heavy_count=0, batch=1, n_kv_heads=2, n_q_heads=4)
    rig = R.Rig(w, build_index=False)
    q = next(W.query_stream(w, rig.q0, 1, R.DEV))
    # three distinct summary rows: 20 pages of a clearly best row, 2000 pages of a middle row, the rest worst
    qbar = q[0].float().reshape(w.batch, w.n_kv_heads, w.group, w.head_dim).mean(dim=2)        # [B, Hkv, D]
    summ = torch.zeros(w.units, w.n_pages, w.head_dim, device=R.DEV)
    unit_q = qbar.reshape(w.units, w.head_dim)
    best = torch.arange(100, 120, device=R.DEV)
    mid = torch.arange(500, 2500, device=R.DEV)
    summ[:, :, :] = (-unit_q / unit_q.norm(dim=-1, keepdim=True))[:, None, :]
    summ[:, mid, :] = 0.0
    summ[:, best, :] = (unit_q / unit_q.norm(dim=-1, keepdim=True))[:, None, :]
    rig.summaries.copy_(summ.to(w.torch_dtype).view(rig.summaries.shape))
    rig.kvd.score_select(0, q[0], rig.sel_pages, rig.scores)
    torch.cuda.synchronize()
    sel = rig.sel_pages.cpu().numpy()
    want = np.concatenate([np.arange(100, 120), np.arange(500, 520)])
    for u in range(w.units):
        assert np.array_equal(sel[u], want), u
    # and the whole step on it agrees with the oracle
    s64 = H.f64(rig.summaries.view(w.units, w.n_pages, w.head_dim))
    for u in range(w.units):
        b, h = divmod(u, w.n_kv_heads)
        qg = H.f64(q[0][b, h * w.group:(h + 1) * w.group])
        sc = orc.page_scores(orc.pooled_query(qg), s64[u], 1.0 / math.sqrt(w.head_dim))
        assert np.array_equal(orc.select_pages(sc, w.topk_pages), want)
    rig.close()
