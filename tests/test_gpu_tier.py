"""The decode step with the third tier behind the GPU window (backing file -> pool of extents in
pinned host memory -> slots), through the C ABI, against the oracle: outputs and cache traces as for
the plain step, and the tier's own trace (extents needed / hit / read / evicted, read runs) bit for
bit against the oracle's extent pool fed with the oracle's misses."""
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
    from tests.test_gpu_parity import SCALED, all_units, small


def run_tiered(rig, units, steps, otier, opos, progress=""):
    """Every unit of every layer has an oracle mirror; after each layer-step the tier's trace must
    equal what the oracle's extent pool does with the oracle's miss sets."""
    w = rig.w
    rep = R.StepReport()
    by_layer = {l: sorted((ou for ou in units if ou.layer == l), key=lambda ou: ou.u) for l in range(w.n_layers)}
    totals = dict(needed=0, hits=0, reads=0, evictions=0, read_calls=0)
    for t, q in enumerate(W.query_stream(w, rig.q0, steps, R.DEV)):
        for l in range(w.n_layers):
            rig.step(l, t, q[l])
            missed = [R.compare_unit(rig, ou, t, q[l], rep)["misses"] for ou in by_layer[l]]
            lp = l % w.phys_layers
            want = otier.fetch(lp, t, missed, opos[lp])
            got = rig.tier.trace()
            assert (got["needed"], got["hits"], got["reads"]) == (len(want["needed"]), len(want["hits"]), len(want["reads"])), (l, t)
            assert got["evicted"] == want["evicted"], (l, t)
            assert got["runs"] == want["runs"], (l, t)
            assert rig.tier.pooled() == sorted(otier.stamp), (l, t)
            for key in totals:
                totals[key] += got[key]
            if t % 3 == 0 or t == steps - 1:
                R.check_directory(rig, l, by_layer[l])
        if progress:
            print(f"[{progress}] step {t} ok: misses {rep.misses} extents read {totals['reads']} hit {totals['hits']} "
                  f"evicted {totals['evictions']} read calls {totals['read_calls']}", flush=True)
    return rep, totals


def oracle_positions(rig, units, semantic):
    """The oracle's own layout (from the oracle's clusters), checked against the library's."""
    w = rig.w
    opos = []
    for lp in range(w.phys_layers):
        rows = []
        for u in range(w.units):
            ou = next(o for o in units if o.layer == lp and o.u == u)
            rows.append(orc.extent_positions(w.n_pages, ou.members if semantic else None))
        opos.append(rows)
        assert np.array_equal(np.stack(rows), rig.positions[lp]), f"layout of layer {lp} differs"
    return opos


@pytest.mark.parametrize("cfg,kw,tier", [
    # pools of units x k extents: the cold step just fits, every later read evicts
    (3, dict(), dict(extent_pages=8, pool_extents=768, max_run_extents=4, queue_depth=4)),
    (3, dict(), dict(extent_pages=1, pool_extents=768, max_run_extents=8, queue_depth=1)),
    (2, dict(), dict(extent_pages=4, pool_extents=512, max_run_extents=2, queue_depth=8)),             # 3 layers on 2 physical
    (4, dict(), dict(extent_pages=3, pool_extents=192, max_run_extents=8, queue_depth=3)),             # fp16, page 32, ragged last extent
    (5, dict(), dict(extent_pages=2, pool_extents=130, max_run_extents=8, queue_depth=2, direct_io=True)),  # page 64, forced recent pages
    (3, dict(policy="lookahead"), dict(extent_pages=8, pool_extents=4000, max_run_extents=1, queue_depth=4)),
    (3, dict(index_centroids=550, index_iterations=3), dict(extent_pages=4, pool_extents=768, max_run_extents=8, queue_depth=4, semantic=True)),
    (4, dict(index_centroids=150, index_iterations=2), dict(extent_pages=8, pool_extents=192, max_run_extents=8, queue_depth=4, semantic=True)),
])
def test_tiered_step_parity(tmp_path, cfg, kw, tier):
    w = SCALED[cfg].replace(**kw)
    rig = R.Rig(w, micro_batches=1)
    units = all_units(rig)
    semantic = bool(tier.get("semantic"))
    rig.attach_tier(str(tmp_path / "kv.bin"), **tier)
    opos = oracle_positions(rig, units, semantic)
    otier = orc.ExtentTier(w.units, w.n_pages, tier["extent_pages"], tier["pool_extents"], tier["max_run_extents"])
    rep, totals = run_tiered(rig, units, w.steps, otier, opos, progress=f"cfg{cfg}-tier")
    assert rep.unit_steps == w.steps * w.n_layers * w.units and rep.tie_divergences <= 2
    assert rep.misses > 0 and totals["reads"] > 0
    st = rig.tier.stats()
    print(f"[cfg{cfg}-tier] direct I/O mode {st.direct_io}, {st.bytes_read / 2**20:.1f} MiB read in {st.ms_io:.2f} ms", flush=True)
    assert st.extent_reads == totals["reads"] and st.pages_requested == rep.misses
    assert st.bytes_read == totals["reads"] * tier["extent_pages"] * w.page_bytes
    if tier["pool_extents"] < 1000:
        assert totals["evictions"] > 0                               # the pool was under pressure
    rig.close()


def test_tiered_step_equals_plain_step_and_reports_errors(tmp_path):
    """Same workload through kvd_step and kvd_step_tiered: identical traces, outputs equal to the
    last bit (same kernels, same bytes in the slots).  Then the error paths."""
    w = small("tier-eq", batch=3, topk_pages=20, capacity=44, steps=5)
    plain, tiered = R.Rig(w, micro_batches=1), R.Rig(w, micro_batches=1)
    tiered.attach_tier(str(tmp_path / "kv.bin"), extent_pages=4, pool_extents=512, max_run_extents=8)
    for t, q in enumerate(W.query_stream(w, plain.q0, w.steps, R.DEV)):
        plain.step(0, t, q[0])
        tiered.step(0, t, q[0])
        assert np.array_equal(plain.n_sel_pages, tiered.n_sel_pages) and np.array_equal(plain.n_hit_mask, tiered.n_hit_mask)
        assert np.array_equal(plain.n_evicted, tiered.n_evicted) and np.array_equal(plain.n_counts, tiered.n_counts)
        assert np.array_equal(plain.n_out, tiered.n_out) and np.array_equal(plain.n_lse, tiered.n_lse)
    a, b = plain.kvd.cache_export(0), tiered.kvd.cache_export(0)
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
    assert torch.equal(plain.pool.view(torch.int16), tiered.pool.view(torch.int16))
    # a step that needs more extents than the pool holds is refused
    small_pool = R.Rig(w, micro_batches=1)
    small_pool.attach_tier(str(tmp_path / "kv2.bin"), extent_pages=4, pool_extents=8)
    q = next(iter(W.query_stream(w, small_pool.q0, 1, R.DEV)))
    with pytest.raises(K.KvdError) as e:
        small_pool.kvd.step_tiered(0, 0, q[0], small_pool.out, small_pool.lse)
    assert e.value.status == K.ERR_CAPACITY
    torch.cuda.synchronize()
    # no tier bound; a tier of another shape; a pool that is not pinned
    with pytest.raises(K.KvdError) as e:
        plain.kvd.step_tiered(0, 9, q[0], plain.out, plain.lse)
    assert e.value.status == K.ERR_STATE
    mem = torch.zeros(64 * 4 * w.page_bytes + 4096, dtype=torch.uint8)
    mem = mem[(-mem.data_ptr()) % 4096:][: 64 * 4 * w.page_bytes]
    other = K.KvdTier(str(tmp_path / "o.bin"), mem, n_layers=1, n_units=w.units + 1, max_pages=w.n_pages, extent_pages=4,
                      page_bytes=w.page_bytes, pool_extents=64)
    with pytest.raises(K.KvdError) as e:
        plain.kvd.bind_tier(other)
    assert e.value.status == K.ERR_SHAPE
    other.close()
    unpinned = K.KvdTier(str(tmp_path / "u.bin"), mem, n_layers=1, n_units=w.units, max_pages=w.n_pages, extent_pages=4,
                         page_bytes=w.page_bytes, pool_extents=64)
    with pytest.raises(K.KvdError) as e:
        plain.kvd.bind_tier(unpinned)
    assert e.value.status == K.ERR_ARG
    unpinned.close()
    for r in (plain, tiered, small_pool):
        r.close()


def test_append_kv_reaches_the_backing_file_and_the_pool(tmp_path):
    """Tokens appended during decoding must arrive in the backing file and in pooled extents: half
    way through, the GPU window and the DRAM pool are emptied, so that every page a step attends —
    the grown ones included (they are forced into the selection) — comes from the file."""
    w = small("tier-append", recent_pages=2, topk_pages=20, capacity=40, steps=14)
    P = w.page
    seq = [w.ctx - 2 * P - 5, w.ctx - 3 * P]
    rig = R.Rig(w, seq_lens=seq, micro_batches=1)
    units = all_units(rig)
    rig.attach_tier(str(tmp_path / "kv.bin"), extent_pages=4, pool_extents=4000)
    rig.kvd.bind_host_store(rig.store)                               # the growing pages live in the host store
    gen = torch.Generator(device="cpu").manual_seed(7)
    rep = R.StepReport()
    qs = W.query_stream(w, rig.q0, w.steps, R.DEV)
    for t in range(w.steps):
        q = next(qs)
        if t == w.steps // 2:
            rig.kvd.cache_reset()
            rig.tier.drop_pool()
            for ou in units:
                ou.window = type(ou.window)(ou.window.capacity)
        rig.step(0, t, q[0])
        for ou in units:
            R.compare_unit(rig, ou, t, q[0], rep)
        if t == w.steps // 2:
            assert rig.tier.trace()["hits"] == 0 and rig.tier.trace()["reads"] > 0
        k_new = torch.randn((w.batch, w.n_kv_heads, w.head_dim), generator=gen).to(w.torch_dtype)
        v_new = torch.randn((w.batch, w.n_kv_heads, w.head_dim), generator=gen).to(w.torch_dtype)
        rig.kvd.append_kv(0, k_new.to(R.DEV), v_new.to(R.DEV))
        rig.kvd.advance()
        torch.cuda.synchronize()
        for ou in units:
            pos = ou.seq_len
            ou.keys[pos] = H.f64(k_new[ou.b, ou.h])
            ou.values[pos] = H.f64(v_new[ou.b, ou.h])
            ou.seq_len = pos + 1
            ou.summ = orc.page_summaries(ou.keys, P, ou.seq_len, ou.code)
        rig.seq_lens = [s + 1 for s in rig.seq_lens]
        if t % 5 == 0 or t == w.steps - 1:
            R.check_directory(rig, 0, units)
    assert rep.tie_divergences <= 2 and rep.unit_steps == w.steps * w.units
    # the file itself: every page that grew, read back through a fresh pool
    rig.tier.drop_pool()
    for ou in units:
        grown = sorted({p for p in range(seq[ou.b] // P, (seq[ou.b] + w.steps - 1) // P + 1)})
        lst = torch.full((w.units, w.topk_pages, 2), -1, dtype=torch.int32)
        cnt = torch.zeros(w.units, dtype=torch.int32)
        for j, p in enumerate(grown):
            lst[ou.u, j, 0], lst[ou.u, j, 1] = p, 0
        cnt[ou.u] = len(grown)
        off = rig.tier.fetch(0, 1000 + ou.u, lst, cnt)
        for j, p in enumerate(grown):
            o = int(off[ou.u, j])
            got = rig.tier_pool[o:o + w.page_bytes].view(torch.int16)
            assert torch.equal(got, rig.store[0, ou.b, ou.h, p].view(torch.int16).reshape(-1)), (ou.u, p)
    rig.close()
