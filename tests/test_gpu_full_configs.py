"""Parity at the benchmark definition's full per-layer sizes, in the launch
configuration bench.py times: the HIP path runs the whole batch, the oracle
follows a sample of units step by step (selection, cache trace, attention output).

cfg2 and cfg4 keep their full per-layer shape but run 2 of their 32 / 28 layers
(the layers are independent and identical in shape); cfg3 and cfg5 are complete.
"""
import numpy as np
import pytest
import torch

from paper_2605_18071_amd import workloads as W
from tests import helpers as H

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from tests import gpu_rig as R

def _units(layers, batches, heads):
    return [(l, b, h) for l in layers for b in batches for h in heads]


# configuration, decode steps, units the oracle follows in the form bench.py times, and in the other form
FULL = {
    # 2 of the 32 layers, 16 units of each (every second sequence, every second KV head), all 64 steps
    2: (W.CONFIGS[2].replace(n_layers=2, physical_layers=2), 64, _units((0, 1), (0, 2, 5, 7), (0, 3, 4, 7)),
        [(0, 0, 0), (0, 3, 5), (1, 7, 7), (1, 4, 2)]),
    # every one of the 128 units, all 32 steps
    3: (W.CONFIGS[3], 32, _units((0,), range(16), range(8)), [(0, 0, 0), (0, 5, 3), (0, 9, 6), (0, 15, 7)]),
    # 2 of the 28 layers, 16 units of each, all 16 steps
    4: (W.CONFIGS[4].replace(n_layers=2, physical_layers=2), 16, _units((0, 1), (0, 9, 13, 20, 26, 31, 4, 17), (0, 3)),
        [(0, 0, 0), (0, 31, 3), (1, 13, 1), (1, 20, 2)]),
    # every one of the 32 units, all 16 steps
    5: (W.CONFIGS[5], 16, _units((0,), range(4), range(8)), [(0, 0, 0), (0, 1, 4), (0, 3, 7)]),
}
OTHER_STEPS = {2: 12, 3: 32, 4: 10, 5: 16}


def test_full_size_one_launch_equals_chain_over_many_steps():
    """cfg3 at full size, 96 decode steps with the real miss stream: the one-launch step and the
    chain of kernels, fed the same queries from the same cold start, must produce the same
    selections, cache traces and slot contents at every step, and the same outputs up to the fp32
    summation order of the attention."""
    w = W.CONFIGS[3]
    a = R.Rig(w, micro_batches=-1)
    b = R.Rig(w, micro_batches=1, build_index=False)
    b.summaries.copy_(a.summaries)
    assert a.kvd.step_form() == -1 and b.kvd.step_form() == 1
    worst = 0.0
    for t, q in enumerate(W.query_stream(w, a.q0, 96, R.DEV)):
        a.step(0, t, q[0])
        b.step(0, t, q[0])
        assert np.array_equal(a.n_sel_pages, b.n_sel_pages), t
        assert np.array_equal(a.n_hit_mask, b.n_hit_mask), t
        assert np.array_equal(a.n_sel_slots, b.n_sel_slots), t
        assert np.array_equal(np.sort(a.n_evicted, axis=1), np.sort(b.n_evicted, axis=1)), t
        assert np.array_equal(a.n_counts, b.n_counts), t
        assert np.array_equal(a.n_scores, b.n_scores), t
        worst = max(worst, H.attn_rel_err(a.n_out, b.n_out))
        assert worst <= 1e-5, (t, worst)
        if t % 24 == 23:
            print(f"[cfg3 one launch vs chain] step {t} ok, evictions so far {int(a.kvd.stats().evictions)}, "
                  f"max output difference {worst:.2e}", flush=True)
    assert a.kvd.stats().evictions > 0
    sa, _ = a.kvd.cache_export(0)
    sb, _ = b.kvd.cache_export(0)
    assert torch.equal(sa, sb)
    for u in (0, 37, 127):                                            # slot contents, a few units in full
        bb, hh = divmod(u, w.n_kv_heads)
        assert torch.equal(a.pool[0, bb, hh].cpu().view(torch.int16), b.pool[0, bb, hh].cpu().view(torch.int16)), u
    a.close()
    b.close()
    del a, b
    torch.cuda.empty_cache()


def test_full_size_hierarchical_index():
    """cfg3 at full size with half as many centroids as pages: index build and sampled decode parity."""
    w = W.CONFIGS[3].replace(index_centroids=4096, index_iterations=2)
    print("[cfg3-hier] building workload and index", flush=True)
    rig = R.Rig(w)
    print("[cfg3-hier] index built, checking sampled units", flush=True)
    units = [R.OracleUnit(rig, 0, b, h) for (b, h) in [(0, 0), (7, 3), (15, 7)]]
    print(f"[cfg3-hier] k-means assignments that differ inside rounding: {sum(o.kmeans_divergences for o in units)}", flush=True)
    rep = R.run_steps(rig, units, 8, check_dir_every=4, progress="cfg3-hier-full")
    assert rep.unit_steps == 8 * len(units) and rep.tie_divergences <= 2
    rig.close()
    del rig
    torch.cuda.empty_cache()


def test_full_size_third_tier(tmp_path):
    """cfg3 at full size behind the third tier (8 GiB backing file, cluster-ordered extents of 8
    pages, DRAM pool of a quarter of the extents, direct I/O): sampled units against the oracle as
    usual, and the tier's trace of every step against the oracle's extent pool fed with the miss
    sets of the whole batch."""
    from oracle import kvd_oracle as orc
    w = W.CONFIGS[3].replace(index_centroids=4096, index_iterations=2)
    E, pool_extents, max_run = 8, 32768, 8
    print("[cfg3-tier] building workload and index", flush=True)
    rig = R.Rig(w)
    units = [R.OracleUnit(rig, 0, b, h) for (b, h) in [(0, 0), (9, 6)]]
    print("[cfg3-tier] writing the backing file", flush=True)
    rig.attach_tier(str(tmp_path / "kv.bin"), extent_pages=E, pool_extents=pool_extents, max_run_extents=max_run,
                    queue_depth=16, direct_io=True, semantic=True)
    for ou in units:                                                  # the oracle's layout for the units it has clustered
        assert np.array_equal(orc.extent_positions(w.n_pages, ou.members), rig.positions[0][ou.u])
    assert all(sorted(row.tolist()) == list(range(w.n_pages)) for row in rig.positions[0][::17])
    otier = orc.ExtentTier(w.units, w.n_pages, E, pool_extents, max_run)
    rep = R.StepReport()
    reads = 0
    for t, q in enumerate(W.query_stream(w, rig.q0, 8, R.DEV)):
        rig.step(0, t, q[0])
        for ou in units:
            R.compare_unit(rig, ou, t, q[0], rep)
        valid = (rig.n_sel_pages >= 0) & (rig.n_hit_mask == 0)
        missed = [sorted(rig.n_sel_pages[u][valid[u]].tolist()) for u in range(w.units)]
        want = otier.fetch(0, t, missed, rig.positions[0])
        got = rig.tier.trace()
        assert (got["needed"], got["hits"], got["reads"]) == (len(want["needed"]), len(want["hits"]), len(want["reads"])), t
        assert got["evicted"] == want["evicted"] and got["runs"] == want["runs"], t
        reads += got["reads"]
        print(f"[cfg3-tier] step {t} ok: missed pages {sum(map(len, missed))}, extents needed {got['needed']} "
              f"read {got['reads']} in {got['read_calls']} calls, evicted {got['evictions']}", flush=True)
    R.check_directory(rig, 0, units)
    assert rig.tier.pooled() == sorted(otier.stamp)
    st = rig.tier.stats()
    assert st.extent_reads == reads and st.extent_evictions > 0 and rep.unit_steps == 8 * len(units)
    print(f"[cfg3-tier] direct I/O mode {st.direct_io}, {st.bytes_read / 2**30:.2f} GiB in {st.ms_io:.0f} ms", flush=True)
    rig.close()
    del rig
    torch.cuda.empty_cache()


@pytest.mark.parametrize("cfg,mb,part", [(3, 0, 0), (3, 0, 1), (3, 0, 2), (3, 0, 3), (3, 1, 0), (2, 0, 0), (2, 1, 0), (4, 0, 0), (4, 1, 0),
                                         (5, 0, 0), (5, 0, 1), (5, 1, 0)])
def test_full_size_parity(cfg, mb, part):
    """mb = 0: the form the library chooses, which is what bench.py times (one launch for all four);
    there the oracle follows every unit of cfg3 and cfg5 (a quarter / a half of the sequences per run
    of the workload, `part`: the oracle needs about 20 ms per unit and step of cfg3) and 32 units of cfg2 and cfg4,
    over all of the configuration's decode steps.  mb = 1: the chain of kernels, a few units."""
    w, steps, wide, few = FULL[cfg]
    if mb == 0 and cfg in (3, 5):
        parts = 4 if cfg == 3 else 2
        wide = [x for x in wide if x[1] * parts // w.batch == part]
    sample = wide if mb == 0 else few
    steps = steps if mb == 0 else OTHER_STEPS[cfg]
    print(f"[cfg{cfg}] building workload", flush=True)
    rig = R.Rig(w, micro_batches=mb)
    assert rig.kvd.step_form() == (-1 if mb == 0 else 1)
    print(f"[cfg{cfg}] workload ready, building {len(sample)} oracle units", flush=True)
    units = []
    for i, (l, b, h) in enumerate(sample):
        units.append(R.OracleUnit(rig, l, b, h, lazy=True))
        if i % 16 == 15:
            print(f"[cfg{cfg}] {i + 1} oracle units built", flush=True)
    rep = R.run_steps(rig, units, steps, check_dir_every=max(1, steps // 3), progress=f"cfg{cfg}-full-mb{mb}")
    assert rep.unit_steps == steps * len(sample)
    assert rep.tie_divergences <= max(2, rep.unit_steps // 500)
    st = rig.kvd.stats()
    assert st.hits + st.misses == steps * w.n_layers * w.units * w.topk_pages
    print(f"[cfg{cfg}] {len(sample)} units x {steps} steps = {rep.unit_steps} unit-steps against the oracle; "
          f"hit rate over the whole batch {st.hits / (st.hits + st.misses):.3f}, "
          f"max attention rel err {rep.max_attn_err:.2e}, max score err {rep.max_score_err:.2e}, "
          f"tie divergences {rep.tie_divergences}", flush=True)
    rig.close()
    del rig, units
    torch.cuda.empty_cache()
