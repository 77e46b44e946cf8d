"""The third tier's host engine (backing file, DRAM pool of extents, read plan) against the
oracle and the hand-worked fixture.  Runs without a GPU: the engine is plain host code and its pool
is ordinary memory here."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import kvd_oracle as orc
from paper_2605_18071_amd import kvd
from tests import helpers as H

RNG = np.random.default_rng(77001)


def _ints(s):
    return [int(x) for x in s.split() if x != "-"]


def _aligned_pool(nbytes, align=4096):
    raw = torch.zeros(nbytes + align, dtype=torch.uint8)
    shift = (-raw.data_ptr()) % align
    return raw[shift:shift + nbytes]


def _miss_tensors(missed, k):
    U = len(missed)
    lst = torch.full((U, k, 2), -7, dtype=torch.int32)
    cnt = torch.zeros(U, dtype=torch.int32)
    for u, pages in enumerate(missed):
        cnt[u] = len(pages)
        for j, p in enumerate(pages):
            lst[u, j, 0] = p
            lst[u, j, 1] = j                                  # any slot >= 0
    return lst, cnt


def _open(tmp_path, pages, positions, E, pool_extents, max_run, qd=3, direct=False, name="kv.bin"):
    L, U, NP, nbytes = pages.shape
    pool = _aligned_pool(pool_extents * E * nbytes)
    tier = kvd.KvdTier(str(tmp_path / name), pool, n_layers=L, n_units=U, max_pages=NP, extent_pages=E, page_bytes=nbytes,
                       pool_extents=pool_extents, queue_depth=qd, max_run_extents=max_run, direct_io=direct)
    for l in range(L):
        tier.set_layout(l, torch.from_numpy(np.stack(positions[l]).astype(np.int32)))
        tier.write_layer(l, torch.from_numpy(pages[l].copy()))
    return tier, pool


def _check_step(tier, pool, oracle_tier, l, t, missed, positions, pages, k):
    lst, cnt = _miss_tensors(missed, k)
    off = tier.fetch(l, t, lst, cnt)
    want = oracle_tier.fetch(l, t, missed, positions[l])
    got = tier.trace()
    assert got["needed"] == len(want["needed"]) and got["hits"] == len(want["hits"])
    assert got["reads"] == len(want["reads"]) and got["evicted"] == want["evicted"]
    assert got["runs"] == want["runs"]
    assert tier.pooled() == sorted(oracle_tier.stamp)
    nbytes = pages.shape[-1]
    for u, pg in enumerate(missed):
        for j, p in enumerate(pg):
            o = int(off[u, j])
            assert o >= 0 and o % nbytes == 0
            assert np.array_equal(pool[o:o + nbytes].numpy(), pages[l, u, p]), (t, u, p)
    return got


def test_engine_reproduces_the_hand_worked_trace(tmp_path):
    rows = H.read_golden("tier_trace_2units.txt")
    head = {r[0].split(":")[0].strip(): r[0].split(":")[1] for r in rows if ":" in r[0] and len(r) == 1}
    positions = [[np.array(_ints(head["position 0"])), np.array(_ints(head["position 1"]))]]
    pages = RNG.integers(0, 256, size=(1, 2, 8, 64), dtype=np.uint8)
    tier, pool = _open(tmp_path, pages, positions, E=2, pool_extents=3, max_run=2)
    lib = kvd.load()
    for step, m0, m1, needed, hits, reads, evicted, runs, pooled in [r for r in rows if len(r) == 9]:
        missed = [_ints(m0), _ints(m1)]
        lst, cnt = _miss_tensors(missed, 4)
        off = tier.fetch(0, int(step), lst, cnt)
        got = tier.trace()
        assert (got["needed"], got["hits"], got["reads"]) == (len(_ints(needed)), len(_ints(hits)), len(_ints(reads))), step
        assert got["evicted"] == _ints(evicted), step
        assert got["runs"] == [tuple(int(x) for x in r.split(":")) for r in runs.split()], step
        assert tier.pooled() == _ints(pooled), step
        for u in range(2):
            for j, p in enumerate(missed[u]):
                o = int(off[u, j])
                assert np.array_equal(pool[o:o + 64].numpy(), pages[0, u, p]), (step, u, p)
    st = tier.stats()
    assert st.steps == 7 and st.extent_reads == 14 and st.bytes_read == 14 * 2 * 64 and st.reads_issued == 11
    assert lib.kvd_tier_last_errno(tier.handle) == 0
    tier.close()


@pytest.mark.parametrize("E,pool_extents,max_run,qd,direct", [
    (2, 9, 3, 1, False), (4, 6, 8, 4, False), (3, 64, 2, 8, False), (8, 5, 1, 2, False), (1, 17, 4, 3, False),
    (4, 6, 8, 4, True),
])
def test_engine_matches_oracle_on_random_traces(tmp_path, E, pool_extents, max_run, qd, direct):
    L, U, NP = 2, 3, 37
    nbytes = 4096 if direct else 48                      # direct I/O wants extents that are multiples of 4096 bytes
    k = 6
    pages = RNG.integers(0, 256, size=(L, U, NP, nbytes), dtype=np.uint8)
    positions = [[orc.extent_positions(NP, [np.nonzero(a == c)[0] for c in range(5)])
                  for a in RNG.integers(0, 5, size=(U, NP))] for _ in range(L)]
    tier, pool = _open(tmp_path, pages, positions, E, pool_extents, max_run, qd, direct)
    ot = orc.ExtentTier(U, NP, E, pool_extents, max_run)
    n_reads = 0
    for t in range(50):
        l = int(RNG.integers(0, L))
        missed, budget = [], pool_extents
        for u in range(U):
            pg = sorted(RNG.choice(NP, size=int(RNG.integers(0, k + 1)), replace=False).tolist())
            ext = {positions[l][u][p] // E for p in pg}
            if len(ext) > budget:
                pg, ext = [], set()
            budget -= len(ext)
            missed.append(pg)
        n_reads += _check_step(tier, pool, ot, l, t, missed, positions, pages, k)["reads"]
    st = tier.stats()
    assert st.extent_reads == n_reads and st.bytes_read == n_reads * E * nbytes and st.steps == 50
    assert st.direct_io in (0, 1) and (direct or st.direct_io == 0)
    # rewriting a layer drops its extents from the pool, and the new bytes are what comes back
    pages[0] = RNG.integers(0, 256, size=pages[0].shape, dtype=np.uint8)
    tier.write_layer(0, torch.from_numpy(pages[0].copy()))
    for g in [g for g in ot.stamp if g < U * ot.NE]:
        del ot.stamp[g]
    assert tier.pooled() == sorted(ot.stamp)
    _check_step(tier, pool, ot, 0, 50, [[0, 5], [], [36]], positions, pages, k)
    tier.drop_pool()
    assert tier.pooled() == []
    tier.close()


@pytest.mark.parametrize("E,pool_extents,max_run", [(2, 9, 3), (4, 6, 8), (1, 17, 4)])
def test_engine_matches_oracle_when_step_indices_repeat(tmp_path, E, pool_extents, max_run):
    """Every step index three times: pooled extents then tie in stamp with the ones a step needs,
    so the victim order (stamp, extent number) and the exclusion of needed extents both show."""
    L, U, NP, nbytes, k = 2, 3, 37, 48, 6
    pages = RNG.integers(0, 256, size=(L, U, NP, nbytes), dtype=np.uint8)
    positions = [[orc.extent_positions(NP) for _ in range(U)] for _ in range(L)]
    tier, pool = _open(tmp_path, pages, positions, E, pool_extents, max_run, name="kv_repeat.bin")
    ot = orc.ExtentTier(U, NP, E, pool_extents, max_run)
    evicted = 0
    for i in range(60):
        l = int(RNG.integers(0, L))
        missed, budget = [], pool_extents
        for u in range(U):
            pg = sorted(RNG.choice(NP, size=int(RNG.integers(0, k + 1)), replace=False).tolist())
            ext = {positions[l][u][p] // E for p in pg}
            if len(ext) > budget:
                pg, ext = [], set()
            budget -= len(ext)
            missed.append(pg)
        evicted += len(_check_step(tier, pool, ot, l, i // 3, missed, positions, pages, k)["evicted"])
    assert evicted > 0
    tier.close()


def test_engine_refuses_what_it_cannot_do(tmp_path):
    lib = kvd.load()
    pages = RNG.integers(0, 256, size=(1, 2, 16, 32), dtype=np.uint8)
    positions = [[orc.extent_positions(16), orc.extent_positions(16)]]
    tier, pool = _open(tmp_path, pages, positions, E=2, pool_extents=3, max_run=4)
    ot = orc.ExtentTier(2, 16, 2, 3, 4)
    _check_step(tier, pool, ot, 0, 0, [[0, 1], [4]], positions, pages, 8)
    before = tier.pooled()
    # four extents in one step do not fit a pool of three: refused, nothing changed
    lst, cnt = _miss_tensors([[0, 2, 4, 6], []], 8)
    with pytest.raises(kvd.KvdError) as e:
        tier.fetch(0, 1, lst, cnt)
    assert e.value.status == kvd.ERR_CAPACITY and tier.pooled() == before
    with pytest.raises(ValueError):
        orc.ExtentTier(2, 16, 2, 3, 4).fetch(0, 1, [[0, 2, 4, 6], []], positions[0])
    # a page outside the unit, a count beyond k, a layer that does not exist
    for bad_list, bad_cnt, layer in [([[16], []], None, 0), ([[0], []], [9, 0], 0), ([[0], []], None, 1)]:
        lst, cnt = _miss_tensors(bad_list, 8)
        if bad_cnt:
            cnt = torch.tensor(bad_cnt, dtype=torch.int32)
        with pytest.raises(kvd.KvdError) as e:
            tier.fetch(layer, 1, lst, cnt)
        assert e.value.status == kvd.ERR_ARG
    assert tier.pooled() == before
    # entries without a slot are skipped
    lst, cnt = _miss_tensors([[9], [3]], 8)
    lst[0, 0, 1] = -1
    off = tier.fetch(0, 2, lst, cnt)
    assert int(off[0, 0]) == -1 and tier.trace()["needed"] == 1
    # a layout must be a permutation
    bad = torch.arange(16, dtype=torch.int32).repeat(2, 1)
    bad[1, 3] = 4
    with pytest.raises(kvd.KvdError) as e:
        tier.set_layout(0, bad)
    assert e.value.status == kvd.ERR_ARG
    tier.close()
    # open: misaligned pool, sizes out of range, a path that cannot be created
    cfg = kvd.KvdTierConfig(1, 2, 16, 2, 32, 3, 2, 4, 0)
    h = C.c_void_p()
    mem = _aligned_pool(4096)
    path = str(tmp_path / "x.bin").encode()
    assert lib.kvd_tier_open(C.byref(cfg), path, mem.data_ptr() + 8, C.byref(h)) == kvd.ERR_ARG
    for field, value in [("extent_pages", 0), ("queue_depth", 0), ("queue_depth", 65), ("max_run_extents", 65),
                         ("pool_extents", 0), ("page_bytes", 24), ("n_units", 0)]:
        c2 = kvd.KvdTierConfig(1, 2, 16, 2, 32, 3, 2, 4, 0)
        setattr(c2, field, value)
        assert lib.kvd_tier_open(C.byref(c2), path, mem.data_ptr(), C.byref(h)) == kvd.ERR_SHAPE, field
    assert lib.kvd_tier_open(C.byref(cfg), str(tmp_path / "no" / "dir.bin").encode(), mem.data_ptr(), C.byref(h)) == kvd.ERR_STATE
    assert lib.kvd_tier_open(None, path, mem.data_ptr(), C.byref(h)) == kvd.ERR_ARG
    assert lib.kvd_tier_close(None) == kvd.ERR_ARG and lib.kvd_tier_fetch(None, 0, 0, None, None, 1, None) == kvd.ERR_ARG


def test_sequential_read_covers_the_file(tmp_path):
    pages = RNG.integers(0, 256, size=(1, 4, 64, 256), dtype=np.uint8)
    positions = [[orc.extent_positions(64)] * 4]
    tier, _ = _open(tmp_path, pages, positions, E=4, pool_extents=16, max_run=4, qd=4)
    assert tier.sequential_read_gbps() > 0.0 and tier.pooled() == []
    tier.close()
    tier, _ = _open(tmp_path, pages, positions, E=4, pool_extents=15, max_run=4, qd=4, name="b.bin")
    with pytest.raises(kvd.KvdError) as e:                # 4 readers x 4 extents of scratch do not fit 15
        tier.sequential_read_gbps()
    assert e.value.status == kvd.ERR_CAPACITY
    tier.close()


def test_patch_page_reaches_file_and_pool(tmp_path):
    pages = RNG.integers(0, 256, size=(1, 2, 12, 4096), dtype=np.uint8)
    positions = [[orc.extent_positions(12, [np.array([7, 1, 3]), np.array([0, 2, 4, 5, 6, 8, 9, 10, 11])]), orc.extent_positions(12)]]
    for direct in (False, True):
        tier, pool = _open(tmp_path, pages, positions, E=2, pool_extents=4, max_run=2, direct=direct, name=f"p{int(direct)}.bin")
        ot = orc.ExtentTier(2, 12, 2, 4, 2)
        _check_step(tier, pool, ot, 0, 0, [[1], [5]], positions, pages, 4)           # page 1 of unit 0 is pooled now
        new = RNG.integers(0, 256, size=300, dtype=np.uint8)
        for u, p, at in [(0, 1, 100), (0, 9, 0), (1, 5, 3796)]:                       # pooled, not pooled, pooled (end of page)
            tier.patch_page(0, u, p, at, torch.from_numpy(new.copy()))
            pages[0, u, p, at:at + 300] = new
        _check_step(tier, pool, ot, 0, 1, [[1, 9], [5]], positions, pages, 4)        # pooled copies and the file agree
        tier.drop_pool()
        ot.stamp.clear()
        _check_step(tier, pool, ot, 0, 2, [[1, 9, 3], [5, 4]], positions, pages, 4)  # and so does a fresh read
        with pytest.raises(kvd.KvdError) as e:
            tier.patch_page(0, 0, 1, 4000, torch.from_numpy(new.copy()))             # runs over the end of the page
        assert e.value.status == kvd.ERR_ARG
        tier.close()
    # the file image is the oracle's
    image = orc.extent_file_image(pages[0], positions[0], 2)
    raw = np.fromfile(str(tmp_path / "p1.bin"), dtype=np.uint8).reshape(image.shape)   # (the file of the last round)
    assert np.array_equal(raw, image)
