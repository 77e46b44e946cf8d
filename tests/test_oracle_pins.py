"""Pins for the CPU oracle: each stage is checked against something other than
itself — hand-worked fixtures, closed forms, brute force, library routines and
invariants — chosen so that a dropped term, a wrong sign or index, or a
transposed operand fails at least one of them.  CPU only.
"""
import itertools
import math

import numpy as np
import pytest
import scipy.special
import torch

from oracle import kvd_oracle as orc
from tests import helpers as H

RNG = np.random.default_rng(20260518)


# --------------------------------------------------------------------------- #
# dtype conversions
# --------------------------------------------------------------------------- #
def _all_values(dtype):
    b = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    if dtype == orc.F16:
        v = torch.from_numpy(b.view(np.int16)).view(torch.float16).to(torch.float64).numpy()
    else:
        v = torch.from_numpy(b.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    return b, v


@pytest.mark.parametrize("dtype", [orc.F16, orc.BF16])
def test_bits_to_f64_matches_torch_widening(dtype):
    b, v = _all_values(dtype)
    got = orc.bits_to_f64(b, dtype)
    same = (got == v) | (np.isnan(got) & np.isnan(v))
    assert same.all()


@pytest.mark.parametrize("dtype", [orc.F16, orc.BF16])
def test_round_f64_is_nearest_even_by_brute_force(dtype):
    """Nearest representable value found by searching the sorted table of all
    finite values of the format; ties resolved to the even mantissa."""
    b, v = _all_values(dtype)
    fin = np.isfinite(v) & ~((v == 0) & (b >> 15 == 1))          # drop -0 duplicate
    vals, pats = v[fin], b[fin]
    order = np.argsort(vals, kind="stable")
    vals, pats = vals[order], pats[order]
    scale = 2.0 ** RNG.integers(-30 if dtype == orc.F16 else -140, 14, size=4000)
    x = RNG.standard_normal(4000) * scale
    # exact midpoints between neighbours must go to the even pattern
    mids_i = RNG.integers(0, len(vals) - 1, size=500)
    mids = (vals[mids_i] + vals[mids_i + 1]) / 2.0                # exact in fp64
    x = np.concatenate([x, mids, vals[RNG.integers(0, len(vals), 200)]])
    got = orc.round_f64(x, dtype)
    for xi, gi in zip(x, got):
        if abs(xi) > vals[-1]:
            continue
        j = np.searchsorted(vals, xi)
        cands = [c for c in (j - 1, j) if 0 <= c < len(vals)]
        best = min(cands, key=lambda c: (abs(vals[c] - xi), int(pats[c]) & 1))
        assert gi == vals[best], (xi, gi, vals[best])


def test_f16_rounding_matches_numpy_cast():
    x = RNG.standard_normal(20000) * 2.0 ** RNG.integers(-26, 17, size=20000)
    want = x.astype(np.float16)
    got = orc.f64_to_bits(x, orc.F16).view(np.float16)
    assert np.array_equal(got.view(np.uint16), want.view(np.uint16))


def test_bf16_rounding_known_values():
    # 1 + 2^-8 is the midpoint between 1 and 1 + 2^-7: ties to even -> 1
    assert orc.round_f64(np.array([1.0 + 2.0 ** -8]), orc.BF16)[0] == 1.0
    # 1 + 3*2^-8 is the midpoint between 1+2^-7 (odd) and 1+2^-6 (even)
    assert orc.round_f64(np.array([1.0 + 3 * 2.0 ** -8]), orc.BF16)[0] == 1.0 + 2.0 ** -6
    assert orc.round_f64(np.array([1.0 + 2.0 ** -8 + 2.0 ** -40]), orc.BF16)[0] == 1.0 + 2.0 ** -7
    assert orc.f64_to_bits(np.array([1.0]), orc.BF16)[0] == 0x3F80
    assert orc.f64_to_bits(np.array([-2.5]), orc.BF16)[0] == 0xC020
    # fp32 -> bf16 of torch agrees wherever the value is an exact fp32
    x32 = (RNG.standard_normal(20000) * 2.0 ** RNG.integers(-20, 20, size=20000)).astype(np.float32)
    want = H.bits(torch.from_numpy(x32).to(torch.bfloat16))
    assert np.array_equal(orc.f64_to_bits(x32.astype(np.float64), orc.BF16), want)


# --------------------------------------------------------------------------- #
# summaries
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("dtype", [orc.F16, orc.BF16])
def test_summaries_closed_forms(dtype):
    P, D = 16, 8
    keys = np.zeros((3 * P, D))
    keys[:P] = np.linspace(-2, 2, D)[None, :] * 0.5               # constant page -> the key itself
    keys[P:2 * P] = np.where(np.arange(P)[:, None] % 2 == 0, 1.75, -1.75)   # +x,-x alternating -> 0
    keys[2 * P:] = np.arange(P)[:, None] * np.ones(D)              # 0..15 -> 7.5
    s = orc.page_summaries(keys, P, 3 * P, dtype)
    assert np.array_equal(s[0], orc.round_f64(keys[0], dtype))
    assert np.array_equal(s[1], np.zeros(D))
    assert np.array_equal(s[2], np.full(D, 7.5))


def test_summaries_vs_numpy_mean_and_partial_page():
    P, D, T = 8, 16, 8 * 5 + 3                                     # ragged last page: 3 valid tokens
    k16 = (RNG.standard_normal((48, D))).astype(np.float16)
    keys = k16.astype(np.float64)
    s = orc.page_summaries(keys, P, T, orc.F16)
    assert s.shape == (6, D)
    for p in range(6):
        lo, hi = p * P, min((p + 1) * P, T)
        want = np.mean(keys[lo:hi], axis=0).astype(np.float16).astype(np.float64)
        assert np.array_equal(s[p], want)
    # tokens beyond seq_len must not leak into the last page
    keys2 = keys.copy()
    keys2[T:] = 1e4
    assert np.array_equal(orc.page_summaries(keys2, P, T, orc.F16), s)


# --------------------------------------------------------------------------- #
# scores
# --------------------------------------------------------------------------- #
def test_pooled_query_and_scores_reduce_to_dot_products():
    G, D, T = 4, 32, 50
    q = RNG.standard_normal((G, D))
    k = RNG.standard_normal((T, D))
    qbar = orc.pooled_query(q)
    assert np.allclose(qbar, q.mean(axis=0), rtol=0, atol=1e-15)
    # page size 1: the summary is the key, the score is the scaled dot product
    summ = orc.page_summaries(orc.round_f64(k, orc.F16), 1, T, orc.F16)
    scale = 1.0 / math.sqrt(D)
    sc = orc.page_scores(qbar, summ, scale)
    want = np.array([sum(qbar[d] * summ[t, d] for d in range(D)) * scale for t in range(T)])
    assert np.allclose(sc, want, rtol=1e-13, atol=1e-14)
    # linearity in the query
    q2 = RNG.standard_normal((G, D))
    lhs = orc.page_scores(orc.pooled_query(q + q2), summ, scale)
    rhs = sc + orc.page_scores(orc.pooled_query(q2), summ, scale)
    assert np.allclose(lhs, rhs, rtol=0, atol=1e-12)
    # a transposed operand or a pooled sum instead of a mean would break this:
    e0 = np.zeros((G, D)); e0[:, 3] = 2.0
    assert np.allclose(orc.page_scores(orc.pooled_query(e0), summ, 1.0), 2.0 * summ[:, 3])


# --------------------------------------------------------------------------- #
# selection
# --------------------------------------------------------------------------- #
def test_select_golden_fixture():
    for scores, k, sink, recent, want in H.read_golden("select_ties.txt"):
        s = np.array([float(x) for x in scores.split()])
        got = orc.select_pages(s, int(k), int(sink), int(recent))
        assert got.tolist() == [int(x) for x in want.split()], (scores, k, sink, recent)


def test_select_vs_lexsort_and_special_cases():
    for n, k in [(7, 3), (64, 64), (100, 1), (257, 31), (1000, 128)]:
        s = np.round(RNG.standard_normal(n), 1)                   # coarse grid -> many ties
        got = orc.select_pages(s, k)
        order = np.lexsort((np.arange(n), -s))                    # primary: -score, then page
        assert got.tolist() == sorted(order[:k].tolist())
        if k == 1:
            assert got[0] == int(np.argmax(s))                     # argmax returns the first maximum
        if k == n:
            assert got.tolist() == list(range(n))
    s = RNG.standard_normal(300)
    prev = set()
    for k in range(1, 60):
        cur = set(orc.select_pages(s, k).tolist())
        assert prev < cur and len(cur) == k
        prev = cur


def test_select_forced_pages_and_errors():
    s = RNG.standard_normal(40)
    got = orc.select_pages(s, 10, sink_pages=2, recent_pages=3)
    assert {0, 1, 37, 38, 39} <= set(got.tolist())
    rest = sorted(set(got.tolist()) - {0, 1, 37, 38, 39})
    free = np.argsort(-s[2:37], kind="stable")[:5] + 2
    assert rest == sorted(free.tolist())
    with pytest.raises(ValueError):
        orc.select_pages(s, 4, sink_pages=2, recent_pages=3)


def test_planted_heavy_pages_are_selected_on_config1():
    from paper_2605_18071_amd import workloads as W
    w = W.CONFIGS[1]
    q0 = W.initial_queries(w)
    store = W.make_kv_store(w, q0, pin=False)
    q = next(W.query_stream(w, q0, 1))
    u = W.query_direction(w, q0)
    code = H.dtype_code(w.torch_dtype)
    scale = 1.0 / math.sqrt(w.head_dim)
    for h in range(w.n_kv_heads):
        keys = H.f64(store[0, 0, h, :, 0]).reshape(-1, w.head_dim)
        summ = orc.page_summaries(keys, w.page, w.ctx, code)
        qg = H.f64(q[0, 0, h * w.group:(h + 1) * w.group])
        sc = orc.page_scores(orc.pooled_query(qg), summ, scale)
        sel = set(orc.select_pages(sc, w.topk_pages).tolist())
        # the planted pages are the ones whose mean key has a large component along u
        proj = summ @ H.f64(u[0, 0, h])
        heavy = set(np.nonzero(proj > 1.5)[0].tolist())
        assert len(heavy) == w.heavy_count
        assert heavy <= sel


# --------------------------------------------------------------------------- #
# LRU window
# --------------------------------------------------------------------------- #
def _ints(cell):
    return [] if cell == "-" else [int(x) for x in cell.split()]


def test_lru_golden_trace():
    win = orc.LruWindow(3)
    for step, sel, hits, misses, evicted, resident in H.read_golden("lru_trace_5pages.txt"):
        h, m, e = win.resolve(_ints(sel), int(step))
        assert (h, m, e) == (_ints(hits), _ints(misses), _ints(evicted)), step
        want = {int(a.split(":")[0]): int(a.split(":")[1]) for a in resident.split()}
        assert win.stamp == want, step


def _batch_lru(resident, sel, step, cap):
    """A different route to the same answer: the victims of a step are the
    e = max(0, |resident| + |misses| - cap) smallest (stamp, page) among resident
    pages outside the selection."""
    selset = set(sel)
    hits = sorted(p for p in sel if p in resident)
    misses = sorted(p for p in sel if p not in resident)
    e = max(0, len(resident) + len(misses) - cap)
    cands = sorted((s, p) for p, s in resident.items() if p not in selset)
    evicted = sorted(p for _, p in cands[:e])
    for p in evicted:
        del resident[p]
    for p in sel:
        resident[p] = step
    return hits, misses, evicted


@pytest.mark.parametrize("n_pages,k,cap", [(40, 6, 6), (40, 6, 11), (64, 8, 24), (30, 5, 30)])
def test_lru_against_batch_formulation_and_invariants(n_pages, k, cap):
    win = orc.LruWindow(cap)
    shadow = {}
    prev_sel, seen = None, set()
    for t in range(60):
        centre = (t // 3) % n_pages
        weights = np.exp(-0.15 * np.abs(np.arange(n_pages) - centre)) + 0.02
        sel = sorted(RNG.choice(n_pages, size=k, replace=False, p=weights / weights.sum()).tolist())
        before = len(win.stamp)
        h, m, e = win.resolve(sel, t)
        assert (h, m, e) == _batch_lru(shadow, sel, t, cap)
        assert win.stamp == shadow
        assert len(h) + len(m) == k and set(h) | set(m) == set(sel)
        assert len(win.stamp) <= cap
        assert len(e) == max(0, before + len(m) - cap)
        assert not (set(e) & set(sel))
        assert all(win.stamp[p] == t for p in sel)
        if cap == k and prev_sel is not None:                     # the "x1" window: misses = S_t \ S_{t-1}
            assert m == sorted(set(sel) - set(prev_sel))
        if cap == n_pages:                                        # everything fits: a page misses at most once
            assert not (set(m) & seen) and not e
        seen |= set(sel)
        prev_sel = sel


def test_lru_inclusion_property_over_capacity():
    n_pages, k = 50, 5
    trace = []
    for t in range(80):
        centre = (t // 2) % n_pages
        w = np.exp(-0.2 * np.abs(np.arange(n_pages) - centre)) + 0.01
        trace.append(sorted(RNG.choice(n_pages, size=k, replace=False, p=w / w.sum()).tolist()))
    caps = [5, 8, 13, 21, 34, 50]
    wins = [orc.LruWindow(c) for c in caps]
    total = [0] * len(caps)
    for t, sel in enumerate(trace):
        for i, win in enumerate(wins):
            total[i] += len(win.resolve(sel, t)[1])
        for a, b in zip(wins, wins[1:]):
            assert set(a.stamp) <= set(b.stamp)
    assert all(x >= y for x, y in zip(total, total[1:]))
    assert total[-1] == len(set(itertools.chain.from_iterable(trace)))


def test_lru_rejects_k_above_capacity_and_warm():
    win = orc.LruWindow(2)
    with pytest.raises(ValueError):
        win.resolve([0, 1, 2], 0)
    win.warm([3, 4])
    assert win.resolve([3, 5], 0) == ([3], [5], [4])
    with pytest.raises(ValueError):
        orc.LruWindow(2).warm([1, 2, 3])                              # a warm list longer than the window
    again = orc.LruWindow(2)
    again.warm([1, 2])
    again.warm([2, 1])                                                # pages already resident take no room


def test_lru_never_evicts_a_page_selected_in_the_same_step():
    """Hand-worked: when a step index repeats (a replayed step), resident pages that were not
    selected tie in stamp with the selected ones; the victim is still taken from the unselected
    pages only, lowest page first."""
    win = orc.LruWindow(3)
    assert win.resolve([0, 1], 5) == ([], [0, 1], [])
    assert win.resolve([1, 2], 5) == ([1], [2], [])                   # window full: {0, 1, 2}, all stamped 5
    assert win.resolve([0, 3], 5) == ([0], [3], [1])                  # 0 is selected: 1 leaves, not 0
    assert win.resident() == [0, 2, 3]
    assert win.resolve([2, 4], 5) == ([2], [4], [0])                  # unselected: 0 and 3, equal stamps -> lower page
    la = orc.LookaheadWindow(3)
    sc = np.array([0.0, 1.0, 2.0, 3.0, 4.0])                          # page 0 scores lowest but is selected
    la.warm([0, 1, 2])
    assert la.resolve([0, 3], 1, scores=sc) == ([0], [3], [1])


# --------------------------------------------------------------------------- #
# lookahead eviction
# --------------------------------------------------------------------------- #
def test_lookahead_golden_trace():
    win = orc.LookaheadWindow(3)
    for step, scores, sel, hits, misses, evicted, resident in H.read_golden("la_trace_5pages.txt"):
        sc = np.array([float(x) for x in scores.split()])
        assert orc.select_pages(sc, 2).tolist() == _ints(sel), step
        h, m, e = win.resolve(_ints(sel), int(step), scores=sc)
        assert (h, m, e) == (_ints(hits), _ints(misses), _ints(evicted)), step
        assert win.resident() == _ints(resident), step


def test_lookahead_pool_golden_traces():
    wins = {}
    for name, cap, pool, step, scores, sel, pool_pages, hits, misses, evicted, resident in H.read_golden("la_pool_trace_6pages.txt"):
        win = wins.setdefault(name, orc.LookaheadWindow(int(cap), pool=int(pool)))
        sc = np.array([float(x) for x in scores.split()])
        assert orc.select_pages(sc, 2).tolist() == _ints(sel), (name, step)
        assert sorted(win.pool_pages(sc)) == _ints(pool_pages), (name, step)
        h, m, e = win.resolve(_ints(sel), int(step), scores=sc)
        assert (h, m, e) == (_ints(hits), _ints(misses), _ints(evicted)), (name, step)
        assert win.resident() == _ints(resident), (name, step)


def test_lookahead_pool_reduces_to_the_policy_without_a_pool_and_to_lru():
    """A pool that covers every scored page is the policy without a pool; a pool that is exactly the
    selection (M = k, no forced pages) leaves only recency to order the victims: LRU.  In between,
    the victims are the batch formulation: unselected residents outside the pool by (stamp, page),
    then those inside by (score, -page)."""
    n_pages, k, cap = 60, 7, 19
    for pool in (n_pages, n_pages + 5, 0, k, 12, 30):
        win, plain, lru = orc.LookaheadWindow(cap, pool=pool), orc.LookaheadWindow(cap), orc.LruWindow(cap)
        for t in range(70):
            scores = np.round(RNG.normal(size=n_pages), 1) + 0.3 * np.exp(-0.1 * np.abs(np.arange(n_pages) - (3 * t) % n_pages))
            sel = orc.select_pages(scores, k).tolist()
            before = dict(win.stamp)
            got = win.resolve(sel, t, scores=scores)
            if pool == 0 or pool >= n_pages:
                assert got == plain.resolve(sel, t, scores=scores) and win.stamp == plain.stamp
            elif pool == k:
                assert got == lru.resolve(sel, t) and win.stamp == lru.stamp
            else:
                inside = set(np.lexsort((np.arange(n_pages), -scores))[:pool].tolist())
                assert inside == win.pool_pages(scores)
                cands = [p for p in before if p not in set(sel)]
                order = sorted((p for p in cands if p not in inside), key=lambda p: (before[p], p)) + \
                        sorted((p for p in cands if p in inside), key=lambda p: (scores[p], -p))
                need = max(0, len(before) + len(got[1]) - cap)
                assert got[2] == sorted(order[:need])
                assert len(win.stamp) <= cap and not (set(got[2]) & set(sel))


def test_lookahead_with_recency_scores_is_lru():
    """If the score of a resident page is the step at which it was last selected (plus a
    page-increasing sliver that orders equal stamps as LRU does), "lowest score first" is
    "least recently selected first": the policy must then reproduce the LRU trace."""
    n_pages, k, cap = 48, 6, 15
    la, lru = orc.LookaheadWindow(cap), orc.LruWindow(cap)
    for t in range(80):
        centre = (2 * t) % n_pages
        w = np.exp(-0.2 * np.abs(np.arange(n_pages) - centre)) + 0.02
        sel = sorted(RNG.choice(n_pages, size=k, replace=False, p=w / w.sum()).tolist())
        recency = np.full(n_pages, -1.0)
        for p, s in lru.stamp.items():
            recency[p] = s
        recency += np.arange(n_pages) * 2.0 ** -20
        assert la.resolve(sel, t, scores=recency) == lru.resolve(sel, t)
        assert la.stamp == lru.stamp


@pytest.mark.parametrize("n_pages,k,cap", [(40, 6, 6), (40, 6, 11), (64, 8, 24), (30, 5, 30)])
def test_lookahead_invariants_and_batch_formulation(n_pages, k, cap):
    win = orc.LookaheadWindow(cap)
    for t in range(60):
        scores = np.round(RNG.normal(size=n_pages), 1)            # one decimal: plenty of exact ties
        sel = orc.select_pages(scores, k).tolist()
        before = dict(win.stamp)
        h, m, e = win.resolve(sel, t, scores=scores)
        need = max(0, len(before) + len(m) - cap)
        assert len(e) == need and not (set(e) & set(sel)) and set(e) <= set(before)
        assert len(h) + len(m) == k and len(win.stamp) <= cap
        # a different route: rank all unselected residents once, lowest (score, -page) first
        cands = sorted((scores[p], -p) for p in before if p not in set(sel))
        assert e == sorted(-n for _, n in cands[:need])
        # whoever stayed does not score below whoever left
        kept = [p for p in before if p not in set(sel) and p not in set(e)]
        if e and kept:
            assert max(scores[p] for p in e) <= min(scores[p] for p in kept)
        assert all(win.stamp[p] == t for p in sel)


def test_lookahead_forced_eviction_and_errors():
    win = orc.LookaheadWindow(3)
    sc = np.array([0.5, 0.4, 0.3, 0.2, 0.1, 0.0])
    win.warm([0, 1, 2])
    with pytest.raises(ValueError):
        win.resolve([3, 4], 0)                                      # no scores
    with pytest.raises(ValueError):
        win.resolve([3, 4], 0, scores=sc, forced_evicted=[0])       # one victim short
    with pytest.raises(ValueError):
        win.resolve([3, 4], 0, scores=sc, forced_evicted=[0, 5])    # page 5 is not resident
    assert win.resolve([3, 4], 0, scores=sc, forced_evicted=[0, 1]) == ([], [3, 4], [0, 1])
    assert win.resident() == [2, 3, 4]
    assert win.resolve([0, 3], 1, scores=sc) == ([3], [0], [4])     # own choice: lowest score (page 4) leaves


# --------------------------------------------------------------------------- #
# hierarchical index
# --------------------------------------------------------------------------- #
def _blobs(n_blobs, per_blob, dim, spread, seed):
    rng = np.random.default_rng(seed)
    centres = rng.normal(size=(n_blobs, dim)) * 4.0
    pts = np.concatenate([c + spread * rng.normal(size=(per_blob, dim)) for c in centres])
    return orc.round_f64(pts[rng.permutation(len(pts))], orc.BF16)


def test_kmeans_matches_sklearn_lloyd():
    """The same initial centroids and iteration count through scikit-learn's Lloyd k-means."""
    from sklearn.cluster import KMeans
    pts = _blobs(12, 40, 24, 0.6, 3)
    for n_c, iters in [(12, 5), (30, 4), (60, 7)]:
        _, assign, exact = orc.kmeans_centroids(pts, n_c, iters, orc.BF16)
        assert np.bincount(assign, minlength=n_c).min() > 0          # sklearn would relocate empty clusters
        km = KMeans(n_clusters=n_c, init=orc.kmeans_init(pts, n_c), n_init=1, max_iter=iters, tol=0.0, algorithm="lloyd").fit(pts)
        assert np.allclose(km.cluster_centers_, exact, rtol=1e-9, atol=1e-9)


def test_kmeans_closed_forms_and_invariants():
    rng = np.random.default_rng(8)
    # the initial centroids are the points at the middles of n_centroids equal stretches of the
    # sequence, floor((i + 1/2) n / n_centroids): 10 points, 2 centroids -> points 2 and 7; 7 points,
    # 3 centroids -> points 1, 3, 5 (hand-worked)
    line = np.arange(10, dtype=np.float64)[:, None] * np.ones((1, 4))
    assert np.array_equal(orc.kmeans_init(line, 2), line[[2, 7]])
    assert np.array_equal(orc.kmeans_init(line[:7], 3), line[[1, 3, 5]])
    assert np.array_equal(orc.kmeans_init(line, 10), line)
    pts = orc.round_f64(rng.normal(size=(96, 16)), orc.F16)
    # as many centroids as points: every point is its own cluster and its own centroid
    cent, assign, _ = orc.kmeans_centroids(pts, 96, 3, orc.F16)
    assert np.array_equal(assign, np.arange(96)) and np.array_equal(cent, pts)
    # one centroid: the mean of everything (one rounding)
    cent, assign, exact = orc.kmeans_centroids(pts, 1, 2, orc.F16)
    assert np.all(assign == 0) and np.allclose(exact[0], pts.mean(axis=0), rtol=0, atol=1e-12)
    assert np.array_equal(cent[0], orc.round_f64(exact[0], orc.F16))
    # well separated blobs, one initial centroid inside each: the blobs are recovered
    centres = np.eye(6, 16) * 50.0
    blob_pts = np.concatenate([centres[i] + 0.1 * rng.normal(size=(10, 16)) for i in range(6)])   # evenly spaced init hits every blob
    _, assign, exact = orc.kmeans_centroids(blob_pts, 6, 4, orc.BF16)
    assert np.array_equal(assign, np.repeat(np.arange(6), 10))
    assert np.allclose(exact, blob_pts.reshape(6, 10, 16).mean(axis=1))
    # Lloyd never increases the within-cluster sum of squares; a centroid is the mean of its members;
    # every point sits with a nearest centroid of the round it was assigned in
    pts = _blobs(9, 30, 12, 1.0, 5)
    prev = np.inf
    for iters in range(1, 7):
        cent, assign, exact = orc.kmeans_centroids(pts, 20, iters, orc.BF16)
        inertia = float(np.sum((pts - exact[assign]) ** 2))
        assert inertia <= prev + 1e-9
        prev = inertia
        for c in range(20):
            members = np.nonzero(assign == c)[0]
            if len(members):
                assert np.allclose(exact[c], pts[members].mean(axis=0), rtol=0, atol=1e-12)
        assert np.array_equal(cent, orc.round_f64(exact, orc.BF16))
    before = orc.kmeans_centroids(pts, 20, 5, orc.BF16)[2]
    d = ((pts[:, None, :] - before[None, :, :]) ** 2).sum(axis=2)                 # brute-force distances
    _, assign6, _ = orc.kmeans_centroids(pts, 20, 6, orc.BF16)
    assert np.allclose(d[np.arange(len(pts)), assign6], d.min(axis=1), rtol=1e-12, atol=1e-12)
    # distance ties go to the lower centroid; an empty cluster keeps its centroid
    pts2 = np.array([[0.0, 0.0], [2.0, 0.0], [1.0, 0.0]])
    cents = np.array([[0.0, 0.0], [2.0, 0.0], [9.0, 9.0]])
    assert orc.kmeans_assign(pts2, cents).tolist() == [0, 1, 0]
    assert np.array_equal(orc.kmeans_update(pts2, np.array([0, 1, 0]), cents), np.array([[0.5, 0.0], [2.0, 0.0], [9.0, 9.0]]))
    # forcing the assignments replaces the oracle's own decisions
    forced = [np.array([1, 1, 0]), np.array([0, 0, 1])]
    _, a, exact = orc.kmeans_centroids(pts2, 2, 2, orc.BF16, forced_assign=forced)
    assert a.tolist() == [0, 0, 1] and np.array_equal(exact, np.array([[1.0, 0.0], [1.0, 0.0]]))


def test_hier_select_golden_fixture():
    members = [np.array(m, dtype=np.int32) for m in ([0, 1], [2, 7, 9], [], [3, 4, 5, 6], [8, 11], [10])]
    for scores, k, sink, recent, want in H.read_golden("hier_select_6clusters.txt"):
        sc = np.array([float(x) for x in scores.split()])
        got = orc.select_pages_hier(sc, members, int(k), 12, int(sink), int(recent))
        exp = _ints(want)
        assert got.tolist() == exp + [-1] * (int(k) - len(exp)), (scores, k)


def test_hier_select_reduces_to_flat_selection_and_brute_force():
    rng = np.random.default_rng(21)
    # one page per cluster, cluster c = page c: the hierarchical rule is the flat Top-K rule
    for n, k, sink, recent in [(50, 7, 0, 0), (64, 16, 2, 3), (10, 10, 0, 0), (9, 12, 1, 1)]:
        sc = np.round(rng.normal(size=n), 1)
        members = [np.array([c], dtype=np.int32) for c in range(n)]
        assert np.array_equal(orc.select_pages_hier(sc, members, k, n, sink, recent), orc.select_pages(sc, k, sink, recent))
    # random clusters: page by page simulation of "walk the ranked clusters, one page at a time"
    for trial in range(30):
        n, n_c, k = 80, 23, int(rng.integers(1, 60))
        assign = rng.integers(0, n_c, size=n)
        members = orc.cluster_members(assign, n_c)
        sc = np.round(rng.normal(size=n_c), 1)
        ranked = np.lexsort((np.arange(n_c), -sc))
        walk = [p for c in ranked for p in np.sort(np.nonzero(assign == c)[0])]
        want = sorted(walk[:k])
        got = orc.select_pages_hier(sc, members, k, n)
        assert got[got >= 0].tolist() == want and len(want) == min(k, n)
        # with forced pages: they go in first and the walk skips them
        sink, recent = int(rng.integers(0, 3)), int(rng.integers(0, 4))
        forced = sorted(set(range(sink)) | set(range(n - recent, n)))
        if len(forced) <= k:
            walk2 = [p for p in walk if p not in forced]
            want2 = sorted(forced + walk2[:k - len(forced)])
            got2 = orc.select_pages_hier(sc, members, k, n, sink, recent)
            assert got2[got2 >= 0].tolist() == want2
    with pytest.raises(ValueError):
        orc.select_pages_hier(np.zeros(3), [np.array([0]), np.array([1]), np.array([2])], 2, 3, sink_pages=2, recent_pages=1)


# --------------------------------------------------------------------------- #
# attention
# --------------------------------------------------------------------------- #
def test_attention_closed_form_fixture():
    for case, q, keys, values, out, lse in H.read_golden("attention_closed_form.txt"):
        qv = np.array([[H.parse_num(x) for x in q.split()]])
        kv = np.array([[H.parse_num(x) for x in r.split()] for r in keys.split(";")])
        vv = np.array([[H.parse_num(x) for x in r.split()] for r in values.split(";")])
        o, l = orc.attend(qv, kv, vv, 1.0)
        assert np.allclose(o[0], [H.parse_num(x) for x in out.split()], rtol=0, atol=1e-14), case
        assert abs(l[0] - H.parse_num(lse)) < 1e-14, case


def test_attention_equals_dense_softmax_when_all_pages_selected():
    G, D, P, T = 4, 32, 8, 8 * 9 + 5
    q = RNG.standard_normal((G, D))
    k = RNG.standard_normal((80, D))
    v = RNG.standard_normal((80, D))
    scale = 1.0 / math.sqrt(D)
    n_pages = -(-T // P)
    toks = orc.selected_tokens(np.arange(n_pages), P, T)
    assert toks.tolist() == list(range(T))                        # ragged last page masked
    o, l = orc.attend(q, k[toks], v[toks], scale)
    logits = scale * (q @ k[:T].T)                                # [G, T]
    w = scipy.special.softmax(logits, axis=1)
    assert np.allclose(o, w @ v[:T], rtol=1e-12, atol=1e-13)
    assert np.allclose(l, scipy.special.logsumexp(logits, axis=1), rtol=0, atol=1e-12)


def test_selected_tokens_are_the_valid_tokens_of_the_selected_pages():
    """Hand-worked: page size 4, 10 valid tokens: page 2 is partial (tokens 8, 9); padding entries
    (-1) stand for no page at all."""
    assert orc.selected_tokens([0, 2], 4, 10).tolist() == [0, 1, 2, 3, 8, 9]
    assert orc.selected_tokens([-1, 1, -1], 4, 10).tolist() == [4, 5, 6, 7]
    assert orc.selected_tokens([-1, -1], 4, 10).tolist() == []


def test_attention_invariants():
    G, D, n = 1, 16, 40
    q = RNG.standard_normal((G, D))
    k = RNG.standard_normal((n, D))
    v = RNG.standard_normal((n, D))
    scale = 0.25
    o, l = orc.attend(q, k, v, scale)
    # shift invariance: K_i += c/(scale |q|^2) q adds c to every logit
    c = 3.5
    k2 = k + (c / (scale * float(q[0] @ q[0]))) * q[0]
    o2, l2 = orc.attend(q, k2, v, scale)
    assert np.allclose(o2, o, rtol=0, atol=1e-12) and abs(l2[0] - l[0] - c) < 1e-12
    # constant values come back unchanged (weights sum to one)
    oc, _ = orc.attend(q, k, np.tile(np.arange(D, dtype=float), (n, 1)), scale)
    assert np.allclose(oc[0], np.arange(D), rtol=0, atol=1e-13)
    # permutation of the tokens
    perm = RNG.permutation(n)
    op, lp = orc.attend(q, k[perm], v[perm], scale)
    assert np.allclose(op, o, rtol=0, atol=1e-13) and abs(lp[0] - l[0]) < 1e-13
    # one dominating key takes all the weight
    k3 = k.copy(); k3[7] = 400.0 * q[0] / float(q[0] @ q[0]) / scale
    od, _ = orc.attend(q, k3, v, scale)
    assert np.allclose(od[0], v[7], rtol=0, atol=1e-9)
    # heads are independent: a second head must not change the first
    q2 = np.vstack([q, RNG.standard_normal((1, D))])
    o22, _ = orc.attend(q2, k, v, scale)
    assert np.array_equal(o22[0], o[0])


# --------------------------------------------------------------------------- #
# whole step
# --------------------------------------------------------------------------- #
def test_step_output_does_not_depend_on_cache_state():
    G, D, P, NP = 2, 16, 4, 12
    T = P * NP - 1
    keys = orc.round_f64(RNG.standard_normal((P * NP, D)), orc.BF16)
    vals = orc.round_f64(RNG.standard_normal((P * NP, D)), orc.BF16)
    q = orc.round_f64(RNG.standard_normal((G, D)), orc.BF16)
    summ = orc.page_summaries(keys, P, T, orc.BF16)
    cold, warm = orc.LruWindow(6), orc.LruWindow(6)
    kw = dict(k=4, page_size=P, seq_len=T, scale=0.25)
    first = orc.decode_unit_step(q, summ, keys, vals, warm, 0, **kw)
    a = orc.decode_unit_step(q, summ, keys, vals, cold, 1, **kw)
    b = orc.decode_unit_step(q, summ, keys, vals, warm, 1, **kw)
    assert a["misses"] == first["misses"] and b["misses"] == [] and b["hits"] == a["misses"]
    assert np.array_equal(a["out"], b["out"]) and np.array_equal(a["sel"], b["sel"])
    # the selected set is the brute-force top-k of the printed scores
    order = np.lexsort((np.arange(NP), -a["scores"]))
    assert a["sel"].tolist() == sorted(order[:4].tolist())
    # and the attention is dense attention restricted to those pages' valid tokens
    toks = [t for p in a["sel"] for t in range(p * P, min((p + 1) * P, T))]
    w = scipy.special.softmax(0.25 * (q @ keys[toks].T), axis=1)
    assert np.allclose(a["out"], w @ vals[toks], rtol=1e-12, atol=1e-13)


def test_lookahead_under_the_hierarchical_index_uses_the_cluster_score():
    """Hand-worked: 6 pages in clusters {2,3} {0,1} {4,5} with scores 0.1, 0.9, 0.5; all but page 5
    resident, capacity 5; page 5 comes in -> the lowest cluster score is cluster 0's, its higher
    page 3 leaves.  Then page 3 comes back -> page 2 (cluster 0's other page) leaves; then a page of
    no cluster (6, score -inf) is the first to go."""
    members = [np.array([2, 3]), np.array([0, 1]), np.array([4, 5])]
    per_page = orc.cluster_scores_by_page(np.array([0.1, 0.9, 0.5]), members, 7)
    assert per_page.tolist() == [0.9, 0.9, 0.1, 0.1, 0.5, 0.5, -np.inf]
    win = orc.LookaheadWindow(5)
    win.warm([0, 1, 2, 3, 4])
    assert win.resolve([4, 5], 0, scores=per_page) == ([4], [5], [3])
    assert win.resolve([3, 5], 1, scores=per_page) == ([5], [3], [2])
    win2 = orc.LookaheadWindow(3)
    win2.warm([0, 2, 6])
    assert win2.resolve([1], 0, scores=per_page) == ([], [1], [6])


def test_unit_step_wires_the_stages_together():
    """Hand-worked wiring of decode_unit_step.  (a) A selection forced on the step replaces the
    step's own in the window *and* in the attention: the output is the attention over the forced
    pages' tokens.  (b) With the hierarchical index under lookahead eviction the victim is ranked by
    the score of its cluster, not by the entry of the cluster-score array at the page's own index:
    clusters {2,3} {0,1} with centroid scores (low, high) -> pages 2 and 3 score low, 0 and 1 high."""
    G, D, P, NP = 2, 8, 2, 6
    T = P * NP
    keys = orc.round_f64(RNG.standard_normal((T, D)), orc.BF16)
    vals = orc.round_f64(RNG.standard_normal((T, D)), orc.BF16)
    summ = orc.page_summaries(keys, P, T, orc.BF16)
    q = orc.round_f64(RNG.standard_normal((G, D)), orc.BF16)
    win = orc.LruWindow(4)
    own = orc.decode_unit_step(q, summ, keys, vals, orc.LruWindow(4), 0, k=2, page_size=P, seq_len=T, scale=0.5)
    other = sorted(set(range(NP)) - set(own["sel"].tolist()))[:2]
    got = orc.decode_unit_step(q, summ, keys, vals, win, 0, k=2, page_size=P, seq_len=T, scale=0.5, forced_sel=other)
    assert got["sel"].tolist() == own["sel"].tolist() and got["used"].tolist() == other
    assert got["misses"] == other and win.resident() == other
    toks = np.array([t for p in other for t in range(p * P, (p + 1) * P)])
    want, want_lse = orc.attend(q, keys[toks], vals[toks], 0.5)
    assert np.array_equal(got["out"], want) and np.array_equal(got["lse"], want_lse)
    assert not np.allclose(got["out"], own["out"])
    # (b): two centroids; qbar . centroid: cluster 0 = pages {2, 3} low, cluster 1 = pages {0, 1} high
    members = [np.array([2, 3]), np.array([0, 1])]
    qh = np.zeros((1, D)); qh[0, 0] = 1.0
    cent = np.zeros((2, D)); cent[0, 0] = -1.0; cent[1, 0] = 2.0
    la = orc.LookaheadWindow(3)
    la.warm([0, 2, 3])
    r = orc.decode_unit_step(qh, summ[:4], keys[:4 * P], vals[:4 * P], la, 0, k=2, page_size=P, seq_len=4 * P, scale=1.0,
                             centroids=cent, members=members)
    assert r["sel"].tolist() == [0, 1]                                # the high cluster
    assert r["evict_scores"].tolist() == [2.0, 2.0, -1.0, -1.0]
    assert (r["hits"], r["misses"], r["evicted"]) == ([0], [1], [3])  # low cluster, higher page first


def test_hierarchical_step_with_one_page_per_cluster_is_the_flat_lookahead_step():
    """Clusters of one page each, the page's summary as centroid: the step through the index
    must be the flat step, lookahead victims included."""
    G, D, P, NP = 2, 16, 4, 30
    T = P * NP
    keys = orc.round_f64(RNG.standard_normal((T, D)), orc.BF16)
    vals = orc.round_f64(RNG.standard_normal((T, D)), orc.BF16)
    summ = orc.page_summaries(keys, P, T, orc.BF16)
    members = [np.array([p]) for p in range(NP)]
    flat, hier = orc.LookaheadWindow(9), orc.LookaheadWindow(9)
    kw = dict(k=5, page_size=P, seq_len=T, scale=0.25)
    for t in range(12):
        q = orc.round_f64(RNG.standard_normal((G, D)), orc.BF16)
        a = orc.decode_unit_step(q, summ, keys, vals, flat, t, **kw)
        b = orc.decode_unit_step(q, summ, keys, vals, hier, t, centroids=summ, members=members, **kw)
        assert (a["hits"], a["misses"], a["evicted"]) == (b["hits"], b["misses"], b["evicted"])
        assert np.array_equal(a["sel"], b["sel"]) and np.array_equal(a["out"], b["out"])
    assert flat.stamp == hier.stamp and len(flat.stamp) == 9


# --------------------------------------------------------------------------- #
# third tier: layout of the backing file, DRAM pool of extents, read plan
# --------------------------------------------------------------------------- #
def _tier_fixture():
    rows = H.read_golden("tier_trace_2units.txt")
    head = {r[0].split(":")[0].strip(): r[0].split(":")[1] for r in rows if ":" in r[0] and len(r) == 1}
    clusters = [np.array(_ints(c), dtype=np.int32) for c in head["clusters 1"].split(";")]
    positions = [np.array(_ints(head["position 0"])), np.array(_ints(head["position 1"]))]
    steps = [r for r in rows if len(r) == 9]
    return clusters, positions, steps


def test_extent_layout_matches_hand_worked_fixture():
    clusters, positions, _ = _tier_fixture()
    assert orc.extent_positions(8).tolist() == positions[0].tolist()
    assert orc.extent_positions(8, clusters).tolist() == positions[1].tolist()


def test_extent_tier_matches_hand_worked_trace():
    _, positions, steps = _tier_fixture()
    tier = orc.ExtentTier(n_units=2, n_pages=8, extent_pages=2, pool_extents=3, max_run_extents=2)
    assert len(steps) == 7
    for step, m0, m1, needed, hits, reads, evicted, runs, pooled in steps:
        got = tier.fetch(0, int(step), [_ints(m0), _ints(m1)], positions)
        assert got["needed"] == _ints(needed), step
        assert got["hits"] == _ints(hits), step
        assert got["reads"] == _ints(reads), step
        assert got["evicted"] == _ints(evicted), step
        assert got["runs"] == [tuple(int(x) for x in r.split(":")) for r in runs.split()], step
        assert sorted(tier.stamp) == _ints(pooled), step


def test_extent_positions_keep_clusters_together():
    n_pages = 57
    assign = RNG.integers(0, 9, size=n_pages)
    assign[RNG.choice(n_pages, size=5, replace=False)] = -1          # pages of no cluster (beyond the valid length)
    members = [np.nonzero(assign == c)[0] for c in range(9)]
    pos = orc.extent_positions(n_pages, members)
    assert sorted(pos.tolist()) == list(range(n_pages))
    start = 0
    for c in range(9):                                               # cluster c fills the next len(c) places, pages ascending
        assert pos[members[c]].tolist() == list(range(start, start + len(members[c])))
        start += len(members[c])
    rest = np.nonzero(assign < 0)[0]
    assert pos[rest].tolist() == list(range(start, n_pages))
    with pytest.raises(ValueError):
        orc.extent_positions(4, [np.array([0, 1]), np.array([1, 2])])


def test_extent_tier_of_single_page_extents_is_the_lru_window():
    """Extents of one page, one unit, page order: "extent needed" is "page selected", so the
    pool must behave exactly as the page-granular LRU window (pinned on its own above)."""
    n_pages, cap = 40, 11
    tier = orc.ExtentTier(1, n_pages, 1, cap, 1)
    lru = orc.LruWindow(cap)
    pos = [orc.extent_positions(n_pages)]
    for t in range(80):
        want = sorted(RNG.choice(n_pages, size=int(RNG.integers(0, 7)), replace=False).tolist())
        got = tier.fetch(0, t, [want], pos)
        hits, misses, evicted = lru.resolve(want, t)
        assert (got["hits"], got["reads"], got["evicted"]) == (hits, misses, evicted)
        assert got["runs"] == [(p, 1) for p in misses]
        assert tier.stamp == lru.stamp


def test_extent_tier_never_evicts_an_extent_the_step_needs():
    """Hand-worked: with a repeated step index the pooled extents all tie in stamp; the victim is
    still taken from the extents that the step does not need."""
    tier = orc.ExtentTier(n_units=1, n_pages=8, extent_pages=2, pool_extents=2, max_run_extents=4)
    pos = [np.arange(8)]
    assert tier.fetch(0, 5, [[0]], pos)["reads"] == [0]
    assert tier.fetch(0, 5, [[2]], pos)["reads"] == [1]               # pool full: extents 0 and 1, both stamped 5
    r = tier.fetch(0, 5, [[0, 4]], pos)                               # needs extents 0 (pooled) and 2
    assert (r["hits"], r["reads"], r["evicted"]) == ([0], [2], [1])   # 1 leaves, not the needed 0


@pytest.mark.parametrize("E,pool,max_run", [(2, 7, 3), (4, 5, 8), (3, 42, 2), (8, 4, 1)])
def test_extent_tier_invariants_and_plan_delivers_every_missed_page(E, pool, max_run):
    """Random traces: what the plan reads, followed literally on the file image, must put every
    missed page's bytes into the pool; the bookkeeping obeys the cache invariants; the runs
    are the maximal ones."""
    L, U, NP, nbytes = 2, 3, 19, 8
    NE = -(-NP // E)
    pages = RNG.integers(0, 256, size=(L, U, NP, nbytes), dtype=np.uint8)
    positions = [[orc.extent_positions(NP, [np.nonzero(a == c)[0] for c in range(4)])
                  for a in RNG.integers(0, 4, size=(U, NP))] for _ in range(L)]
    image = [orc.extent_file_image(pages[l], positions[l], E).reshape(U * NE, E, nbytes) for l in range(L)]
    tier = orc.ExtentTier(U, NP, E, pool, max_run)
    pool_bytes = {}
    reads_of = {}
    for t in range(60):
        l = t % L
        missed = []
        budget = pool                                            # a step may not need more extents than the pool holds
        for u in range(U):
            n = int(RNG.integers(0, 4))
            pg = sorted(RNG.choice(NP, size=n, replace=False).tolist())
            ext = {positions[l][u][p] // E for p in pg}
            if len(ext) > budget:
                pg = []
                ext = set()
            budget -= len(ext)
            missed.append(pg)
        before = set(tier.stamp)
        stamps_before = dict(tier.stamp)
        got = tier.fetch(l, t, missed, positions[l])
        need = set(got["needed"])
        assert set(got["hits"]) == need & before and set(got["reads"]) == need - before
        assert set(got["evicted"]) <= before - need
        assert len(got["evicted"]) == max(0, len(before) + len(got["reads"]) - pool)
        assert set(tier.stamp) == (before - set(got["evicted"])) | need and len(tier.stamp) <= pool
        assert all(tier.stamp[g] == t for g in need)
        if got["evicted"]:                                           # nothing older stays behind
            kept_old = [(tier.stamp[g], g) for g in set(tier.stamp) - need]
            gone = max((s, g) for g, s in stamps_before.items() if g in got["evicted"])
            assert all(x > gone for x in kept_old)
        flat = [first + i for first, n in got["runs"] for i in range(n)]
        assert flat == got["reads"]
        for (f0, n0), (f1, n1) in zip(got["runs"], got["runs"][1:]):
            assert not (f0 + n0 == f1 and f0 // NE == f1 // NE and n0 < max_run)
        assert all(1 <= n <= max_run and (f // NE) == ((f + n - 1) // NE) for f, n in got["runs"])
        for g in got["evicted"]:
            del pool_bytes[g]
        for first, n in got["runs"]:                                  # one sequential read of n extents
            base = l * U * NE
            chunk = image[l][first - base:first - base + n]
            for i in range(n):
                pool_bytes[first + i] = chunk[i]
                reads_of[first + i] = reads_of.get(first + i, 0) + 1
        for u in range(U):
            for p in missed[u]:
                place = positions[l][u][p]
                g = tier.extent_of(l, u, place)
                assert np.array_equal(pool_bytes[g][place % E], pages[l, u, p])
    if pool >= L * U * NE:
        assert max(reads_of.values()) == 1                           # nothing is ever read twice
