"""CPU oracle for the offloaded sparse-decode hot path of KVDrive.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain definition that the
HIP library is checked against.  It may be imported by ``tests/``, by
``__graft_entry__.smoke()`` and by the ``cpu_baseline`` leg of ``bench.py``,
and by nothing else; the product path never calls it and shares no code,
constants or helpers with it.

Everything is numpy in fp64, one (layer, sequence, KV-head) *unit* at a time,
in the order the paper gives for one decode step of one layer
(Background, "KV Cache Offloading": (1) select critical entries through the
index held in GPU memory, (2) fetch them, (3) compute sparse attention):

  page_summaries   index entry = mean key of each page          (System Overview)
  pooled_query     one query per KV head for the GQA group      (reading, see below)
  page_scores      query x index                                (Background, "retrieving the Top-K")
  select_pages     Top-K pages, sink/local pages always kept    (Background; Experiment "Baselines")
  LruWindow        the in-GPU window of recently critical pages (Motivation "critical KV window";
                   with LRU replacement                          Cache Management: LRU is the baseline policy)
  LookaheadWindow  the same window with the paper's own policy:  (Cache Management, "Sliding Window w/
                   the lowest current-step scores leave          Lookahead Eviction")
  attend           softmax attention over the selected tokens   (System Overview, step 3)
  kmeans_centroids the hierarchical index: page means grouped   (System Overview: the page means form
  select_pages_hier  into centroids; selection over centroids    higher-level centroids for similarity grouping)
  extent_positions the third tier: the layout of the backing    (SSD-Aware Layout Planning)
  extent_file_image  file, and which extents a step reads       (Parallel Sparse Synchronization, (b) and (c))
  ExtentTier

Readings taken where the paper is silent (each one is also listed in the design
notes of the repository):
  * the page representative is the mean over the page's *valid* tokens, per KV
    head, rounded once to the KV dtype (the index is stored in that dtype);
  * the G query heads of a GQA group are mean-pooled into one query;
  * score = pooled_query . summary / sqrt(D)   (same scale as attention logits);
  * ties in the Top-K go to the lower page index;
  * sink / recent pages are selected unconditionally and count inside k;
  * every selected page gets stamp = step index; LRU victim = smallest
    (stamp, page) among resident pages that are not selected in this step;
  * lookahead eviction ranks resident pages by the page score of the current
    step (the only importance known for pages outside the selection); the
    victim is the lowest-scoring resident page not selected in this step, and
    among equal scores the higher page index leaves first (the reverse of the
    selection order).  The look-ahead pool of the evaluation (M = 2560 for
    K = 2048) is read as "all scored pages": with every page score at hand a
    finite pool only coarsens the order beyond rank M.

  * hierarchical index: Lloyd's k-means over the page summaries of a unit (the
    paper names k-means clustering and a number of centroids, nothing more):
    squared Euclidean distance, ties to the lower centroid index, initial
    centroids = the pages at evenly spaced positions, a fixed number of
    iterations, an empty cluster keeps its centroid; a cluster's representative
    is the mean of its pages' summaries in ascending page order, rounded once to
    the KV dtype.  Selection ranks clusters by centroid score (ties to the lower
    cluster) and takes whole clusters until the page budget k is used up; the
    first cluster that does not fit gives its lowest pages; sink / recent pages
    are in unconditionally and are left out of the clusters' count.  With this
    index a step scores clusters, not pages: lookahead eviction then takes the
    score of a page's cluster as the page's score (equal scores, i.e. pages of
    one cluster: the higher page leaves first, as before).

  * third tier: the backing file holds every page; a unit's pages sit in one
    contiguous segment (layer-head partitioning), cut into extents of a fixed
    number of pages; inside the segment the pages are ordered cluster by cluster
    of the hierarchical index (cluster ascending, page ascending within; pages
    of no cluster last), or in page order when there is no such index.  Host
    DRAM holds a bounded pool of whole extents.  A step asks for the pages that
    missed in the GPU window; an extent that holds one of them and is not in the
    pool is read whole; runs of extents that are neighbours in the file, within
    one segment, are one read, up to a maximal run length.  The paper names no
    replacement rule for the DRAM tier: LRU over extents is used, victim =
    smallest (stamp, extent) among pooled extents that this step does not need.

Parity status.  select/LRU/attend/summaries are pinned in tests by brute force,
closed forms, library routines and hand-worked fixtures (tests/golden).
Fidelity to numbers *printed in the paper* is "parity unpinned": the paper
prints no worked numeric example for this path.
"""
from __future__ import annotations

import numpy as np

F16 = 0
BF16 = 1

# (exponent bits, stored mantissa bits) of the two KV dtypes
_FORMAT = {F16: (5, 10), BF16: (8, 7)}


# --------------------------------------------------------------------------- #
# exact dtype conversions
# --------------------------------------------------------------------------- #
def bits_to_f64(bits, dtype):
    """Widen fp16 / bf16 bit patterns (uint16) to fp64.  Exact."""
    bits = np.asarray(bits, dtype=np.uint16)
    if dtype == F16:
        return bits.view(np.float16).astype(np.float64)
    if dtype == BF16:
        return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    raise ValueError("dtype")


def round_f64(x, dtype):
    """Round fp64 values to the nearest fp16 / bf16 value (ties to even), in one
    rounding, and return them still as fp64.

    The quantum of a binary format at magnitude 2^(e-1) <= |x| < 2^e is
    2^(e-1-mbits), never below the subnormal quantum; x / quantum is an exact
    power-of-two scaling, and rint rounds half to even.
    """
    ebits, mbits = _FORMAT[dtype]
    bias = (1 << (ebits - 1)) - 1
    x = np.asarray(x, dtype=np.float64)
    _, e = np.frexp(x)                                   # |x| in [2^(e-1), 2^e)
    qexp = np.maximum(e - 1 - mbits, 1 - bias - mbits)   # clamp at the subnormal quantum
    q = np.ldexp(1.0, qexp)
    r = np.rint(x / q) * q
    max_finite = (2.0 - 2.0 ** (-mbits)) * 2.0 ** bias
    r = np.where(np.abs(r) > max_finite, np.copysign(np.inf, r), r)
    return np.where(np.isfinite(x), r, x)


def f64_to_bits(x, dtype):
    """fp64 -> fp16 / bf16 bit patterns with a single round-to-nearest-even."""
    r = round_f64(x, dtype)
    if dtype == F16:
        return r.astype(np.float16).view(np.uint16)       # exact: r is representable
    return (r.astype(np.float32).view(np.uint32) >> np.uint32(16)).astype(np.uint16)


# --------------------------------------------------------------------------- #
# index: page summaries
# --------------------------------------------------------------------------- #
def page_summaries(keys, page_size, seq_len, dtype):
    """Mean key of each page (System Overview: "the mean key of each page is
    used as its representative").

    keys    : [T_alloc, D] fp64 keys of one unit (already widened from the KV dtype)
    returns : [NPvalid, D] fp64, each entry rounded once to `dtype`;
              NPvalid = ceil(seq_len / page_size); a partial last page averages
              its valid tokens only.
    """
    P = int(page_size)
    seq_len = int(seq_len)
    n_valid = -(-seq_len // P)
    D = keys.shape[1]
    acc = np.zeros((n_valid, D), dtype=np.float64)
    count = np.zeros(n_valid, dtype=np.float64)
    first = np.arange(n_valid) * P                        # first token of each page
    for j in range(P):                                    # token order inside the page
        tok = first + j
        ok = tok < seq_len
        acc[ok] = acc[ok] + keys[tok[ok]]
        count[ok] += 1.0
    return round_f64(acc / count[:, None], dtype)


# --------------------------------------------------------------------------- #
# selection
# --------------------------------------------------------------------------- #
def pooled_query(q_group):
    """One query per KV head: the mean of the group's G query heads
    (g ascending).  q_group: [G, D] fp64."""
    G = q_group.shape[0]
    acc = np.zeros(q_group.shape[1], dtype=np.float64)
    for g in range(G):
        acc = acc + q_group[g]
    return acc / float(G)


def page_scores(qbar, summaries, scale):
    """score[p] = scale * sum_d qbar[d] * summary[p, d]
    (Background: the query is multiplied with the index representatives)."""
    return scale * (summaries @ qbar)


def select_pages(scores, k, sink_pages=0, recent_pages=0):
    """Top-K pages of one unit (Background: "retrieving only the Top-K").

    scores : [NPvalid] fp64.  Pages p < sink_pages and p >= NPvalid - recent_pages
             are always kept (Experiment, Baselines: sink and local tokens stay
             on the GPU) and count inside k.
    Order  : larger score first, ties to the lower page index.
    returns: int32 [k], ascending page index, padded with -1 if NPvalid < k.
    """
    n = int(scores.shape[0])
    s = np.array(scores, dtype=np.float64)
    forced = np.zeros(n, dtype=bool)
    forced[: min(int(sink_pages), n)] = True
    if recent_pages > 0:
        forced[max(0, n - int(recent_pages)):] = True
    if int(forced.sum()) > k:
        raise ValueError("forced pages exceed k")
    s[forced] = np.inf
    order = sorted(range(n), key=lambda p: (-s[p], p))    # (score desc, page asc)
    chosen = sorted(order[: min(k, n)])
    out = np.full(k, -1, dtype=np.int32)
    out[: len(chosen)] = chosen
    return out


# --------------------------------------------------------------------------- #
# hierarchical index: centroids over page summaries
# --------------------------------------------------------------------------- #
def kmeans_init(points, n_centroids):
    """Initial centroids: the points at evenly spaced positions
    floor((i + 1/2) * n / n_centroids), i = 0 .. n_centroids - 1."""
    n = points.shape[0]
    idx = ((np.arange(n_centroids) + 0.5) * n / n_centroids).astype(np.int64)
    return points[idx].copy()


def kmeans_distances(points, centroids):
    """Squared Euclidean distance of every point to every centroid, [n, n_centroids]."""
    pn = np.sum(points * points, axis=1)
    cn = np.sum(centroids * centroids, axis=1)
    return pn[:, None] - 2.0 * (points @ centroids.T) + cn[None, :]


def kmeans_assign(points, centroids):
    """Nearest centroid of every point; equal distances go to the lower index."""
    return np.argmin(kmeans_distances(points, centroids), axis=1).astype(np.int32)


def kmeans_update(points, assign, centroids):
    """New centroid = mean of the cluster's points, summed in ascending point order;
    a cluster without points keeps its centroid."""
    out = centroids.copy()
    for c in range(centroids.shape[0]):
        members = np.nonzero(assign == c)[0]
        if len(members) == 0:
            continue
        acc = np.zeros(points.shape[1], dtype=np.float64)
        for p in members:
            acc = acc + points[p]
        out[c] = acc / float(len(members))
    return out


def kmeans_centroids(points, n_centroids, iterations, dtype, forced_assign=None):
    """The hierarchical index of one unit (System Overview: the page means form
    higher-level centroids for similarity grouping).

    points  [NPvalid, D] fp64 page summaries.  `iterations` rounds of (assign to the
    nearest centroid, move every centroid to the mean of its pages).
    forced_assign: optional list, one assignment array per iteration, that replaces
            the oracle's own nearest-centroid decision (parity harness, after a
            distance tie inside the tolerance band).
    returns (centroids [n_centroids, D] rounded once to `dtype`,
             assign [NPvalid] int32: the cluster of every page, used for the last move,
             exact [n_centroids, D] the unrounded centroids)
    """
    cent = kmeans_init(points, n_centroids)
    assign = np.zeros(points.shape[0], dtype=np.int32)
    for it in range(int(iterations)):
        assign = kmeans_assign(points, cent) if forced_assign is None else np.asarray(forced_assign[it], dtype=np.int32)
        cent = kmeans_update(points, assign, cent)
    return round_f64(cent, dtype), assign, cent


def cluster_members(assign, n_centroids):
    """Pages of every cluster in ascending order."""
    return [np.nonzero(assign == c)[0].astype(np.int32) for c in range(n_centroids)]


def select_pages_hier(cluster_scores, members, k, n_valid, sink_pages=0, recent_pages=0):
    """Selection through the hierarchical index.

    cluster_scores [n_centroids] fp64 (scale * pooled query . centroid); members[c] the
    ascending pages of cluster c.  Clusters are taken in the order (score descending,
    cluster ascending) until k pages are used: whole clusters while they fit, then the
    lowest pages of the first one that does not.  Pages p < sink_pages and
    p >= n_valid - recent_pages are always in, are charged first, and do not count as
    members of their clusters.
    returns int32 [k] ascending pages, padded with -1.
    """
    forced = set(range(min(int(sink_pages), n_valid)))
    if recent_pages > 0:
        forced |= set(range(max(0, n_valid - int(recent_pages)), n_valid))
    if len(forced) > k:
        raise ValueError("forced pages exceed k")
    chosen = set(forced)
    budget = k - len(forced)
    order = sorted(range(len(members)), key=lambda c: (-float(cluster_scores[c]), c))
    for c in order:
        if budget <= 0:
            break
        take = [int(p) for p in members[c] if int(p) not in forced][:budget]
        chosen |= set(take)
        budget -= len(take)
    out = np.full(k, -1, dtype=np.int32)
    pages = sorted(chosen)
    out[: len(pages)] = pages
    return out


def cluster_scores_by_page(cluster_scores, members, n_pages):
    """The importance that lookahead eviction sees for a page when the index is
    hierarchical: the current-step score of the page's cluster (the only score the
    step computes).  A page of no cluster gets -inf: it leaves first.
    returns fp64 [n_pages]
    """
    out = np.full(int(n_pages), -np.inf)
    for c, pages in enumerate(members):
        out[np.asarray(pages, dtype=np.int64)] = float(cluster_scores[c])
    return out


# --------------------------------------------------------------------------- #
# the in-GPU window with LRU replacement
# --------------------------------------------------------------------------- #
class LruWindow:
    """Resident set of one unit: at most `capacity` pages, each with the step
    index at which it was last selected (Motivation: a window of recently
    critical entries kept in GPU memory; only entries outside it are fetched —
    Roofline section: "only out-of-cache critical KV entries" move).
    """

    def __init__(self, capacity):
        self.capacity = int(capacity)
        self.stamp = {}                                   # page -> step of last selection

    def warm(self, pages, stamp=-1):
        for p in pages:
            if len(self.stamp) >= self.capacity and p not in self.stamp:
                raise ValueError("warm list exceeds capacity")
            self.stamp[int(p)] = int(stamp)

    def resident(self):
        return sorted(self.stamp)

    def resolve(self, sel, step, scores=None, forced_evicted=None):
        """Process one step's selection.  Returns (hits, misses, evicted), each a
        sorted list of page indices.  Misses are inserted in ascending page
        order; when the window is full the victim is the resident page, not
        selected in this step, with the smallest (stamp, page).  `scores` and
        `forced_evicted` are not used by this policy.
        """
        sel = [int(p) for p in sel if p >= 0]
        if len(sel) > self.capacity:
            raise ValueError("k exceeds capacity")
        selset = set(sel)
        hits = sorted(p for p in sel if p in self.stamp)
        misses = sorted(p for p in sel if p not in self.stamp)
        for p in hits:
            self.stamp[p] = int(step)
        evicted = []
        for p in misses:
            if len(self.stamp) >= self.capacity:
                cands = [(s, r) for r, s in self.stamp.items() if r not in selset]
                _, victim = min(cands)
                del self.stamp[victim]
                evicted.append(victim)
            self.stamp[p] = int(step)
        return hits, misses, sorted(evicted)


class LookaheadWindow(LruWindow):
    """The window with lookahead eviction (Cache Management, "Sliding Window w/
    Lookahead Eviction": at each step the entries with the lowest current-step
    scores are discarded, as they are least likely to be reused).

    pool: the look-ahead candidate pool M of the evaluation ("Generality of
    Eviction Policy": M = 2560 entries for a budget of K = 2048), in pages; 0 =
    every scored page.  The figure the policy is motivated by counts how many of a
    step's Top-M entries are in the next step's Top-K and finds that the count
    saturates as M grows: beyond rank M the current scores say nothing more about
    reuse.  Read here as: the M best-scoring pages of the step (score descending,
    ties to the lower page) are the candidates for reuse and leave last, lowest
    score first; resident pages outside that pool leave before any of them, least
    recently selected first (smallest (stamp, page)), the order that remains when
    the score carries no information.  pool >= number of scored pages is the
    policy without a pool; a pool that is exactly the selection is LRU.
    """

    def __init__(self, capacity, pool=0):
        super().__init__(capacity)
        self.pool = int(pool)

    def pool_pages(self, scores):
        """The pages of the look-ahead pool for this step's scores, or None when the
        pool covers every scored page."""
        n = len(scores)
        if self.pool <= 0 or self.pool >= n:
            return None
        order = sorted(range(n), key=lambda p: (-float(scores[p]), p))
        return set(order[: self.pool])

    def resolve(self, sel, step, scores=None, forced_evicted=None):
        """As LruWindow.resolve, but the victim is the resident page, not selected
        in this step, that comes first in this order: pages outside the look-ahead
        pool by (stamp, page) ascending; then pool pages by the lowest
        scores[page], equal scores: the higher page index first.

        scores         [NPvalid] fp64 page scores of this step.
        forced_evicted if given, exactly these pages leave instead of the oracle's
                       own choice (used by the parity harness after a score tie
                       inside the 1e-6 band); they must be resident, unselected and
                       as many as the step has to evict.
        """
        if scores is None:
            raise ValueError("lookahead eviction needs the page scores of the step")
        sel = [int(p) for p in sel if p >= 0]
        if len(sel) > self.capacity:
            raise ValueError("k exceeds capacity")
        selset = set(sel)
        hits = sorted(p for p in sel if p in self.stamp)
        misses = sorted(p for p in sel if p not in self.stamp)
        for p in hits:
            self.stamp[p] = int(step)
        evicted = []
        if forced_evicted is not None:
            forced = sorted(int(p) for p in forced_evicted)
            need = max(0, len(self.stamp) + len(misses) - self.capacity)
            if len(forced) != need or any(p not in self.stamp or p in selset for p in forced):
                raise ValueError("forced eviction set is not admissible")
            for p in forced:
                del self.stamp[p]
            evicted = forced
            for p in misses:
                self.stamp[p] = int(step)
            return hits, misses, evicted
        pool = self.pool_pages(scores)
        for p in misses:
            if len(self.stamp) >= self.capacity:
                cands = []
                for r, st in self.stamp.items():
                    if r in selset:
                        continue
                    if pool is not None and r not in pool:
                        cands.append((0, float(st), r, r))
                    else:
                        cands.append((1, float(scores[r]), -r, r))
                victim = min(cands)[3]
                del self.stamp[victim]
                evicted.append(victim)
            self.stamp[p] = int(step)
        return hits, misses, sorted(evicted)


# --------------------------------------------------------------------------- #
# sparse attention
# --------------------------------------------------------------------------- #
def selected_tokens(sel, page_size, seq_len):
    """Token indices covered by the selected pages, valid tokens only."""
    toks = []
    for p in sel:
        if p < 0:
            continue
        lo, hi = int(p) * page_size, min((int(p) + 1) * page_size, int(seq_len))
        toks.extend(range(lo, hi))
    return np.asarray(toks, dtype=np.int64)


def attend(q_group, keys, values, scale):
    """Exact softmax attention of each query head of the group over the given
    tokens (System Overview step 3: attention over resident + fetched entries).

    q_group [G, D], keys [n, D], values [n, D] fp64.
    returns out [G, D], lse [G]   with lse = log sum_i exp(scale * q.k_i).
    """
    G, D = q_group.shape
    out = np.zeros((G, D), dtype=np.float64)
    lse = np.zeros(G, dtype=np.float64)
    for g in range(G):
        x = scale * (keys @ q_group[g])
        m = np.max(x)
        w = np.exp(x - m)
        denom = np.sum(w)
        out[g] = (w @ values) / denom
        lse[g] = m + np.log(denom)
    return out, lse


# --------------------------------------------------------------------------- #
# the third tier: backing file cut into extents, DRAM pool of extents
# --------------------------------------------------------------------------- #
def extent_positions(n_pages, members=None):
    """Place of every page in its unit's segment of the backing file (SSD-Aware
    Layout Planning: entries of one attention cluster are stored one after
    another; every {layer, head} has a segment of its own).

    members: the clusters' ascending page lists, or None for the flat index.
    returns int32 [n_pages], a permutation of 0 .. n_pages-1.
    """
    if members is None:
        return np.arange(n_pages, dtype=np.int32)
    order = [int(p) for c in members for p in c]
    inside = set(order)
    order += [p for p in range(n_pages) if p not in inside]
    if sorted(order) != list(range(n_pages)):
        raise ValueError("cluster lists are not disjoint pages of the unit")
    pos = np.empty(n_pages, dtype=np.int32)
    pos[np.asarray(order, dtype=np.int64)] = np.arange(n_pages, dtype=np.int32)
    return pos


def extent_file_image(pages, positions, extent_pages):
    """Bytes of the backing file for one layer.

    pages [U][NP][page_bytes] uint8, positions [U][NP]; every segment is padded with
    zero pages to a whole number of extents.
    returns uint8 [U][NE * extent_pages][page_bytes]
    """
    U, NP, nbytes = pages.shape
    n_ext = -(-NP // extent_pages)
    image = np.zeros((U, n_ext * extent_pages, nbytes), dtype=np.uint8)
    for u in range(U):
        for p in range(NP):
            image[u, int(positions[u][p])] = pages[u, p]
    return image


class ExtentTier:
    """Which extents the DRAM pool holds, and what a step reads from the backing
    file (Parallel Sparse Synchronization: only the blocks that the current
    queries need are transferred; requests are merged into sequential reads of
    whole extents; they land in a fixed pool of host buffers).

    An extent is named by its number in the file: ((layer * U) + unit) * NE + e.
    """

    def __init__(self, n_units, n_pages, extent_pages, pool_extents, max_run_extents):
        self.U = int(n_units)
        self.E = int(extent_pages)
        self.NE = -(-int(n_pages) // self.E)
        self.pool_extents = int(pool_extents)
        self.max_run = int(max_run_extents)
        self.stamp = {}                                   # pooled extent -> step of last use

    def extent_of(self, layer, unit, position):
        return (int(layer) * self.U + int(unit)) * self.NE + int(position) // self.E

    def fetch(self, layer, step, missed, positions):
        """One step of one layer.  missed[u]: the pages of unit u that missed in
        the GPU window; positions[u][p]: place of page p in the unit's segment.
        returns dict(needed, hits, reads, evicted, runs): ascending extent numbers;
        runs = [(first extent, count)] covering `reads` in file order.
        """
        needed = sorted({self.extent_of(layer, u, positions[u][int(p)])
                         for u in range(self.U) for p in missed[u]})
        hits = [g for g in needed if g in self.stamp]
        reads = [g for g in needed if g not in self.stamp]
        for g in hits:
            self.stamp[g] = int(step)
        n_evict = len(self.stamp) + len(reads) - self.pool_extents
        evicted = []
        if n_evict > 0:
            cands = sorted((s, g) for g, s in self.stamp.items() if g not in set(needed))
            if len(cands) < n_evict:
                raise ValueError("the step needs more extents than the pool holds")
            evicted = sorted(g for _, g in cands[:n_evict])
            for g in evicted:
                del self.stamp[g]
        for g in reads:
            self.stamp[g] = int(step)
        runs = []
        for g in reads:
            if runs:
                first, count = runs[-1]
                if g == first + count and g // self.NE == first // self.NE and count < self.max_run:
                    runs[-1] = (first, count + 1)
                    continue
            runs.append((g, 1))
        return dict(needed=needed, hits=hits, reads=reads, evicted=evicted, runs=runs)


# --------------------------------------------------------------------------- #
# one unit, one step: the three stages in the paper's order
# --------------------------------------------------------------------------- #
def decode_unit_step(q_group, summaries, keys, values, window, step, *, k, page_size,
                     seq_len, scale, sink_pages=0, recent_pages=0, forced_sel=None,
                     forced_evicted=None, centroids=None, members=None):
    """select -> fetch bookkeeping -> attend for one unit.

    q_group   [G, D] fp64 (queries already rounded to the KV dtype by the caller)
    summaries [NPvalid, D] fp64, keys/values [T, D] fp64 (the host store of this unit)
    window    LruWindow carried across steps
    forced_sel: if given, this selection replaces the oracle's own (used by the
              parity harness after a score tie inside the 1e-6 band).
    forced_evicted: likewise for the victims of a LookaheadWindow.
    centroids, members: if given, selection goes through the hierarchical index
              (cluster scores instead of page scores; `scores` in the result are then
              the cluster scores).  Lookahead eviction then ranks a resident page by
              the score of its cluster (`evict_scores` in the result, see
              cluster_scores_by_page).
    returns dict(scores, evict_scores, sel, used, hits, misses, evicted, out, lse)
    """
    qbar = pooled_query(q_group)
    n_valid = -(-int(seq_len) // int(page_size))
    if centroids is None:
        scores = page_scores(qbar, summaries, scale)
        sel = select_pages(scores, k, sink_pages, recent_pages)
        evict_scores = scores
    else:
        scores = page_scores(qbar, centroids, scale)
        sel = select_pages_hier(scores, members, k, n_valid, sink_pages, recent_pages)
        evict_scores = cluster_scores_by_page(scores, members, n_valid)
    used = sel if forced_sel is None else np.asarray(forced_sel, dtype=np.int32)
    hits, misses, evicted = window.resolve(used, step, scores=evict_scores, forced_evicted=forced_evicted)
    toks = selected_tokens(used, page_size, seq_len)
    out, lse = attend(q_group, keys[toks], values[toks], scale)
    return dict(scores=scores, evict_scores=evict_scores, sel=sel, used=used, hits=hits, misses=misses,
                evicted=evicted, out=out, lse=lse)
