"""The acceptance rules of the parity harness (tests/helpers.py) for results that may differ from
the oracle's inside the 1e-6 tie band: they must accept the oracle's own answer and an exchange of
two near-tied items, and refuse everything else.  No GPU needed."""
import numpy as np

from oracle import kvd_oracle as orc
from tests import helpers as H


def _scores():
    # 12 pages; pages 4 and 9 tie within 4e-7 at the k-th place for k = 5
    s = np.array([0.1, 0.9, 0.2, 0.8, 0.5, 0.05, 0.7, 0.6, 0.15, 0.5 + 4e-7, 0.3, 0.25])
    return s


def test_selection_rule_accepts_the_oracle_and_a_near_tie_only():
    s, k = _scores(), 5
    own = orc.select_pages(s, k)
    assert own.tolist() == [1, 3, 6, 7, 9]
    assert H.selection_is_valid(s, own, k)[0]
    swap = np.array([1, 3, 4, 6, 7], dtype=np.int32)                  # 4 instead of 9: inside the band
    assert H.selection_is_valid(s, swap, k)[0]
    for bad in ([1, 3, 6, 7, 10],                                     # 10 scores far below the k-th
                [1, 3, 4, 7, 9],                                      # 6 (clearly above) left out
                [1, 3, 6, 7, -1],                                     # one page short
                [3, 1, 6, 7, 9],                                      # not ascending
                [1, 3, 6, 7, 7],                                      # a page twice
                [1, 3, 6, 7, 12]):                                    # out of range
        assert not H.selection_is_valid(s, np.array(bad, dtype=np.int32), k)[0], bad
    # forced pages: sink 1, recent 2 -> pages 0, 10, 11 must be in whatever they score
    own_f = orc.select_pages(s, k, 1, 2)
    assert own_f.tolist() == [0, 1, 3, 10, 11] and H.selection_is_valid(s, own_f, k, 1, 2)[0]
    assert not H.selection_is_valid(s, np.array([1, 3, 6, 10, 11], dtype=np.int32), k, 1, 2)[0]   # sink page missing
    # fewer valid pages than k: everything selected, padded
    short = np.array([0.3, 0.1, 0.2])
    assert H.selection_is_valid(short, np.array([0, 1, 2, -1, -1], dtype=np.int32), 5)[0]
    assert not H.selection_is_valid(short, np.array([0, 1, -1, -1, -1], dtype=np.int32), 5)[0]
    assert not H.selection_is_valid(short, np.array([0, 1, 2, -1, 0], dtype=np.int32), 5)[0]


def test_eviction_rule_accepts_the_oracle_and_a_near_tie_only():
    s = _scores()
    cands = [0, 2, 4, 5, 8, 9, 10]                                    # scores .1 .2 .5 .05 .15 .5+ .3
    win = orc.LookaheadWindow(7)
    win.warm(cands)
    _, _, own = win.resolve([1, 3, 6], 0, scores=s)                   # three come in: the three lowest leave
    assert own == [0, 5, 8] and H.eviction_is_valid(s, cands, own, 3)[0]
    assert not H.eviction_is_valid(s, cands, [0, 5, 2], 3)[0]         # 2 (0.2) instead of 8 (0.15): outside the band
    assert not H.eviction_is_valid(s, cands, [0, 5], 3)[0]            # too few
    assert not H.eviction_is_valid(s, cands, [0, 5, 5], 3)[0]         # twice the same
    assert not H.eviction_is_valid(s, cands, [0, 5, 1], 3)[0]         # 1 is not a candidate
    # six must leave: the cut falls between 4 (0.5) and 9 (0.5 + 4e-7): either may stay
    assert H.eviction_is_valid(s, cands, [0, 2, 4, 5, 8, 10], 6)[0]
    assert H.eviction_is_valid(s, cands, [0, 2, 5, 8, 9, 10], 6)[0]
    assert H.eviction_is_valid(s, cands, cands, 7)[0] and H.eviction_is_valid(s, cands, [], 0)[0]


def test_pooled_eviction_rule_accepts_the_oracle_and_near_ties_only():
    # scores, best first: 1 .9 | 3 .8 | 6 .7 | 7 .6 | 9 .5+4e-7 | 4 .5 | 10 .3 | 11 .25 | 2 .2 | 8 .15 | 0 .1 | 5 .05
    s = _scores()
    cands = [0, 2, 4, 5, 8, 9, 10]
    stamps = {0: 3, 2: 1, 4: 5, 5: 2, 8: 4, 9: 0, 10: 6}

    def own(pool, st):
        win = orc.LookaheadWindow(7, pool=pool)
        win.stamp.update(st)
        return win.resolve([1, 3, 6], 7, scores=s)[2]                 # three come in, the window is full: three leave

    # pool of 7 = {1, 3, 6, 7, 9, 4, 10}: outside it 2, 5, 0, 8 in stamp order -> 2, 5, 0 leave
    got = own(7, stamps)
    assert got == [0, 2, 5] and H.pooled_eviction_is_valid(s, stamps, cands, got, 3, 7)[0]
    assert not H.pooled_eviction_is_valid(s, stamps, cands, [0, 2, 8], 3, 7)[0]      # 8 (stamp 4) before 0 (stamp 3): wrong order
    assert not H.pooled_eviction_is_valid(s, stamps, cands, [0, 2, 10], 3, 7)[0]     # a pool page while outside ones remain
    assert not H.pooled_eviction_is_valid(s, stamps, cands, [0, 2], 3, 7)[0]
    assert not H.pooled_eviction_is_valid(s, stamps, cands, [0, 2, 1], 3, 7)[0]      # not a candidate
    # pool of 10: only 0 and 5 are outside; the third victim is the pool page with the lowest score: 8 (0.15)
    got = own(10, stamps)
    assert got == [0, 5, 8] and H.pooled_eviction_is_valid(s, stamps, cands, got, 3, 10)[0]
    assert not H.pooled_eviction_is_valid(s, stamps, cands, [0, 5, 2], 3, 10)[0]     # 2 (0.2) is clearly above 8 (0.15)
    # pool of 5: its last member is 9 (0.5 + 4e-7), with 4 (0.5) just outside, inside the band.  With equal
    # stamps the pages outside leave by page number: 0, 2, 4.  Counting 4 as inside and 9 as outside
    # instead gives 0, 2, 5 (9 would be next): acceptable; 0, 2, 8 is not, in either reading.
    flat = {p: 0 for p in cands}
    got = own(5, flat)
    assert got == [0, 2, 4] and H.pooled_eviction_is_valid(s, flat, cands, got, 3, 5)[0]
    assert H.pooled_eviction_is_valid(s, flat, cands, [0, 2, 5], 3, 5)[0]
    assert not H.pooled_eviction_is_valid(s, flat, cands, [0, 2, 8], 3, 5)[0]
    # no pool: the plain rule
    assert H.pooled_eviction_is_valid(s, stamps, cands, [0, 5, 8], 3, 0)[0]
    assert not H.pooled_eviction_is_valid(s, stamps, cands, [0, 5, 2], 3, 0)[0]


def test_hierarchical_selection_rule():
    members = [np.array([0, 1, 2]), np.array([3, 4]), np.array([5, 6, 7, 8]), np.array([9, 10])]
    cs = np.array([0.2, 0.9, 0.5, 0.5 + 4e-7])                        # clusters 2 and 3 tie inside the band
    k, n = 5, 11
    own = orc.select_pages_hier(cs, members, k, n)
    assert own.tolist() == [3, 4, 5, 9, 10]                           # cluster 1, cluster 3, then the lowest page of cluster 2
    assert H.hier_selection_is_valid(cs, members, own, k, n)[0]
    other = np.array([3, 4, 5, 6, 7], dtype=np.int32)                 # cluster 2 first (inside the band), cut after three pages
    assert H.hier_selection_is_valid(cs, members, other, k, n)[0]
    for bad in ([0, 1, 2, 3, 4],                                      # cluster 0 scores clearly below the ones left out
                [3, 4, 6, 9, 10],                                     # the cut cluster does not give its lowest page
                [3, 4, 5, 9, -1],                                     # a page short of the budget
                [3, 5, 6, 9, 10],                                     # two clusters cut
                [4, 3, 5, 9, 10]):                                    # not ascending
        assert not H.hier_selection_is_valid(cs, members, np.array(bad, dtype=np.int32), k, n)[0], bad
    # forced pages are in first and do not count as members
    own_f = orc.select_pages_hier(cs, members, k, n, sink_pages=1, recent_pages=1)
    assert own_f.tolist() == [0, 3, 4, 9, 10] and H.hier_selection_is_valid(cs, members, own_f, k, n, 1, 1)[0]
    assert not H.hier_selection_is_valid(cs, members, np.array([3, 4, 5, 9, 10], dtype=np.int32), k, n, 1, 1)[0]


def test_attention_error_measure():
    want = np.array([[1.0, -2.0, 0.5], [0.0, 0.0, 1e-9]])
    assert H.attn_rel_err(want, want) == 0.0
    got = want + np.array([[0.002, 0.0, 0.0], [0.0, 0.0, 0.0]])
    assert abs(H.attn_rel_err(got, want) - 0.001) < 1e-12             # largest deviation of a row over the row's largest entry
    tiny = want + np.array([[0.0, 0.0, 0.0], [1e-9, 0.0, 0.0]])
    assert abs(H.attn_rel_err(tiny, want) - 1e-3) < 1e-9              # rows near zero are measured against 1e-6
