"""Shared test utilities: tensor <-> numpy conversion and the tie-band rule.

Nothing here computes any stage of the method; conversions use torch's own
widening casts so that they are independent of the oracle's bit-level ones.
"""
from __future__ import annotations

import math
import os

import numpy as np
import torch

from oracle import kvd_oracle as orc

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
TIE_EPS = 1e-6          # absolute band on the scaled score around the k-th score
ATTN_RTOL = 2e-3        # max |gpu - oracle| / max(|oracle row|, 1e-6) per output row


def dtype_code(torch_dtype) -> int:
    return orc.F16 if torch_dtype == torch.float16 else orc.BF16


def f64(t: torch.Tensor) -> np.ndarray:
    """Exact widening of an fp16/bf16/fp32 tensor to a float64 numpy array."""
    return t.detach().to("cpu").to(torch.float64).numpy()


def bits(t: torch.Tensor) -> np.ndarray:
    """Raw 16-bit patterns of an fp16/bf16 tensor."""
    return t.detach().to("cpu").contiguous().view(torch.int16).numpy().view(np.uint16)


def selection_is_valid(scores64: np.ndarray, sel: np.ndarray, k: int, sink: int = 0, recent: int = 0,
                       eps: float = TIE_EPS):
    """The acceptance rule for a selection that may differ from the oracle's at a
    near-tie: right size, unique, ascending, contains every page scoring above
    s* + eps and none below s* - eps, where s* is the oracle's k-th score; forced
    pages present.  Returns (ok, message)."""
    n = scores64.shape[0]
    s = np.array(scores64, dtype=np.float64)
    forced = np.zeros(n, dtype=bool)
    forced[: min(sink, n)] = True
    if recent > 0:
        forced[max(0, n - recent):] = True
    s[forced] = np.inf
    kk = min(k, n)
    got = sel[sel >= 0]
    if len(got) != kk or np.any(sel[kk:] != -1):
        return False, f"size {len(got)} != {kk} or bad padding"
    if np.any(np.diff(got) <= 0):
        return False, "not strictly ascending"
    if got.min(initial=0) < 0 or got.max(initial=0) >= n:
        return False, "page out of range"
    if kk == n:
        return True, ""
    kth = np.sort(s)[::-1][kk - 1]
    inset = np.zeros(n, dtype=bool)
    inset[got] = True
    must = s > kth + eps
    never = s < kth - eps
    if np.any(must & ~inset):
        return False, f"missing pages clearly above the k-th score: {np.nonzero(must & ~inset)[0][:8]}"
    if np.any(never & inset):
        return False, f"pages clearly below the k-th score: {np.nonzero(never & inset)[0][:8]}"
    return True, ""


def hier_selection_is_valid(cluster_scores64, members, sel, k, n_valid, sink=0, recent=0, eps: float = TIE_EPS):
    """The acceptance rule for a selection through the hierarchical index that differs from the
    oracle's at a near-tie of cluster scores: ascending unique pages with -1 padding; every forced
    page in; as many pages as the budget allows; of every cluster either all, none or (for at most
    one cluster) the lowest of its unforced pages; and no cluster that is left out or cut scores
    clearly (by more than 2 eps) above a cluster that has pages in.  Returns (ok, message)."""
    got = sel[sel >= 0]
    if np.any(np.diff(got) <= 0) or np.any(sel[len(got):] != -1):
        return False, "not ascending / bad padding"
    forced = set(range(min(sink, n_valid)))
    if recent > 0:
        forced |= set(range(max(0, n_valid - recent), n_valid))
    gs = set(int(p) for p in got)
    if not forced <= gs:
        return False, "forced pages missing"
    free = [np.array([p for p in m if int(p) not in forced], dtype=np.int64) for m in members]
    total_free = sum(len(f) for f in free)
    if len(gs) != min(k, len(forced) + total_free):
        return False, f"{len(gs)} pages selected, {min(k, len(forced) + total_free)} expected"
    owned = set(int(p) for f in free for p in f) | forced
    if not gs <= owned:
        return False, "a selected page belongs to no cluster"
    partial, s_in, s_out = 0, np.inf, -np.inf
    for c, f in enumerate(free):
        if len(f) == 0:
            continue
        n_in = sum(1 for p in f if int(p) in gs)
        if n_in:
            s_in = min(s_in, cluster_scores64[c])
        if n_in < len(f):
            s_out = max(s_out, cluster_scores64[c])
            if n_in:
                partial += 1
                if [int(p) for p in f[:n_in]] != sorted(int(p) for p in f if int(p) in gs):
                    return False, f"cluster {c} is cut but does not give its lowest pages"
    if partial > 1:
        return False, f"{partial} clusters are cut"
    if s_out > s_in + 2 * eps:
        return False, "a clearly better cluster is left out"
    return True, ""


def eviction_is_valid(scores64: np.ndarray, candidates, evicted, need: int, eps: float = TIE_EPS):
    """The acceptance rule for the victims of lookahead eviction when they differ from the
    oracle's at a near-tie: `need` distinct pages out of `candidates` (resident, not selected),
    containing every candidate scoring below v* - eps and none scoring above v* + eps, where v*
    is the need-th lowest candidate score.  Returns (ok, message)."""
    cands = sorted(int(p) for p in candidates)
    ev = sorted(int(p) for p in evicted)
    if len(ev) != need or len(set(ev)) != need:
        return False, f"{len(ev)} victims, {need} needed"
    if not set(ev) <= set(cands):
        return False, "a victim is not an unselected resident page"
    if need == 0 or need == len(cands):
        return True, ""
    v = np.sort(np.asarray([scores64[p] for p in cands]))[need - 1]
    must = {p for p in cands if scores64[p] < v - eps}
    never = {p for p in cands if scores64[p] > v + eps}
    if not must <= set(ev):
        return False, f"pages clearly below the cut stayed: {sorted(must - set(ev))[:8]}"
    if never & set(ev):
        return False, f"pages clearly above the cut left: {sorted(never & set(ev))[:8]}"
    return True, ""


def pooled_eviction_is_valid(scores64: np.ndarray, stamps: dict, candidates, evicted, need: int, pool: int,
                             eps: float = TIE_EPS):
    """The acceptance rule for the victims of lookahead eviction with a finite look-ahead pool when
    they differ from the oracle's.  Two float decisions can fall differently at a near-tie: whether
    a page belongs to the pool (its score against m*, the pool-th best score of the step) and, among
    pool pages, which score lowest.  The set is accepted iff, for some way of counting the candidates
    whose score lies within eps of m* as inside or outside the pool, it consists of the pages outside
    the pool in exact (stamp, page) order and then, if more must leave, of pool pages chosen by the
    rule of eviction_is_valid.  `stamps`: page -> stamp before the step.  Returns (ok, message)."""
    cands = sorted(int(p) for p in candidates)
    ev = [int(p) for p in evicted]
    if len(ev) != need or len(set(ev)) != need:
        return False, f"{len(ev)} victims, {need} needed"
    if not set(ev) <= set(cands):
        return False, "a victim is not an unselected resident page"
    n = scores64.shape[0]
    if pool <= 0 or pool >= n:
        return eviction_is_valid(scores64, cands, ev, need, eps)
    m_star = np.sort(scores64)[::-1][pool - 1]
    sure_in = [p for p in cands if scores64[p] > m_star + eps]
    sure_out = [p for p in cands if scores64[p] < m_star - eps]
    amb = [p for p in cands if abs(scores64[p] - m_star) <= eps]
    if len(amb) > 12:                                   # degenerate scores: every split of the tie is a reading
        return True, ""
    for mask in range(1 << len(amb)):
        inside = sure_in + [p for i, p in enumerate(amb) if (mask >> i) & 1]
        outside = sure_out + [p for i, p in enumerate(amb) if not (mask >> i) & 1]
        order = sorted(outside, key=lambda p: (stamps[p], p))
        if need <= len(order):
            if set(ev) == set(order[:need]):
                return True, ""
        elif set(order) <= set(ev):
            rest = sorted(set(ev) - set(order))
            if eviction_is_valid(scores64, inside, rest, need - len(order), eps)[0]:
                return True, ""
    return False, "no reading of the near-ties at the pool's edge gives these victims"


def attn_rel_err(got: np.ndarray, want: np.ndarray) -> float:
    """max over rows of ||got - want||_inf / max(||want||_inf, 1e-6)."""
    got = got.reshape(-1, got.shape[-1]).astype(np.float64)
    want = want.reshape(-1, want.shape[-1]).astype(np.float64)
    num = np.abs(got - want).max(axis=1)
    den = np.maximum(np.abs(want).max(axis=1), 1e-6)
    return float((num / den).max())


def parse_num(tok: str) -> float:
    tok = tok.strip()
    if tok.startswith("ln"):
        return math.log(float(tok[2:]))
    return float(tok)


def read_golden(name: str):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            rows.append([c.strip() for c in line.split("|")])
    return rows


def slot_image(page: torch.Tensor) -> torch.Tensor:
    """The 16-bit pattern a slot must hold for a host page [2, P, D] (K then V), written here
    from the documented slot layout: pages of a multiple of 16 tokens are stored as 16-token
    tiles, each a K part [chunk c][group g][token i][8 dims 32c+8g+e] followed by a V part
    [chunk c][token group g][dim i][half hh][4 tokens 4g+k] holding V[4g+k][32c+16hh+i];
    pages of 4 or 8 tokens are packed the same way, one page per slot (see below);
    any other page size keeps the host order."""
    raw = page.detach().cpu().contiguous().view(torch.int16).numpy()
    P, D = raw.shape[1], raw.shape[2]
    if P in (4, 8):
        # packed layout: K part [chunk c][group g][token t][8 dims 32c+8g+e], then V part
        # [chunk c][token group tg][dim i][half hh][4 tokens 4tg+k] holding V[4tg+k][32c+16hh+i]
        k = raw[0].reshape(P, 4, 4, 8)                                # [t, c, g, e]
        v = raw[1].reshape(P // 4, 4, 4, 2, 16)                       # [tg, k, c, hh, i]
        return torch.from_numpy(np.concatenate([k.transpose(1, 2, 0, 3).reshape(-1),
                                                v.transpose(2, 0, 4, 3, 1).reshape(-1)]).copy())
    if P % 16 != 0:
        return torch.from_numpy(raw.reshape(-1).copy())
    tiles = []
    for t in range(P // 16):
        k = raw[0, 16 * t:16 * t + 16].reshape(16, 4, 4, 8)           # [i, c, g, e]
        v = raw[1, 16 * t:16 * t + 16].reshape(4, 4, 4, 2, 16)        # [g, k, c, hh, i]
        tiles.append(k.transpose(1, 2, 0, 3).reshape(-1))             # [c, g, i, e]
        tiles.append(v.transpose(2, 0, 4, 3, 1).reshape(-1))          # [c, g, i, hh, k]
    return torch.from_numpy(np.concatenate(tiles).copy())
