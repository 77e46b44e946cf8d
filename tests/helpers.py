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
