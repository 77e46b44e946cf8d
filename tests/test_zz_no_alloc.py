"""kvd_sparse_decode_attn_noalloc (the attention stage for callers that cannot allocate) against
kvd_sparse_decode_attn on the same pool, selection and slots, through the C ABI: two calls in a
row on the library's one scratch array, the second with a smaller input; page sizes of both
attention kernels; the refusal of sizes beyond the array."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2605_18071_amd import kvd as K
from paper_2605_18071_amd import workloads as W

pytestmark = pytest.mark.gpu
TOL = 2e-3          # max over rows of |a - b|_inf / max(|b|_inf, 1e-6): the bar of the attention parity tests


def _rel(got: torch.Tensor, want: torch.Tensor) -> float:
    g, w = got.double().flatten(0, -2), want.double().flatten(0, -2)
    return float(((g - w).abs().amax(dim=1) / w.abs().amax(dim=1).clamp_min(1e-6)).max())


def _filled_context(page, dtype, batch, seq_lens):
    """A context after two steps from a cold cache: pool, selection and slots as the library left them."""
    from tests.gpu_rig import Rig
    w = W.Workload(name="noalloc", n_layers=1, batch=batch, ctx=page * 200, page=page, n_q_heads=8, n_kv_heads=2,
                   dtype=dtype, topk_pages=48, capacity=96, steps=2, importance="planted", heavy_count=6, seed=23)
    rig = Rig(w, seq_lens=seq_lens, micro_batches=1)
    qs = [q[0].contiguous() for q in W.query_stream(w, rig.q0, 2, "cuda")]
    for t, q in enumerate(qs):
        rig.step(0, t, q)
    return w, rig, qs[-1]


@pytest.mark.parametrize("page,dtype", [(16, "bf16"), (32, "f16"), (8, "bf16")])
def test_noalloc_attention_matches_the_context_entry_point_twice_in_a_row(page, dtype):
    B = 5
    seq_lens = [page * 200, page * 200 - 3, page * 150 + 1, page * 200, page * 97]
    w, rig, q = _filled_context(page, dtype, B, seq_lens)
    dev = "cuda"
    seq = torch.tensor(seq_lens, dtype=torch.int32, device=dev)
    want = torch.empty_like(rig.out)
    want_lse = torch.empty_like(rig.lse)
    rig.kvd.sparse_decode_attn(0, q, rig.sel_pages, rig.sel_slots, want, want_lse)
    torch.cuda.synchronize()
    shape = dict(n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, page_size=w.page, topk_pages=w.topk_pages,
                 capacity_max=w.capacity, kv_dtype=w.torch_dtype)
    # first call: the whole batch
    got = torch.full_like(want, float("nan"))
    got_lse = torch.full_like(want_lse, float("nan"))
    K.sparse_decode_attn_noalloc(q, rig.pool[0], rig.sel_pages, rig.sel_slots, seq, got, got_lse, batch=B, **shape)
    # second call, at once, on the same scratch: the first two sequences only
    small = torch.full_like(want[:2], float("nan"))
    small_lse = torch.full_like(want_lse[:2], float("nan"))
    K.sparse_decode_attn_noalloc(q[:2].contiguous(), rig.pool[0], rig.sel_pages, rig.sel_slots, seq, small, small_lse,
                                 batch=2, **shape)
    torch.cuda.synchronize()
    assert torch.isfinite(got).all() and torch.isfinite(small).all()
    e1, e2 = _rel(got, want), _rel(small, want[:2])
    l1 = float((got_lse - want_lse).abs().max())
    l2 = float((small_lse - want_lse[:2]).abs().max())
    print(f"page {page} {dtype}: full batch rel {e1:.2e} lse {l1:.2e}; two sequences rel {e2:.2e} lse {l2:.2e}")
    assert e1 <= TOL and e2 <= TOL
    assert l1 <= 1e-3 and l2 <= 1e-3
    # a third call with another split factor still agrees (more partials in the same array)
    again = torch.full_like(want, float("nan"))
    K.sparse_decode_attn_noalloc(q, rig.pool[0], rig.sel_pages, rig.sel_slots, seq, again, None, batch=B,
                                 attn_splits=3, **shape)
    torch.cuda.synchronize()
    assert _rel(again, want) <= TOL
    rig.kvd.close()


def test_noalloc_attention_refuses_what_does_not_fit():
    lib = K.load()
    dev = "cuda"
    x = torch.zeros(4096, dtype=torch.int32, device=dev)
    f = torch.zeros(4096, dtype=torch.float32, device=dev)
    args = lambda **kw: dict(dict(batch=1, n_q_heads=8, n_kv_heads=2, page_size=16, topk_pages=4, capacity_max=8,
                                  kv_dtype=K.KVD_BF16), **kw)
    def status(**kw):
        try:
            K.sparse_decode_attn_noalloc(x, x, x, x, x, f, None, **args(**kw))
        except K.KvdError as e:
            return e.status
        return K.OK
    # 8192 units x 64 splits x 8 heads of partials: far beyond the 8 MiB array
    assert status(batch=8192, n_q_heads=8, n_kv_heads=1, topk_pages=2048, attn_splits=64) == K.ERR_CAPACITY
    assert status(n_q_heads=18) == K.ERR_SHAPE            # G = 9
    assert status(page_size=0) == K.ERR_SHAPE
    assert status(kv_dtype=5) == K.ERR_DTYPE
    assert lib.kvd_sparse_decode_attn_noalloc(None, None, None, None, None, None, None, 1, 8, 2, 16, 4, 8, 1, 0.0, 0, None) == K.ERR_ARG
