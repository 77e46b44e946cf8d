"""CPU-side checks of the C-ABI library: it loads, exports every symbol the header
declares, and rejects bad configurations before touching any device."""
import ctypes as C
import os
import re

import pytest

from paper_2605_18071_amd import kvd

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "kvd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(kvd_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = kvd.load()
    names = _declared()
    assert len(names) >= 20
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(kvd.EXPORTS) == names
    assert lib.kvd_abi_version() == 2
    assert lib.kvd_strerror(0) == b"ok"
    assert b"capacity" in lib.kvd_strerror(kvd.ERR_CAPACITY)


def _cfg(**kw):
    base = dict(n_layers=1, batch=1, n_q_heads=32, n_kv_heads=8, head_dim=128, page_size=16, max_pages=256,
                topk_pages=64, sink_pages=0, recent_pages=0, kv_dtype=kvd.KVD_F16, policy=0, softmax_scale=0.0,
                capacity_max=256, physical_layers=0, micro_batches=0, attn_splits=0)
    base.update(kw)
    c = kvd.KvdConfig()
    for k, v in base.items():
        setattr(c, k, v)
    return c


@pytest.mark.parametrize("kw,want", [
    (dict(head_dim=64), kvd.ERR_SHAPE),
    (dict(n_q_heads=30), kvd.ERR_SHAPE),
    (dict(n_q_heads=72), kvd.ERR_SHAPE),                    # G = 9
    (dict(page_size=0), kvd.ERR_SHAPE),
    (dict(page_size=512), kvd.ERR_SHAPE),
    (dict(topk_pages=0), kvd.ERR_SHAPE),
    (dict(topk_pages=4096), kvd.ERR_SHAPE),
    (dict(kv_dtype=7), kvd.ERR_DTYPE),
    (dict(policy=3), kvd.ERR_ARG),
    (dict(topk_pages=64, capacity_max=32), kvd.ERR_CAPACITY),
    (dict(sink_pages=40, recent_pages=40), kvd.ERR_CAPACITY),
    (dict(physical_layers=2), kvd.ERR_SHAPE),
    (dict(micro_batches=99), kvd.ERR_SHAPE),
    (dict(softmax_scale=float("nan")), kvd.ERR_ARG),
    (dict(softmax_scale=float("inf")), kvd.ERR_ARG),
    (dict(micro_batches=-2), kvd.ERR_SHAPE),
    (dict(attn_splits=65), kvd.ERR_SHAPE),
    (dict(attn_splits=-1), kvd.ERR_SHAPE),
    (dict(index_centroids=9000, max_pages=16384, capacity_max=256), kvd.ERR_SHAPE),   # more than 8192 centroids
    (dict(index_centroids=300), kvd.ERR_SHAPE),                                        # more centroids than pages
    (dict(index_centroids=64, max_pages=20000), kvd.ERR_SHAPE),                        # hierarchical index: at most 16384 pages
    (dict(index_centroids=-1), kvd.ERR_SHAPE),
    (dict(batch=9000), kvd.ERR_SHAPE),                                                 # more than 65535 units
    (dict(n_layers=0), kvd.ERR_SHAPE),
    (dict(max_pages=0), kvd.ERR_SHAPE),
    (dict(capacity_max=70000), kvd.ERR_SHAPE),
    (dict(sink_pages=-1), kvd.ERR_SHAPE),
    (dict(policy=1, lookahead_pool=-3), kvd.ERR_SHAPE),
])
def test_create_rejects_bad_config_without_a_device(kw, want):
    lib = kvd.load()
    ctx = C.c_void_p()
    cfg = _cfg(**kw)
    assert lib.kvd_create(C.byref(cfg), C.byref(ctx)) == want
    assert not ctx.value


def test_create_rejects_small_per_unit_capacity_and_null():
    lib = kvd.load()
    ctx = C.c_void_p()
    cfg = _cfg()
    caps = (C.c_int32 * 8)(*([256] * 7 + [63]))
    cfg.capacity = C.cast(caps, C.POINTER(C.c_int32))
    assert lib.kvd_create(C.byref(cfg), C.byref(ctx)) == kvd.ERR_CAPACITY
    assert lib.kvd_create(None, C.byref(ctx)) == kvd.ERR_ARG
    assert lib.kvd_create(C.byref(cfg), None) == kvd.ERR_ARG
    assert lib.kvd_destroy(None) == kvd.ERR_ARG
    assert lib.kvd_step(None, 0, 0, None, None, None, None) == kvd.ERR_ARG
    assert lib.kvd_step_layers(None, 0, 1, 0, None, None, None, None) == kvd.ERR_ARG
    assert lib.kvd_step_tiered(None, 0, 0, None, None, None, None) == kvd.ERR_ARG
    assert lib.kvd_set_step_form(None, 1) == kvd.ERR_ARG
    assert lib.kvd_step_form(None) == kvd.ERR_ARG
    caps_big = (C.c_int32 * 8)(*([256] * 7 + [257]))                  # a unit's capacity above capacity_max
    cfg.capacity = C.cast(caps_big, C.POINTER(C.c_int32))
    assert lib.kvd_create(C.byref(cfg), C.byref(ctx)) == kvd.ERR_SHAPE


def test_noalloc_attention_rejects_bad_arguments_without_a_device():
    """kvd_sparse_decode_attn_noalloc checks pointers and sizes, and refuses what cannot fit its
    fixed scratch array, before it touches any device."""
    lib = kvd.load()
    fn = lib.kvd_sparse_decode_attn_noalloc
    p = 4096                                                       # any non-null, 16-byte aligned address: never dereferenced here
    ok = dict(batch=1, hq=8, hkv=2, page=16, k=4, cmax=8, dt=kvd.KVD_BF16, scale=0.0, splits=2)

    def call(q=p, pool=p, sel=p, slots=p, seq=p, out=p, **kw):
        a = dict(ok, **kw)
        return fn(q, pool, sel, slots, seq, out, None, a["batch"], a["hq"], a["hkv"], a["page"], a["k"], a["cmax"], a["dt"],
                  a["scale"], a["splits"], None)

    assert call(q=None) == kvd.ERR_ARG and call(out=None) == kvd.ERR_ARG and call(seq=None) == kvd.ERR_ARG
    assert call(q=p + 8) == kvd.ERR_ARG                            # misaligned
    assert call(dt=9) == kvd.ERR_DTYPE
    assert call(hq=18) == kvd.ERR_SHAPE                            # G = 9
    assert call(hq=7) == kvd.ERR_SHAPE
    assert call(page=0) == kvd.ERR_SHAPE and call(page=257) == kvd.ERR_SHAPE
    assert call(k=0) == kvd.ERR_SHAPE and call(k=4096) == kvd.ERR_SHAPE
    assert call(cmax=0) == kvd.ERR_SHAPE
    assert call(splits=65) == kvd.ERR_SHAPE and call(splits=-1) == kvd.ERR_SHAPE
    assert call(scale=float("nan")) == kvd.ERR_ARG
    # 8192 units x 64 splits x 8 heads of split partials: 2 GiB, far beyond the 8 MiB array
    assert call(batch=8192, hq=8, hkv=1, k=2048, splits=64) == kvd.ERR_CAPACITY
