"""Host-side pieces of bench.py that need no GPU: how a run's flags name the stored counter
readings, and that stored readings are only ever reported for the kernel sources they were taken on."""
import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import bench  # noqa: E402


def _args(**kw):
    base = dict(centroids=0, policy="lru", lookahead_pool=0.0, window=0.0, batch=0, page_size=0, ctx=0, tier="")
    base.update(kw)
    return argparse.Namespace(**base)


def test_traffic_variant_names_what_changes_a_launch():
    assert bench.traffic_variant(_args()) == ""
    assert bench.traffic_variant(_args(centroids=4096)) == "+centroids4096"
    assert bench.traffic_variant(_args(policy="lookahead")) == "+lookahead"
    assert bench.traffic_variant(_args(policy="lookahead", lookahead_pool=1.25)) == "+lookahead1.25"
    assert bench.traffic_variant(_args(page_size=8, ctx=65536)) == "+page8+ctx65536"
    assert bench.traffic_variant(_args(batch=4, window=2.0, tier="/tmp/x")) == "+window2+batch4+tier"


def test_stored_traffic_is_tied_to_the_kernel_sources(tmp_path, monkeypatch):
    have = bench.kernel_source_hash()
    assert len(have) == 16 and int(have, 16) >= 0
    rec = {"kernel_source_hash": have, "kernels": {"cfg3:step": {"hbm_bytes_per_launch": 552210854}}}
    f = tmp_path / "t.json"
    f.write_text(json.dumps(rec))
    monkeypatch.setattr(bench, "TRAFFIC_FILE", str(f))
    assert bench.stored_traffic("cfg3", "step") == (552210854, None)
    got, why = bench.stored_traffic("cfg3+centroids4096", "step")     # a variant never borrows the plain configuration's reading
    assert got is None and "cfg3+centroids4096" in why
    rec["kernel_source_hash"] = "0" * 16
    f.write_text(json.dumps(rec))
    got, why = bench.stored_traffic("cfg3", "step")
    assert got is None and have in why and "0" * 16 in why
    monkeypatch.setattr(bench, "TRAFFIC_FILE", str(tmp_path / "missing.json"))
    assert bench.stored_traffic("cfg3", "step") == (None, "no stored counter readings")


def test_committed_counter_readings_cover_the_configurations_or_say_why_not():
    """profiles/pmc_traffic.json either belongs to the committed kernel sources — then it has a reading
    for the one-launch step of cfg2..cfg5, each a few per cent above the algorithmic bytes — or
    bench.py reports null with both hashes."""
    from paper_2605_18071_amd import workloads as W
    for n in (2, 3, 4, 5):
        w = W.CONFIGS[n]
        alg = w.units * (w.n_pages * w.head_dim * 2 + w.topk_pages * w.page_bytes)
        got, why = bench.stored_traffic(w.name, "step")
        if got is None:
            assert "kernel sources" in why or "no counter reading" in why
        else:
            assert alg < got < 1.08 * alg, (n, got, alg)
