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

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from tests import gpu_rig as R

FULL = {
    2: (W.CONFIGS[2].replace(n_layers=2, physical_layers=2), 12, [(0, 0, 0), (0, 3, 5), (1, 7, 7), (1, 4, 2)]),
    3: (W.CONFIGS[3], 32, [(0, 0, 0), (0, 5, 3), (0, 9, 6), (0, 15, 7)]),
    4: (W.CONFIGS[4].replace(n_layers=2, physical_layers=2), 10, [(0, 0, 0), (0, 31, 3), (1, 13, 1), (1, 20, 2)]),
    5: (W.CONFIGS[5], 16, [(0, 0, 0), (0, 1, 4), (0, 3, 7)]),
}


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


@pytest.mark.parametrize("cfg,mb", [(3, 0), (3, 1), (2, 0), (4, 0), (5, 0), (5, -1)])
def test_full_size_sampled_parity(cfg, mb):
    """mb = 0: the form the library chooses (what bench.py times: one launch for cfg2-4, the chain of
    kernels for cfg5); 1: the chain of kernels; -1: one launch."""
    w, steps, sample = FULL[cfg]
    print(f"[cfg{cfg}] building workload", flush=True)
    rig = R.Rig(w, micro_batches=mb)
    print(f"[cfg{cfg}] workload ready, building oracle units", flush=True)
    units = [R.OracleUnit(rig, l, b, h) for (l, b, h) in sample]
    rep = R.run_steps(rig, units, steps, check_dir_every=max(1, steps // 3), progress=f"cfg{cfg}-full")
    assert rep.unit_steps == steps * len(sample)
    assert rep.tie_divergences <= 2
    st = rig.kvd.stats()
    assert st.hits + st.misses == steps * w.n_layers * w.units * w.topk_pages
    print(f"[cfg{cfg}] hit rate over the whole batch {st.hits / (st.hits + st.misses):.3f}, "
          f"max attention rel err {rep.max_attn_err:.2e}, max score err {rep.max_score_err:.2e}, "
          f"tie divergences {rep.tie_divergences}", flush=True)
    rig.close()
    del rig
    torch.cuda.empty_cache()
