"""Full-size GPU parity: the benchmark workloads at their real shapes, in the launch configuration
bench.py times, compared with the fp64 oracle on sampled output columns (all rows x 48 seeded
columns of Y and of dX; Hs/Gs enter through them; every task's dA_t, dB_t, d delta_t in full, dl_t on
the sampled columns)."""
import numpy as np
import pytest

import mux_workloads as wlm
from tests import mux_harness as hz

pytestmark = pytest.mark.gpu

CASES = [(1, 0), (1, 4), (1, 6), (2, 0), (2, 6), (3, 0), (3, 4), (3, 6), (4, 0), (4, 3), (4, 4), (4, 6),
         (5, 0),     # 5: the extra workload with two Adapter-Tuning tasks (their rows need x W in full: one projection)
         (6, 0), (6, 6)]   # 6: the extra workload with two Diff-Pruning tasks (d delta_t in full)


@pytest.fixture(scope="module")
def env():
    import torch
    import paper_2603_02885_amd as mx
    assert torch.cuda.is_available()
    mx.load_library()
    return mx, torch


@pytest.mark.parametrize("cfg,layer", CASES)
def test_benchmark_config_layer(env, cfg, layer):
    mx, torch = env
    from oracle import segtab
    wl = wlm.config(cfg)
    name, K, N = wl.layers[layer]
    print(f"config {cfg} layer {name} K={K} N={N}", flush=True)
    ot = segtab.build([t.seq_lens for t in wl.tasks], wl.chunk)
    lt = wlm.layer_tensors(wl, layer, ot.T, seed=cfg, pad_rows=ot.row_task < 0, pad_fill=1e30)
    rng = np.random.default_rng(1000 * cfg + layer)
    cols = np.sort(rng.choice(N, size=48, replace=False)).astype(np.int32)
    kcols = np.sort(rng.choice(K, size=48, replace=False)).astype(np.int32)
    g = hz.GpuLayer(mx, torch, wl, lt, mx.MUX_DT_BF16)
    assert np.array_equal(mx.mux_segtab_serialize(g.st), ot.image)
    g.forward()
    g.backward()
    got = g.results(cols=cols, kcols=kcols)
    pad = ot.row_task < 0
    assert np.all(got["Y"][pad] == 0) and np.all(got["dX"][pad] == 0)
    ref = hz.oracle_results(wl, lt, ot.row_task, cols=cols, kcols=kcols)
    errs = hz.compare(got, ref, hz.TOL_BF16, cols=cols, kcols=kcols, label=f"config{cfg}.{name}")
    print({k: float(f"{v:.2e}") for k, v in list(errs.items())[:6]}, flush=True)
    del g
    torch.cuda.empty_cache()
