"""The backward entry point that allocates nothing (its workspace is a device array inside the library) against the
ordinary one: same table, same inputs, results compared bit for bit (both are deterministic and run the same kernels),
on two calls in a row, the second on a smaller input; then a call too large for the static workspace must be refused
before anything is launched."""
import numpy as np
import pytest

import mux_workloads as wlm
from tests import mux_harness as hz

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    import paper_2603_02885_amd as mx
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    mx.load_library()
    return mx, torch


def workload(tokens, K, N):
    tasks = [wlm.Task(wlm.KIND_LORA, 16, 2.0, [tokens[0]]), wlm.Task(wlm.KIND_IA3, 0, 1.0, [tokens[1], 37]),
             wlm.Task(wlm.KIND_LORA, 40, 0.5, [tokens[2]]), wlm.Task(wlm.KIND_ADAPTER, 24, 1.5, [tokens[3]]),
             wlm.Task(wlm.KIND_NONE, 0, 1.0, [64]), wlm.Task(wlm.KIND_LORA, 8, 1.0, [])]
    return wlm.Workload(name="no_alloc", layers=[("w", K, N)], tasks=tasks, chunk=64, sigma_w=0.05, sigma_ab=0.05)


def both_ways(env, wl, seed):
    """Backward through mux_lora_backward and through mux_lora_backward_static_ws; returns the two result sets."""
    mx, torch = env
    from oracle import segtab
    ot = segtab.build([t.seq_lens for t in wl.tasks], wl.chunk, wl.max_pack_len, 0)
    lt = wlm.layer_tensors(wl, 0, ot.T, seed=seed, pad_rows=ot.row_task < 0, pad_fill=1e30)
    g = hz.GpuLayer(mx, torch, wl, lt, mx.MUX_DT_BF16)
    assert mx.mux_lora_workspace_bytes(g.layer, g.st) <= mx.MUX_STATIC_WS_BYTES
    g.forward()
    g.backward()
    a = g.results()
    # NaN into every output, then the same backward with the library's own workspace
    for t in [g.dX] + [x for x in g.dA + g.dB + g.dL if x is not None]:
        t.fill_(float("nan"))
    n0 = torch.cuda.memory_allocated()
    mx.mux_lora_backward_static_ws(g.layer, g.st, g.dtab, g.X, g.dY, g.saved, g.dX, g.dA, g.dB, g.dL, 0,
                                   torch.cuda.current_stream())
    assert torch.cuda.memory_allocated() == n0
    b = g.results()
    ref = hz.oracle_results(wl, lt, ot.row_task)
    hz.compare(b, ref, hz.TOL_BF16, label="static workspace against the oracle")
    return a, b


def same(a, b):
    assert np.array_equal(a["dX"], b["dX"])
    for name in ("dA", "dB", "dL"):
        for x, y in zip(a[name], b[name]):
            assert (x is None) == (y is None)
            if x is not None:
                assert np.array_equal(x, y), name


def test_static_workspace_backward_twice_then_too_large(env):
    mx, torch = env
    # first call: several 256-row tiles and ragged tails; second call, right after it, on a smaller input: what the
    # first one left in the array must not show
    a, b = both_ways(env, workload([700, 130, 300, 200], 320, 264), seed=3)
    same(a, b)
    a, b = both_ways(env, workload([90, 20, 33, 70], 192, 136), seed=4)
    same(a, b)
    # a call that needs more than the static workspace is refused on the host
    big = wlm.Workload(name="too_large", layers=[("w", 4096, 11008)],
                       tasks=[wlm.Task(wlm.KIND_LORA, 64, 1.0, [4096]) for _ in range(8)], chunk=512)
    st = mx.mux_segtab_build(hz.task_descs(mx, big), big.chunk, 0, 0)
    n = len(big.tasks)
    dummy = torch.zeros(256, dtype=torch.uint8, device="cuda:0")
    desc = mx.LayerDesc(4096, 11008, mx.MUX_DT_BF16, dummy, n, [dummy] * n, [dummy] * n, [None] * n)
    assert mx.mux_lora_workspace_bytes(desc, st) > mx.MUX_STATIC_WS_BYTES
    with pytest.raises(mx.MuxError) as ei:
        mx.mux_lora_backward_static_ws(desc, st, dummy, dummy, dummy, dummy, dummy, [None] * n, [None] * n, [None] * n, 0,
                                       torch.cuda.current_stream())
    assert ei.value.status == 4          # MUX_ERR_WORKSPACE
    torch.cuda.synchronize()
