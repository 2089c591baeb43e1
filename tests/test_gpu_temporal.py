"""GPU tests of temporal multiplexing (section 3.3): hybrid tasks whose calls interleave in time on one GPU, and
micro-batches of one hybrid task whose adapter gradients accumulate over the calls."""
import numpy as np
import pytest

import mux_workloads as wlm
from tests import mux_harness as hz
from tests.test_gpu_parity import diff_workload, mixed_workload, oracle_table, tuning_workload

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    import paper_2603_02885_amd as mx
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    mx.load_library()
    return mx, torch


def all_kinds_tasks():
    """Every adapter kind, several sequences per task so that the batch splits into micro-batches."""
    return [wlm.Task(wlm.KIND_LORA, 16, 2.0, [100, 31, 64, 17, 80, 45]),
            wlm.Task(wlm.KIND_IA3, 0, 1.0, [70, 30, 45, 12]),
            wlm.Task(wlm.KIND_ADAPTER, 24, 0.5, [50, 21, 90]),
            wlm.Task(wlm.KIND_DIFF, 0, 1.0, [33, 120, 64, 9, 40], density=0.03),
            wlm.Task(wlm.KIND_NONE, 0, 1.0, [64, 10]),
            wlm.Task(wlm.KIND_LORA, 40, 1.0, [5, 200])]


@pytest.mark.parametrize("C", [2, 4])
def test_microbatch_gradient_accumulation(env, C):
    """The sequences of every task are dealt to C micro-batches; each micro-batch is one forward/backward call with
    its own table, the adapter gradients accumulating from the second call on.  They must equal the oracle's gradients
    of all rows at once (every task's loss is a sum over its rows), and each call's Y and dX the oracle's rows."""
    mx, torch = env
    import oracle
    K, N, chunk = 192, 160, 32
    tasks = all_kinds_tasks()
    wls, ots, lts, gs = [], [], [], []
    for c in range(C):
        tc = [wlm.Task(t.kind, t.rank, t.scale, t.seq_lens[c::C], density=t.density) for t in tasks]
        wl = wlm.Workload(name=f"mb{c}", layers=[("w", K, N)], tasks=tc, chunk=chunk, sigma_w=0.08, sigma_ab=0.08)
        ot = oracle_table(wl)
        lt = wlm.layer_tensors(wl, 0, ot.T, seed=100 + c, bf16=True, pad_rows=ot.row_task < 0, pad_fill=1e30)
        if c > 0:           # one set of weights, adapters and masks for all micro-batches
            lt.W, lt.A, lt.B, lt.L, lt.masks = lts[0].W, lts[0].A, lts[0].B, lts[0].L, lts[0].masks
        wls.append(wl); ots.append(ot); lts.append(lt)
    for c in range(C):
        g = hz.GpuLayer(mx, torch, wls[c], lts[c], mx.MUX_DT_BF16)
        assert np.array_equal(mx.mux_segtab_serialize(g.st), ots[c].image)
        if c > 0:
            g.dA, g.dB, g.dL = gs[0].dA, gs[0].dB, gs[0].dL
        gs.append(g)
    for c, g in enumerate(gs):
        print(f"micro-batch {c}: {g.T} rows", flush=True)
        g.forward()
        g.backward(accumulate=1 if c > 0 else 0)
    kinds, ranks, scales = [t.kind for t in tasks], [t.rank for t in tasks], [t.scale for t in tasks]
    # the oracle on all rows of all micro-batches at once
    X = np.concatenate([lt.X for lt in lts]); dY = np.concatenate([lt.dY for lt in lts])
    row_task = np.concatenate([ot.row_task for ot in ots])
    l0 = lts[0]
    ref = oracle.backward(X, dY, l0.W, row_task, kinds, ranks, scales, l0.A, l0.B, l0.L, S=l0.masks)
    fwd = oracle.forward(X, l0.W, row_task, kinds, ranks, scales, l0.A, l0.B, l0.L, S=l0.masks)
    got = gs[0].results()
    r0 = 0
    errs = {}
    for c, g in enumerate(gs):
        gc = g.results()
        errs[f"Y{c}"] = hz.norm_err(gc["Y"], fwd["Y"][r0:r0 + g.T])
        errs[f"dX{c}"] = hz.norm_err(gc["dX"], ref["dX"][r0:r0 + g.T])
        r0 += g.T
    for name in ("dA", "dB", "dL"):
        for t, r in enumerate(ref[name]):
            if r is not None:
                errs[f"{name}[{t}]"] = hz.norm_err(got[name][t], r)
    bad = {k: v for k, v in errs.items() if not (v <= hz.TOL_BF16)}
    assert not bad, bad


def test_two_hybrid_tasks_on_two_streams(env):
    """Two hybrid tasks (two tables, two sets of buffers) whose forward and backward calls alternate on two streams
    give, bit for bit, what each gives alone on one stream."""
    mx, torch = env
    cases = []
    for wl, seed in ((mixed_workload(K=320, N=200), 1), (tuning_workload(K=320, N=200), 2), (diff_workload(), 3)):
        ot = oracle_table(wl)
        lt = wlm.layer_tensors(wl, 0, ot.T, seed=seed, bf16=True, pad_rows=ot.row_task < 0, pad_fill=1e30)
        g = hz.GpuLayer(mx, torch, wl, lt, mx.MUX_DT_BF16)
        g.forward(); g.backward()
        torch.cuda.synchronize()
        keep = {"Y": g.Y.clone(), "dX": g.dX.clone(),
                "grads": [None if t is None else t.clone() for k in ("dA", "dB", "dL") for t in getattr(g, k)]}
        cases.append((g, keep))
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]          # default priority
    for rep in range(4):
        for g, _ in cases:
            g.Y.fill_(float("nan")); g.dX.fill_(float("nan"))
            for k in ("dA", "dB", "dL"):
                for t in getattr(g, k):
                    if t is not None:
                        t.fill_(float("nan"))
        for s in streams:
            s.wait_stream(torch.cuda.current_stream())
        for i, (g, _) in enumerate(cases):                          # forward calls alternate between the streams
            with torch.cuda.stream(streams[i % 2]):
                g.forward()
        for i, (g, _) in enumerate(cases):
            with torch.cuda.stream(streams[i % 2]):
                g.backward()
        for s in streams:
            torch.cuda.current_stream().wait_stream(s)
        torch.cuda.synchronize()
        for g, keep in cases:
            assert torch.equal(g.Y, keep["Y"]) and torch.equal(g.dX, keep["dX"]), f"repeat {rep}"
            now = [t for k in ("dA", "dB", "dL") for t in getattr(g, k)]
            for a, b in zip(keep["grads"], now):
                assert a is None or torch.equal(a, b), f"repeat {rep}"
