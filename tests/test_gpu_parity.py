"""GPU parity: the HIP path through the C ABI against the fp64 oracle, same seeded inputs."""
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


def oracle_table(wl, seg_flags=0, max_pack_len=None):
    from oracle import segtab
    return segtab.build([t.seq_lens for t in wl.tasks], wl.chunk,
                        wl.max_pack_len if max_pack_len is None else max_pack_len, seg_flags)


def run_case(env, wl, layer=0, seed=0, dtype=None, seg_flags=0, layer_flags=0, pad_fill=1e30, cols=None, kcols=None,
             label=""):
    mx, torch = env
    dtype = mx.MUX_DT_BF16 if dtype is None else dtype
    ot = oracle_table(wl, seg_flags)
    bf16 = dtype == mx.MUX_DT_BF16
    lt = wlm.layer_tensors(wl, layer, ot.T, seed=seed, bf16=bf16, pad_rows=ot.row_task < 0, pad_fill=pad_fill)
    g = hz.GpuLayer(mx, torch, wl, lt, dtype, seg_flags=seg_flags, layer_flags=layer_flags)
    assert np.array_equal(mx.mux_segtab_serialize(g.st), ot.image)          # table bit-exact
    g.forward()
    g.backward()
    got = g.results()
    ref = hz.oracle_results(wl, lt, ot.row_task, cols=cols, kcols=kcols)
    tol = hz.TOL_BF16 if bf16 else hz.TOL_F32
    errs = hz.compare(got, ref, tol, cols=cols, kcols=kcols, label=label or wl.name)
    pad = ot.row_task < 0
    assert np.all(got["Y"][pad] == 0) and np.all(got["dX"][pad] == 0)       # padding rows written as zero
    return g, got, ref, errs


def mixed_workload(K=320, N=200, chunk=64):
    """All adapter kinds, ragged ranks and token counts, several 64-row tiles and ragged tails."""
    tasks = [wlm.Task(wlm.KIND_LORA, 8, 2.0, [100]), wlm.Task(wlm.KIND_IA3, 0, 1.0, [70, 30, 45]),
             wlm.Task(wlm.KIND_LORA, 33, 0.5, [150, 21]), wlm.Task(wlm.KIND_NONE, 0, 1.0, [64]),
             wlm.Task(wlm.KIND_LORA, 64, 1.5, [5]), wlm.Task(wlm.KIND_LORA, 16, 2.0, [])]
    return wlm.Workload(name="mixed", layers=[("w", K, N)], tasks=tasks, chunk=chunk, sigma_w=0.05, sigma_ab=0.05)


@pytest.mark.parametrize("seg_flags", [0, 1])
@pytest.mark.parametrize("mode", ["bf16", "bf16_ref", "f32"])
def test_config1_tiny(env, mode, seg_flags):
    mx, _ = env
    dtype = mx.MUX_DT_F32 if mode == "f32" else mx.MUX_DT_BF16
    lf = mx.MUX_LAYER_REFERENCE_KERNELS if mode == "bf16_ref" else 0
    for seed in (0, 1, 2):
        run_case(env, wlm.config(0), seed=seed, dtype=dtype, seg_flags=seg_flags, layer_flags=lf)


@pytest.mark.parametrize("seg_flags", [0, 1])
@pytest.mark.parametrize("mode", ["bf16", "bf16_ref", "f32"])
def test_mixed_kinds_ragged(env, mode, seg_flags):
    mx, _ = env
    dtype = mx.MUX_DT_F32 if mode == "f32" else mx.MUX_DT_BF16
    lf = mx.MUX_LAYER_REFERENCE_KERNELS if mode == "bf16_ref" else 0
    run_case(env, mixed_workload(), dtype=dtype, seg_flags=seg_flags, layer_flags=lf)
    run_case(env, mixed_workload(K=264, N=328, chunk=16), dtype=dtype, seg_flags=seg_flags, layer_flags=lf, seed=1)


def test_long_contraction_mixed_ranks(env):
    """Long contraction (64 K-tiles), ranks on both sides of 32 (one and two adapter K-tiles), all adapter kinds;
    results must match the oracle and repeat bit for bit."""
    mx, torch = env
    tasks = [wlm.Task(wlm.KIND_LORA, 16, 2.0, [300]), wlm.Task(wlm.KIND_IA3, 0, 1.0, [200]),
             wlm.Task(wlm.KIND_LORA, 40, 1.0, [129]), wlm.Task(wlm.KIND_NONE, 0, 1.0, [77])]
    wl = wlm.Workload(name="ksplit", layers=[("w", 2048, 768)], tasks=tasks, chunk=64, sigma_w=0.03, sigma_ab=0.05)
    g, got, ref, errs = run_case(env, wl)
    y1, dx1 = g.Y.clone(), g.dX.clone()
    for _ in range(3):
        g.forward(); g.backward()
        torch.cuda.synchronize()
        assert torch.equal(g.Y, y1) and torch.equal(g.dX, dx1)


def test_kernel_choice_by_shape(env):
    """Shapes that select the other kernels: contraction lengths that are multiples of 32 but not of 64 (the 32-deep
    pipelined GEMM, forward and backward), and rows that are not 16-byte aligned (the plain kernels)."""
    tasks = [wlm.Task(wlm.KIND_LORA, 8, 2.0, [90, 40]), wlm.Task(wlm.KIND_IA3, 0, 1.0, [130]),
             wlm.Task(wlm.KIND_LORA, 40, 0.5, [300]), wlm.Task(wlm.KIND_NONE, 0, 1.0, [33]),
             wlm.Task(wlm.KIND_LORA, 16, 1.0, [257])]
    wl = wlm.Workload(name="bk32", layers=[("w", 416, 352)], tasks=tasks, chunk=32, sigma_w=0.05, sigma_ab=0.05)
    run_case(env, wl, seed=3)
    wl = wlm.Workload(name="unaligned", layers=[("w", 100, 52)], tasks=tasks, chunk=16, sigma_w=0.05, sigma_ab=0.05)
    run_case(env, wl, seed=4)


@pytest.mark.parametrize("n_items", [16, 20, 23, 28])
def test_gemm_last_round_pieces(env, n_items):
    """The backbone GEMM cuts the tiles left after the last full round of workgroups (one per compute unit) into
    quarters or halves, or leaves them whole, by how many there are.  With 256 compute units and 16 column tiles the
    four row counts leave 0, 64, 112 and 192 tiles, forward and backward: nothing to cut, quarters, halves, whole
    tiles.  Ragged row items, padding rows and every adapter kind lie in the cut tiles; compared on all rows and a
    sample of the columns of Y and dX."""
    mx, torch = env
    K, N, chunk = 4096, 4096, 256
    kinds = [(wlm.KIND_LORA, 16, 2.0), (wlm.KIND_IA3, 0, 1.0), (wlm.KIND_LORA, 40, 0.5), (wlm.KIND_NONE, 0, 1.0),
             (wlm.KIND_ADAPTER, 24, 1.0)]
    # one 256-row item per chunk; the last chunk of every task is partly padding (some with fewer than 128 rows)
    per = [n_items // len(kinds) + (1 if i < n_items % len(kinds) else 0) for i in range(len(kinds))]
    tails = [100, 256, 129, 7, 200]
    tasks = [wlm.Task(k, r, sc, [chunk * (c - 1) + tails[i]]) for i, ((k, r, sc), c) in enumerate(zip(kinds, per))]
    wl = wlm.Workload(name=f"pieces{n_items}", layers=[("w", K, N)], tasks=tasks, chunk=chunk, sigma_w=0.05, sigma_ab=0.05)
    ot = oracle_table(wl)
    assert ot.T == n_items * chunk
    rng = np.random.default_rng(n_items)
    cols = np.sort(rng.choice(N, 160, replace=False))
    cols[:4] = [0, 127, 128, N - 1]
    kcols = np.sort(rng.choice(K, 160, replace=False))
    kcols[:4] = [0, 127, 128, K - 1]
    run_case(env, wl, seed=n_items, cols=np.unique(cols), kcols=np.unique(kcols))


def test_mfma_probe_runs(env):
    """The diagnostic MFMA loop: launches, reports its FLOP count, leaves finite sums (operands 1 and 0.5: every
    accumulator element of a loop turn grows by 8 products of 16 terms of 0.5), rejects bad arguments."""
    mx, torch = env
    n = mx.mux_probe_mfma_operand_bytes() // 2
    ops = torch.ones(n, dtype=torch.bfloat16, device="cuda:0")
    ops[n // 2:] = 0.5                                   # the B operands
    sink = torch.zeros(mx.mux_probe_mfma_sink_bytes() // 4, dtype=torch.float32, device="cuda:0")
    flop = mx.mux_probe_mfma(ops, sink, 3, torch.cuda.current_stream())
    torch.cuda.synchronize()
    assert flop == 512 * 4 * 3 * 64 * 2 * 32 * 32 * 16
    # a lane sums its 8 x 16 accumulator elements, each 3 turns x 8 products x 16 terms x (1 x 0.5)
    assert torch.all(sink == 8 * 16 * 3 * 8 * 16 * 0.5)
    with pytest.raises(mx.MuxError):
        mx.mux_probe_mfma(ops, sink, 0, None)
    with pytest.raises(mx.MuxError):
        mx.mux_probe_mfma(None, sink, 1, None)


def test_read_probe_runs(env):
    """The diagnostic read stream: reads every 16-byte piece once (the sink holds the sum of the words' XOR, here of
    a buffer of ones), with a ragged size, and rejects bad arguments."""
    mx, torch = env
    n_vec = 2048 * 256 * 8 * 2 + 12345                  # two full turns of the eight-deep loop and a ragged rest
    buf = torch.ones(n_vec * 4 + 3, dtype=torch.int32, device="cuda:0")
    sink = torch.zeros(mx.mux_probe_read_sink_bytes() // 4, dtype=torch.int32, device="cuda:0")
    mx.mux_probe_read(buf, n_vec * 16 + 12, sink, torch.cuda.current_stream())
    torch.cuda.synchronize()
    assert int(sink.sum().item()) == 0                  # 1 ^ 1 ^ 1 ^ 1 = 0 for every piece
    buf[::4] = 3                                        # 3 ^ 1 ^ 1 ^ 1 = 2 for every piece
    mx.mux_probe_read(buf, n_vec * 16 + 12, sink, torch.cuda.current_stream())
    torch.cuda.synchronize()
    assert int(sink.to(torch.int64).sum().item()) == 2 * n_vec
    with pytest.raises(mx.MuxError):
        mx.mux_probe_read(buf, 8, sink, None)
    with pytest.raises(mx.MuxError):
        mx.mux_probe_read(None, 1024, sink, None)


def tuning_workload(K=192, N=160, chunk=32, ranks=(8, 24)):
    """The additive bottleneck kind between the others: ragged ranks and token counts, padding, an empty task.  With
    every bottleneck width a multiple of 8 the matrix-core path reads D_t as it is stored, else a transposed copy."""
    tasks = [wlm.Task(wlm.KIND_LORA, 16, 2.0, [100]), wlm.Task(wlm.KIND_ADAPTER, ranks[0], 1.5, [70, 45]),
             wlm.Task(wlm.KIND_IA3, 0, 1.0, [33]), wlm.Task(wlm.KIND_ADAPTER, ranks[1], 0.5, [150, 21]),
             wlm.Task(wlm.KIND_NONE, 0, 1.0, [64]), wlm.Task(wlm.KIND_ADAPTER, 64, 1.0, [5]),
             wlm.Task(wlm.KIND_ADAPTER, 16, 2.0, [])]
    return wlm.Workload(name="tuning", layers=[("w", K, N)], tasks=tasks, chunk=chunk, sigma_w=0.08, sigma_ab=0.08)


@pytest.mark.parametrize("seg_flags", [0, 1])
@pytest.mark.parametrize("mode", ["bf16", "bf16_ref", "f32"])
def test_adapter_tuning_kind(env, mode, seg_flags):
    """Adapter-Tuning tasks (additive bottleneck after the BaseOp) beside LoRA, IA3 and plain tasks, in the three
    modes; a second shape whose contraction lengths select the other GEMM kernels."""
    mx, _ = env
    dtype = mx.MUX_DT_F32 if mode == "f32" else mx.MUX_DT_BF16
    lf = mx.MUX_LAYER_REFERENCE_KERNELS if mode == "bf16_ref" else 0
    run_case(env, tuning_workload(), dtype=dtype, seg_flags=seg_flags, layer_flags=lf, seed=5)
    run_case(env, tuning_workload(K=104, N=232, chunk=16), dtype=dtype, seg_flags=seg_flags, layer_flags=lf, seed=6)
    run_case(env, tuning_workload(K=256, N=192, ranks=(12, 20)), dtype=dtype, seg_flags=seg_flags, layer_flags=lf, seed=7)


def diff_workload(K=192, N=160, chunk=32, density=0.02):
    """The selective kind (masked sparse update of W) beside the others; one task with an empty mask."""
    tasks = [wlm.Task(wlm.KIND_LORA, 16, 2.0, [100]), wlm.Task(wlm.KIND_DIFF, 0, 1.0, [70, 45], density=density),
             wlm.Task(wlm.KIND_IA3, 0, 1.0, [33]), wlm.Task(wlm.KIND_DIFF, 0, 1.0, [150, 21], density=density * 4),
             wlm.Task(wlm.KIND_ADAPTER, 8, 1.0, [64]), wlm.Task(wlm.KIND_DIFF, 0, 1.0, [5], density=0.0),
             wlm.Task(wlm.KIND_DIFF, 0, 1.0, [], density=density)]
    return wlm.Workload(name="diff", layers=[("w", K, N)], tasks=tasks, chunk=chunk, sigma_w=0.08, sigma_ab=0.08)


@pytest.mark.parametrize("seg_flags", [0, 1])
@pytest.mark.parametrize("mode", ["bf16", "bf16_ref", "f32"])
def test_diff_pruning_kind(env, mode, seg_flags):
    """Diff-Pruning tasks (trainable values on a fixed sparse mask over W) beside every other kind, in the three modes,
    on two shapes."""
    mx, _ = env
    dtype = mx.MUX_DT_F32 if mode == "f32" else mx.MUX_DT_BF16
    lf = mx.MUX_LAYER_REFERENCE_KERNELS if mode == "bf16_ref" else 0
    run_case(env, diff_workload(), dtype=dtype, seg_flags=seg_flags, layer_flags=lf, seed=7)
    run_case(env, diff_workload(K=104, N=328, chunk=16, density=0.05), dtype=dtype, seg_flags=seg_flags, layer_flags=lf, seed=8)


def test_diff_pruning_routes(env):
    """The matrix-core path serves Diff-Pruning rows in one of three ways: where both contraction lengths are multiples
    of 64 the backbone products add the masked entries to their tiles of W in LDS (only a packing kernel runs beside
    them); else, by cost, the products read a merged weight W + M_t * delta_t built for the call (many rows, dense
    masks) or sparse updates follow them (few rows, thin masks).  All against the oracle, forward and backward, thin
    and dense masks (a column with many entries in one K-tile), and the kernel list shows which route ran."""
    mx, torch = env
    for K, N, density, route in ((256, 384, 0.02, "patch"), (256, 384, 0.3, "patch"), (1024, 192, 0.002, "patch"),
                                 (264, 392, 0.02, "merged"), (264, 392, 0.002, "updates")):
        for seg_flags in (0, 1):
            g, got, ref, errs = run_case(env, diff_workload(K=K, N=N, density=density), seed=9, seg_flags=seg_flags)
            mx.mux_profile_enable(1)
            mx.mux_profile_collect()
            g.forward(); g.backward()
            torch.cuda.synchronize()
            names = [e["name"] for e in mx.mux_profile_collect()]
            mx.mux_profile_enable(0)
            assert ("diff_pack" in names) == (route == "patch"), (K, N, density, names)
            assert ("diff_merge" in names) == (route == "merged"), (K, N, density, names)
            assert ("diff_fwd" in names) == (route == "updates") and ("diff_bwd" in names) == (route == "updates"), (K, N, density, names)
            assert "diff_grad" in names, names


def test_diff_pruning_routes_differ_by_direction(env):
    """A LoRA rank that is not a multiple of 8 sends the backward to the register-staged GEMM: the forward still adds
    the masked entries in its tile loop, the backward runs the sparse update after its product."""
    mx, torch = env
    tasks = [wlm.Task(wlm.KIND_LORA, 12, 2.0, [100]), wlm.Task(wlm.KIND_DIFF, 0, 1.0, [70, 45], density=0.02),
             wlm.Task(wlm.KIND_DIFF, 0, 1.0, [150, 21], density=0.08), wlm.Task(wlm.KIND_IA3, 0, 1.0, [33])]
    wl = wlm.Workload(name="diffdir", layers=[("w", 256, 384)], tasks=tasks, chunk=32, sigma_w=0.08, sigma_ab=0.08)
    g, got, ref, errs = run_case(env, wl, seed=13)
    mx.mux_profile_enable(1)
    mx.mux_profile_collect()
    g.forward(); g.backward()
    torch.cuda.synchronize()
    names = [e["name"] for e in mx.mux_profile_collect()]
    mx.mux_profile_enable(0)
    assert names.count("diff_pack") == 1 and "diff_bwd" in names and "diff_fwd" not in names and "diff_merge" not in names, names


def test_diff_pruning_gradient_by_mask_blocks(env):
    """On shapes with enough 512 x 256 blocks of the mask the masked gradient is summed block by block (the lines of
    a row block staged once per mask block): ragged last blocks in both directions, blocks with more entries than one
    pass holds, a task with an empty mask and one without rows, with and without accumulation."""
    mx, torch = env
    g, got, ref, errs = run_case(env, diff_workload(K=2112, N=1600, chunk=64, density=0.01), seed=11)
    first = [None if t is None else t.clone() for t in g.dA]
    g.backward(accumulate=1)
    torch.cuda.synchronize()
    for a, b in zip(first, g.dA):
        assert a is None or torch.allclose(b, 2 * a, rtol=1e-6, atol=0)


@pytest.mark.parametrize("which", ["mixed", "tuning", "diff"])
def test_accumulate_and_determinism(env, which):
    mx, torch = env
    wl = {"mixed": mixed_workload, "tuning": tuning_workload, "diff": diff_workload}[which]()
    g, got, ref, _ = run_case(env, wl)
    first = {k: [None if t is None else t.clone() for t in getattr(g, k)] for k in ("dA", "dB", "dL")}
    y1, dx1 = g.Y.clone(), g.dX.clone()
    g.forward(); g.backward()                     # same inputs again: bit-identical
    torch.cuda.synchronize()
    assert torch.equal(g.Y, y1) and torch.equal(g.dX, dx1)
    for k in first:
        for a, b in zip(first[k], getattr(g, k)):
            assert a is None or torch.equal(a, b)
    g.backward(accumulate=1)                      # adds to what the buffers hold
    torch.cuda.synchronize()
    for k in first:
        for a, b in zip(first[k], getattr(g, k)):
            assert a is None or torch.allclose(b, 2 * a, rtol=1e-6, atol=0)


@pytest.mark.parametrize("which", ["mixed", "tuning", "diff"])
def test_nan_isolation(env, which):
    """Poisoning one task's rows, adapters and every padding row with NaN/Inf leaves the other
    tasks' outputs and gradients bit-identical (section 3.2)."""
    mx, torch = env
    wl = {"mixed": mixed_workload, "tuning": tuning_workload, "diff": diff_workload}[which]()
    g, got, _, _ = run_case(env, wl)
    ot = oracle_table(wl)
    j = 2 if which == "mixed" else 3          # a LoRA task / an Adapter-Tuning task / a Diff-Pruning task
    rows = torch.from_numpy(ot.task_rows[j]).to("cuda:0")
    pad = torch.from_numpy(np.nonzero(ot.row_task < 0)[0]).to("cuda:0")
    g.X[rows] = float("nan"); g.dY[rows] = float("inf")
    g.X[pad] = float("nan"); g.dY[pad] = float("nan")
    g.A[j].fill_(float("nan"))
    if g.B[j] is not None:
        g.B[j].fill_(float("nan"))
    g.forward(); g.backward()
    got2 = g.results()
    for t in range(len(wl.tasks)):
        if t == j:
            continue
        r = ot.task_rows[t]
        assert np.array_equal(got2["Y"][r], got["Y"][r]) and np.array_equal(got2["dX"][r], got["dX"][r])
        for k in ("dA", "dB", "dL"):
            if got[k][t] is not None:
                assert np.array_equal(got2[k][t], got[k][t])
    p = ot.row_task < 0
    assert np.all(got2["Y"][p] == 0) and np.all(got2["dX"][p] == 0)


def test_dynamic_task_attach(env):
    """A task arriving between calls (section 3.1, register_tasks): a new table and a longer layer
    description; the tasks already there get bit-identical results."""
    mx, torch = env
    wl = mixed_workload()
    g, got, _, _ = run_case(env, wl)
    ot = oracle_table(wl)
    wl2 = mixed_workload()
    wl2.tasks = wl.tasks + [wlm.Task(wlm.KIND_LORA, 12, 1.0, [40, 40])]
    ot2 = oracle_table(wl2)
    lt2 = wlm.layer_tensors(wl2, 0, ot2.T, seed=0)
    for t in range(len(wl.tasks)):            # same data for the old tasks
        lt2.X[ot2.task_rows[t]] = g.lt.X[ot.task_rows[t]]
        lt2.dY[ot2.task_rows[t]] = g.lt.dY[ot.task_rows[t]]
        lt2.A[t], lt2.B[t], lt2.L[t] = g.lt.A[t], g.lt.B[t], g.lt.L[t]
    lt2.W = g.lt.W
    g2 = hz.GpuLayer(mx, torch, wl2, lt2, mx.MUX_DT_BF16)
    g2.forward(); g2.backward()
    got2 = g2.results()
    for t in range(len(wl.tasks)):
        assert np.array_equal(got2["Y"][ot2.task_rows[t]], got["Y"][ot.task_rows[t]])
        assert np.array_equal(got2["dX"][ot2.task_rows[t]], got["dX"][ot.task_rows[t]])
        for k in ("dA", "dB", "dL"):
            if got[k][t] is not None:
                assert np.array_equal(got2[k][t], got[k][t])
    ref2 = hz.oracle_results(wl2, lt2, ot2.row_task)
    hz.compare(got2, ref2, hz.TOL_BF16, label="attach")


def test_errors_launch_nothing(env):
    mx, torch = env
    wl = wlm.config(0)
    ot = oracle_table(wl)
    lt = wlm.layer_tensors(wl, 0, ot.T)
    g = hz.GpuLayer(mx, torch, wl, lt, mx.MUX_DT_BF16)
    with pytest.raises(mx.MuxError) as e:
        mx.mux_lora_forward(g.layer, g.st, g.dtab, g.X, g.Y, g.saved, g.ws, 16, torch.cuda.current_stream())
    assert e.value.status == 4
    with pytest.raises(mx.MuxError):
        mx.mux_lora_forward(g.layer, g.st, g.dtab, None, g.Y, g.saved, g.ws, g.ws_bytes, torch.cuda.current_stream())
    torch.cuda.synchronize()
    assert torch.isnan(g.Y.float()).all()          # nothing was written


def test_leading_dimension_packs_and_skipped_outputs(env):
    """W as a column window of a wider matrix (ldw > N), several packs per task (max_pack_len), dX and some
    gradients not requested, and an empty table."""
    mx, torch = env
    from oracle import segtab
    tasks = [wlm.Task(wlm.KIND_LORA, 16, 2.0, [40, 50, 30, 90]), wlm.Task(wlm.KIND_IA3, 0, 1.0, [64, 64, 10]),
             wlm.Task(wlm.KIND_LORA, 24, 1.0, [200])]
    wl = wlm.Workload(name="ldw", layers=[("w", 512, 384)], tasks=tasks, chunk=32, max_pack_len=100, sigma_w=0.05,
                      sigma_ab=0.05)
    ot = segtab.build([t.seq_lens for t in tasks], 32, 100)
    lt = wlm.layer_tensors(wl, 0, ot.T, seed=4, pad_rows=ot.row_task < 0, pad_fill=1e30)
    g = hz.GpuLayer(mx, torch, wl, lt, mx.MUX_DT_BF16)
    assert np.array_equal(mx.mux_segtab_serialize(g.st), ot.image)
    # re-home W inside a wider buffer and describe it with ldw
    wide = torch.full((lt.K, 640), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    wide[:, 128:128 + lt.N] = g.W
    view = wide[:, 128:128 + lt.N]
    g.layer = mx.LayerDesc(lt.K, lt.N, mx.MUX_DT_BF16, view.data_ptr(), len(tasks), g.A, g.B, g.L, ldw=640)
    g.forward(); g.backward()
    got = g.results()
    ref = hz.oracle_results(wl, lt, ot.row_task)
    hz.compare(got, ref, hz.TOL_BF16, label="ldw")
    # dX and task 0's dA not requested: the rest is unchanged, the skipped buffers untouched
    keep = g.dX.clone(); g.dX.fill_(7.0)
    dA0 = g.dA[0]; dA0.fill_(5.0)
    saved_dA = list(g.dA); g.dA = [None] + saved_dA[1:]
    before = {k: [None if t is None else t.clone() for t in getattr(g, k)] for k in ("dB", "dL")}
    g.backward(want_dx=False)
    torch.cuda.synchronize()
    assert torch.all(g.dX == 7.0) and torch.all(dA0 == 5.0)
    for k in before:
        for a, b in zip(before[k], getattr(g, k)):
            assert a is None or torch.equal(a, b)
    assert torch.equal(g.dA[2], saved_dA[2])
    # empty table: both calls return without touching anything
    st0 = mx.mux_segtab_build([mx.TaskDesc(1, 8, 1.0, [])], 64)
    A0 = [torch.zeros(lt.K, 8, dtype=torch.bfloat16, device="cuda:0")]
    B0 = [torch.zeros(8, lt.N, dtype=torch.bfloat16, device="cuda:0")]
    l0 = mx.LayerDesc(lt.K, lt.N, mx.MUX_DT_BF16, g.W, 1, A0, B0, [None])
    ws0 = torch.zeros(max(mx.mux_lora_workspace_bytes(l0, st0), 256), dtype=torch.uint8, device="cuda:0")
    dt0 = torch.zeros(max(mx.mux_segtab_device_bytes(st0), 256), dtype=torch.uint8, device="cuda:0")
    mx.mux_segtab_upload(st0, dt0, dt0.numel())
    mx.mux_lora_forward(l0, st0, dt0, keep, keep, ws0, ws0, ws0.numel())
    dA = [torch.full((lt.K, 8), 3.0, device="cuda:0")]; dB = [torch.full((8, lt.N), 3.0, device="cuda:0")]
    mx.mux_lora_backward(l0, st0, dt0, keep, keep, ws0, keep, dA, dB, [None], 0, ws0, ws0.numel())
    torch.cuda.synchronize()
    assert torch.all(dA[0] == 0) and torch.all(dB[0] == 0)      # a task without tokens has zero gradients


def test_task_table_by_value_and_in_memory(env):
    """Up to 32 tasks travel in the kernel arguments; more than that (here 40, every kind, some without rows) make the
    kernels read the table a small kernel wrote into the workspace.  Both against the oracle, and bit-identical
    repeats."""
    mx, torch = env
    rng = np.random.default_rng(77)
    kinds = [wlm.KIND_LORA, wlm.KIND_LORA, wlm.KIND_IA3, wlm.KIND_ADAPTER, wlm.KIND_NONE, wlm.KIND_DIFF]
    for n_tasks in (32, 40):
        tasks = []
        for t in range(n_tasks):
            kind = kinds[t % len(kinds)]
            rank = int(rng.choice([8, 16, 24])) if kind in (wlm.KIND_LORA, wlm.KIND_ADAPTER) else 0
            tasks.append(wlm.Task(kind, rank, 1.5, [] if t % 11 == 7 else [int(rng.integers(5, 90))],
                                  **({"density": 0.03} if kind == wlm.KIND_DIFF else {})))
        wl = wlm.Workload(name=f"many{n_tasks}", layers=[("w", 256, 192)], tasks=tasks, chunk=32, sigma_w=0.05, sigma_ab=0.05)
        g, got, ref, errs = run_case(env, wl, seed=n_tasks)
        keep = [t.clone() for t in [g.Y, g.dX] + [x for x in g.dA + g.dB + g.dL if x is not None]]
        g.forward(); g.backward()
        torch.cuda.synchronize()
        for a, b in zip(keep, [g.Y, g.dX] + [x for x in g.dA + g.dB + g.dL if x is not None]):
            assert torch.equal(a, b)


def fuse_workload(K, N, toks):
    tasks = [wlm.Task(wlm.KIND_LORA, 16, 2.0, [toks[0]]), wlm.Task(wlm.KIND_IA3, 0, 1.0, [70]),
             wlm.Task(wlm.KIND_LORA, 32, 0.5, [toks[1], 21]), wlm.Task(wlm.KIND_NONE, 0, 1.0, [64]),
             wlm.Task(wlm.KIND_LORA, 8, 1.5, [toks[2]]), wlm.Task(wlm.KIND_LORA, 24, 1.0, [toks[3]]),
             wlm.Task(wlm.KIND_LORA, 16, 2.0, [])]
    return wlm.Workload(name=f"fuse{N}", layers=[("w", K, N)], tasks=tasks, chunk=64, sigma_w=0.05, sigma_ab=0.05)


FUSE_CASES = ((512, 384, (100, 300, 37, 150), True), (256, 2816, (700, 300, 200, 130), False),
              (1024, 200, (33, 64, 5, 129), True))


def check_fused_down(env, half_tiles_too):
    """Parity of the FUSE_CASES and, from the kernel list of a forward, whether a separate down-projection ran."""
    mx, torch = env
    for K, N, toks, quarters in FUSE_CASES:
        for seg_flags in (0, 1):
            g, got, ref, errs = run_case(env, fuse_workload(K, N, toks), seed=K + seg_flags, seg_flags=seg_flags)
            mx.mux_profile_enable(1)
            mx.mux_profile_collect()
            g.forward()
            torch.cuda.synchronize()
            names = [e["name"] for e in mx.mux_profile_collect()]
            mx.mux_profile_enable(0)
            assert "gemm_nn" in names, names
            assert ("down_x" not in names) == (quarters or half_tiles_too), (K, N, names)


def test_down_projection_in_the_tile_loop(env):
    """Forward launches made of quarter tiles only form Hs = s_t X A_t inside the backbone tile loop (no down_x
    launch): ranks 8, 16, 24 and 32 next to IA3 and plain tasks, ragged rows, a ragged last column tile; against the
    oracle, forward and backward (which reads the Hs the tiles of the first column saved), and the kernel list shows
    that no separate down-projection ran.  The launch of half tiles among the cases keeps the separate launch (the
    variants test below runs it with the switch that fuses there too)."""
    check_fused_down(env, False)


def test_dy_pass_row_groups_and_column_slabs(env):
    """The pass over dY on shapes that give it several 512-column slabs (the last one ragged, one wave of it past the
    end), row groups of 1024 and of 256 rows with ragged tails, ranks that fill one, two and four 16-wide pieces, and
    A_t read in place (every rank a multiple of 8) or from the transposed copy (one rank that is not)."""
    for ranks, K, N, toks in (((16, 8, 16), 256, 1352, (2500, 1100, 300)),     # three slabs, 1024-row groups
                              ((32, 24, 64), 192, 1096, (700, 300, 1300)),     # NJ = 2 and 4
                              ((16, 12, 8), 320, 520, (600, 270, 130))):       # rank 12: the transposed copy
        tasks = [wlm.Task(wlm.KIND_LORA, r, 2.0, [n, 17]) for r, n in zip(ranks, toks)]
        tasks.insert(1, wlm.Task(wlm.KIND_IA3, 0, 1.0, [150]))
        wl = wlm.Workload(name=f"s4_{N}", layers=[("w", K, N)], tasks=tasks, chunk=64, sigma_w=0.05, sigma_ab=0.05)
        run_case(env, wl, seed=N)
        run_case(env, wl, seed=N + 1, seg_flags=1)


@pytest.mark.parametrize("block", range(4))
def test_random_sweep(env, block):
    """Seeded random layer calls: every adapter kind at random ranks (1..64), random shapes (multiples of 64, 32, 8
    and odd sizes, so every GEMM kernel is met), chunk sizes, pack lengths, both table modes, empty tasks."""
    mx, _ = env
    rng = np.random.default_rng(9000 + block)
    kinds = [wlm.KIND_LORA, wlm.KIND_LORA, wlm.KIND_IA3, wlm.KIND_ADAPTER, wlm.KIND_NONE, wlm.KIND_DIFF]
    for case in range(6):
        gran = int(rng.choice([64, 64, 32, 8, 1]))
        K = gran * int(rng.integers(1, max(2, 520 // gran)))
        N = gran * int(rng.integers(1, max(2, 520 // gran)))
        chunk = int(rng.choice([16, 32, 64, 128]))
        tasks = []
        for _t in range(int(rng.integers(1, 7))):
            kind = int(rng.choice(kinds))
            rank = int(rng.integers(1, 65)) if kind in (wlm.KIND_LORA, wlm.KIND_ADAPTER) else 0
            nseq = int(rng.integers(0, 4))
            lens = [int(v) for v in rng.integers(1, 200, size=nseq)]
            tasks.append(wlm.Task(kind, rank, float(rng.choice([0.5, 1.0, 2.0])), lens,
                                  density=float(rng.choice([0.0, 0.01, 0.1])) if kind == wlm.KIND_DIFF else 0.0))
        if sum(t.tokens for t in tasks) == 0:
            tasks.append(wlm.Task(wlm.KIND_LORA, 8, 1.0, [17]))
        wl = wlm.Workload(name=f"rnd{block}_{case}", layers=[("w", K, N)], tasks=tasks, chunk=chunk,
                          max_pack_len=int(rng.choice([0, 0, 150])), sigma_w=0.05, sigma_ab=0.05)
        dtype = mx.MUX_DT_F32 if case % 3 == 2 else mx.MUX_DT_BF16
        print(f"case {block}.{case}: K={K} N={N} chunk={chunk} tasks={[(t.kind, t.rank, t.seq_lens) for t in tasks]}", flush=True)
        run_case(env, wl, dtype=dtype, seg_flags=int(rng.integers(0, 2)), seed=100 * block + case)


@pytest.mark.parametrize("which", ["mixed", "tuning", "diff"])
def test_graph_capture_and_replay(env, which):
    """The calls allocate nothing and never synchronise, so a forward + backward pair can be captured into a HIP
    graph; every replay (with eager work and synchronisations in between) must give the eager results bit for bit."""
    mx, torch = env
    wl = {"mixed": mixed_workload, "tuning": tuning_workload, "diff": diff_workload}[which]()
    g, got, ref, _ = run_case(env, wl)                 # eager, also warms up every kernel
    torch.cuda.synchronize()
    keep = {"Y": g.Y.clone(), "dX": g.dX.clone()}
    for k in ("dA", "dB", "dL"):
        keep[k] = [None if t is None else t.clone() for t in getattr(g, k)]
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        with torch.cuda.graph(graph, stream=stream):
            g.forward()
            g.backward()
    torch.cuda.synchronize()
    for rep in range(3):
        g.Y.fill_(float("nan")); g.dX.fill_(float("nan"))
        for k in ("dA", "dB", "dL"):
            for t in getattr(g, k):
                if t is not None:
                    t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(g.Y, keep["Y"]) and torch.equal(g.dX, keep["dX"]), f"replay {rep}"
        for k in ("dA", "dB", "dL"):
            for a, b in zip(keep[k], getattr(g, k)):
                assert a is None or torch.equal(a, b), f"replay {rep} {k}"
        g.forward(); g.backward()                      # eager work between the replays
        torch.cuda.synchronize()


@pytest.mark.parametrize("var", ["MUX_GEMM_BK32", "MUX_GEMM_NO_HALF_TILES", "MUX_GEMM_NO_QUARTER_TILES", "MUX_GEMM_REGSTAGED",
                                 "MUX_GEMM_FUSE_DOWN=0", "MUX_GEMM_FUSE_DOWN=2"])
def test_gemm_variants_in_a_fresh_process(env, var):
    """The switches that are read once per process (32-deep stages where 64-deep ones would be taken; full tiles
    only; half-width tiles where quarters would be taken for the last round; the register-staged kernel, which
    otherwise only sees the shapes the pipelined kernel does not take, on shapes both can run; the down-projection
    never inside the tile loop, or in launches of half tiles as well): a parity case in a child process with the
    switch set."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    code = ("import torch, paper_2603_02885_amd as mx; mx.load_library(); import mux_workloads as wlm;"
            "from tests.test_gpu_parity import run_case, mixed_workload, tuning_workload, check_fused_down;"
            "tasks = [wlm.Task(wlm.KIND_LORA, 16, 2.0, [700]), wlm.Task(wlm.KIND_IA3, 0, 1.0, [300]), wlm.Task(wlm.KIND_LORA, 40, 1.0, [900])];"
            "wl = wlm.Workload(name='v', layers=[('w', 512, 1280)], tasks=tasks, chunk=64, sigma_w=0.04, sigma_ab=0.05);"
            "run_case((mx, torch), wl, seed=5); run_case((mx, torch), mixed_workload(K=320, N=256), seed=6); run_case((mx, torch), tuning_workload(K=192, N=160), seed=22);")
    if var == "MUX_GEMM_FUSE_DOWN=2":
        code += "check_fused_down((mx, torch), True);"
    code += "print('variant ok')"
    envv = dict(os.environ)
    name, _, value = var.partition("=")
    envv[name] = value or "1"
    r = subprocess.run([sys.executable, "-c", code], cwd=root, env=envv, capture_output=True, text=True, timeout=110)
    assert r.returncode == 0 and "variant ok" in r.stdout, r.stdout[-2000:] + r.stderr[-2000:]
