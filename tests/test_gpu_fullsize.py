"""Full-size GPU parity: the benchmark workloads at their real shapes, in the launch configuration
bench.py times, compared with the fp64 oracle on sampled output columns: all rows x one seeded column out of every
128-column piece of Y and of dX (the last, ragged piece included) plus the first and last column of the first and of
the last piece, so that every 256 x 256 tile, half tile and quarter tile of a launch holds compared elements;
Hs/Gs enter through them; every task's dA_t, dB_t, d delta_t in full, dl_t on the sampled columns.
Likewise the attention step on the benchmark sequences with all heads, three heads compared."""
import numpy as np
import pytest

import mux_workloads as wlm
from tests import mux_harness as hz

pytestmark = pytest.mark.gpu


def stratified_columns(rng, n, piece=128):
    """One column of every `piece`-wide piece of 0..n-1, and the edges of the first and of the last piece."""
    cols = set()
    for c0 in range(0, n, piece):
        cols.add(int(rng.integers(c0, min(c0 + piece, n))))
    last0 = ((n - 1) // piece) * piece
    cols.update({0, min(piece, n) - 1, last0, n - 1})
    return np.array(sorted(cols), dtype=np.int32)


CASES = [(1, 0), (1, 4), (1, 6), (2, 0), (2, 4), (2, 6), (3, 0), (3, 4), (3, 6), (4, 0), (4, 3), (4, 4), (4, 6),
         (5, 0),     # 5: the extra workload with two Adapter-Tuning tasks (their rows need x W in full: one projection)
         (6, 0), (6, 4), (6, 6),   # 6: the extra workload with two Diff-Pruning tasks (d delta_t in full); whole, half and quarter tiles
         (9, 0), (9, 4), (9, 5)]   # 9: Table 2's mix A (eight small tasks) on GPT3-2.7B shapes


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
    # the selective kind's oracle walks the whole mask for every sampled column: wider pieces there
    piece = 512 if any(t.kind == wlm.KIND_DIFF for t in wl.tasks) else 128
    cols = stratified_columns(rng, N, piece)
    kcols = stratified_columns(rng, K, piece)
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


@pytest.mark.parametrize("cfg,d", [(1, 128), (3, 128), (3, 80), (1, 64)])
def test_attention_benchmark_sequences(env, cfg, d):
    """The attention step on the sequences of a benchmark workload with all its heads, as `bench.py --attention` runs
    it (fused QKV buffer; heads of 128, and of 80 and 64 as `--head-dim` runs them), compared with the attention oracle
    on three sampled heads."""
    mx, torch = env
    from oracle import attention as oatt
    from oracle import segtab
    wl = wlm.config(cfg)
    H = wl.layers[0][2] // d
    ot = segtab.build([t.seq_lens for t in wl.tasks], wl.chunk)
    seqs = [(s[2], s[3]) for s in segtab.sequences(ot)]
    T = ot.T
    print(f"attention config {cfg}: T={T} H={H} d={d} longest={max(n for _, n in seqs)}", flush=True)
    dev = "cuda:0"
    st = mx.mux_segtab_build([mx.TaskDesc(t.kind, t.rank, t.scale, t.seq_lens) for t in wl.tasks], wl.chunk, 0, 0)
    nb = mx.mux_segtab_device_bytes(st)
    dtab = torch.zeros(nb, dtype=torch.uint8, device=dev)
    mx.mux_segtab_upload(st, dtab, nb)
    gen = torch.Generator(device=dev)
    gen.manual_seed(100 + cfg)
    W = 3 * H * d
    qkv = torch.randn((T, W), device=dev, generator=gen).to(torch.bfloat16)
    dO = torch.randn((T, H * d), device=dev, generator=gen).to(torch.bfloat16)
    pad = torch.from_numpy(ot.row_task < 0).to(dev)
    qkv[pad] = float("nan")
    dO[pad] = float("nan")
    dqkv = torch.full_like(qkv, float("nan"))
    O = torch.full((T, H * d), float("nan"), dtype=torch.bfloat16, device=dev)
    desc = mx.AttnDesc(H, d, W, W, W, H * d)
    saved = torch.zeros(max(mx.mux_attn_saved_bytes(desc, st), 256), dtype=torch.uint8, device=dev)
    wsb = mx.mux_attn_workspace_bytes(desc, st)
    ws = torch.zeros(max(wsb, 256), dtype=torch.uint8, device=dev)
    Q, K, V = qkv[:, :H * d], qkv[:, H * d:2 * H * d], qkv[:, 2 * H * d:]
    dQ, dK, dV = dqkv[:, :H * d], dqkv[:, H * d:2 * H * d], dqkv[:, 2 * H * d:]
    stream = torch.cuda.current_stream()
    mx.mux_attn_forward(desc, st, dtab, Q, K, V, O, saved, stream)
    mx.mux_attn_backward(desc, st, dtab, Q, K, V, O, dO, saved, dQ, dK, dV, ws, wsb, stream)
    torch.cuda.synchronize()
    f = lambda t: t.float().cpu().numpy().astype(np.float64)
    padn = ot.row_task < 0
    for h in (0, H // 2 - 1, H - 1):
        c = slice(h * d, (h + 1) * d)
        q, k, v, do = f(Q[:, c]), f(K[:, c]), f(V[:, c]), f(dO[:, c])
        ref = oatt.forward(q, k, v, seqs, 1)
        ref.update(oatt.backward(q, k, v, do, seqs, 1))
        got = {"O": f(O[:, c]), "dQ": f(dQ[:, c]), "dK": f(dK[:, c]), "dV": f(dV[:, c])}
        errs = {}
        for name in got:
            assert np.all(got[name][padn] == 0), name
            errs[name] = hz.norm_err(got[name], ref[name])
        print(f"head {h}:", {k_: float(f"{v_:.2e}") for k_, v_ in errs.items()}, flush=True)
        assert all(v_ <= hz.TOL_BF16 for v_ in errs.values()), errs
