"""GPU parity of the attention step (include/mux_attn.h) against the fp64 attention oracle, same seeded inputs,
through the C ABI: forward and backward, sequences of every length relation to the 128-token blocks and 64-token
tiles, packed and chunk-cut, padding rows poisoned."""
import numpy as np
import pytest

from oracle import attention as oatt
from oracle import segtab

pytestmark = pytest.mark.gpu

TOL = 2e-2     # bf16 storage, fp32 accumulation: max |gpu - ref| / max |ref| per tensor


@pytest.fixture(scope="module")
def env():
    import torch
    import paper_2603_02885_amd as mx
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    mx.load_library()
    return mx, torch


def bf16_round(a):
    """Round fp32 values to bfloat16 (nearest even) so that both sides start from the same numbers."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = ((u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000).astype(np.uint32)
    return r.view(np.float32)


def run(env, task_lens, chunk, H, seed, max_pack_len=0, flags=0, fused=False, sigma=1.0, check_repeat=False, Hkv=None,
        d=128):
    mx, torch = env
    ot = segtab.build(task_lens, chunk, max_pack_len, flags)
    seqs = [(s[2], s[3]) for s in segtab.sequences(ot)]
    T = ot.T
    rng = np.random.default_rng(seed)
    Hkv = H if Hkv is None else Hkv
    Q, dO = (bf16_round(rng.standard_normal((T, H * d)) * sigma) for _ in range(2))
    K, V = (bf16_round(rng.standard_normal((T, Hkv * d)) * sigma) for _ in range(2))
    pad = ot.row_task < 0
    for a in (Q, K, V, dO):
        a[pad] = np.nan if seed % 2 else 1e30            # padding rows must not leak anywhere
    print(f"attention case: T={T} H={H} d={d} chunk={chunk} seqs={len(seqs)} longest={max([n for _, n in seqs] + [0])}", flush=True)
    st = mx.mux_segtab_build([mx.TaskDesc(mx.MUX_ADAPTER_NONE, 0, 1.0, l) for l in task_lens], chunk, max_pack_len, flags)
    assert np.array_equal(mx.mux_segtab_serialize(st), ot.image)
    dev = "cuda:0"
    nb = mx.mux_segtab_device_bytes(st)
    dtab = torch.zeros(nb, dtype=torch.uint8, device=dev)
    mx.mux_segtab_upload(st, dtab, nb)
    up = lambda a: torch.from_numpy(a).to(dev).to(torch.bfloat16)
    if fused:        # the three slices of one [T, 3 H d] buffer
        qkv = torch.cat([up(Q), up(K), up(V)], dim=1).contiguous()
        tq, tk, tv = qkv[:, :H * d], qkv[:, H * d:(H + Hkv) * d], qkv[:, (H + Hkv) * d:]
        ldq = ldk = (H + 2 * Hkv) * d
    else:
        tq, tk, tv = up(Q), up(K), up(V)
        ldq, ldk = H * d, Hkv * d
    tdo = up(dO)
    desc = mx.AttnDesc(H, d, ldq, ldk, ldk, H * d, n_kv_heads=Hkv)
    nan = float("nan")
    O = torch.full((T, H * d), nan, dtype=torch.bfloat16, device=dev)
    dQ = torch.full((T, H * d), nan, dtype=torch.bfloat16, device=dev)
    dK, dV = (torch.full((T, Hkv * d), nan, dtype=torch.bfloat16, device=dev) for _ in range(2))
    saved = torch.full((max(mx.mux_attn_saved_bytes(desc, st), 256),), 0xFF, dtype=torch.uint8, device=dev)
    wsb = mx.mux_attn_workspace_bytes(desc, st)
    ws = torch.full((max(wsb, 256),), 0xFF, dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream()
    mx.mux_attn_forward(desc, st, dtab, tq, tk, tv, O, saved, stream)
    torch.cuda.synchronize()
    if fused:        # backward writes dQ, dK, dV with the leading dimensions of Q, K, V: give it a fused buffer too
        dqkv = torch.full((T, (H + 2 * Hkv) * d), nan, dtype=torch.bfloat16, device=dev)
        dQ, dK, dV = dqkv[:, :H * d], dqkv[:, H * d:(H + Hkv) * d], dqkv[:, (H + Hkv) * d:]
    mx.mux_attn_backward(desc, st, dtab, tq, tk, tv, O, tdo, saved, dQ, dK, dV, ws, wsb, stream)
    torch.cuda.synchronize()
    got = {k: v.float().cpu().numpy().astype(np.float64) for k, v in (("O", O), ("dQ", dQ), ("dK", dK), ("dV", dV))}
    ref = oatt.forward(Q, K, V, seqs, H, n_kv_heads=Hkv)
    # the backward consumes the O the forward stored (bf16); the oracle's dO.O term uses its own O: same to rounding
    ref.update(oatt.backward(Q, K, V, dO, seqs, H, n_kv_heads=Hkv))
    errs = {}
    for k in ("O", "dQ", "dK", "dV"):
        assert np.isfinite(got[k]).all(), k
        assert np.all(got[k][pad] == 0), f"{k}: padding rows must be zero"
        scale = np.max(np.abs(ref[k])) or 1.0
        errs[k] = float(np.max(np.abs(got[k] - ref[k])) / scale)
    print({k: float(f"{v:.2e}") for k, v in errs.items()}, flush=True)
    assert all(v <= TOL for v in errs.values()), errs
    lse = saved[: T * H * 4].view(torch.float32).view(H, T).cpu().numpy().astype(np.float64)
    valid = ~pad
    assert np.allclose(lse[:, valid], ref["lse"][:, valid], rtol=0, atol=2e-2)
    if check_repeat:
        keep = [t.clone() for t in (O, dQ, dK, dV)]
        for _ in range(3):
            mx.mux_attn_forward(desc, st, dtab, tq, tk, tv, O, saved, stream)
            mx.mux_attn_backward(desc, st, dtab, tq, tk, tv, O, tdo, saved, dQ, dK, dV, ws, wsb, stream)
            torch.cuda.synchronize()
            for a, b in zip(keep, (O, dQ, dK, dV)):
                assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    return errs


def test_short_and_ragged_sequences(env):
    """Lengths around every boundary: 1 token, below / at / above a 32-token wave, a 64-token tile, a 128-token block."""
    lens = [[1, 2, 31, 32, 33], [63, 64, 65], [127, 128, 129], [200, 5], []]
    run(env, lens, chunk=64, H=2, seed=0, check_repeat=True)
    run(env, lens, chunk=16, H=1, seed=1)
    run(env, lens, chunk=64, H=2, seed=2, flags=1)                   # dense table: sequences back to back


def test_long_sequences_span_chunks(env):
    """Packs longer than a chunk: later chunks reuse the keys and values of the earlier ones (several blocks a sequence)."""
    run(env, [[700], [300, 260], [513]], chunk=128, H=3, seed=3)
    run(env, [[1000, 24]], chunk=256, H=2, seed=4, max_pack_len=1024)


def test_long_sequence_many_blocks(env):
    """Sequences of 2048 tokens and more (16 and more blocks, 32 and more key tiles) beside short ones, ragged ends
    included."""
    run(env, [[2100], [300, 260], [1]], chunk=128, H=2, seed=8, check_repeat=True)
    run(env, [[2048, 255, 257]], chunk=256, H=1, seed=9)


def test_fused_qkv_buffer_and_large_scores(env):
    """Q, K, V as slices of one buffer (leading dimension 3 H d), and scores far from zero (softmax close to one-hot)."""
    run(env, [[150, 90], [257]], chunk=64, H=2, seed=5, fused=True)
    run(env, [[150, 90], [257]], chunk=64, H=2, seed=6, sigma=3.0)


def test_grouped_query_heads(env):
    """Fewer key/value heads than query heads: groups of 2 and of 4 (one key/value head for all), separate and fused
    buffers; dK and dV add up the query heads of a group."""
    run(env, [[300, 70], [129]], chunk=64, H=4, Hkv=2, seed=10, check_repeat=True)
    run(env, [[300, 70], [129]], chunk=64, H=4, Hkv=1, seed=11, fused=True)
    run(env, [[1000]], chunk=128, H=8, Hkv=8, seed=12)                    # eight heads: the XCD-wise work mapping


def test_llama_heads_one_block(env):
    """32 heads of 128 (the q/k/v width of the 4096-wide projections), ragged lengths."""
    run(env, [[384, 100], [77]], chunk=128, H=32, seed=7)


@pytest.mark.parametrize("d", [64, 80, 96])
def test_other_head_dimensions(env, d):
    """Head dimensions below 128: 64 and 96 (two and three 32-column tiles of an output row) and 80 (GPT3-2.7B: 2560 / 32
    heads; the third tile half used).  Ragged lengths around every boundary, long sequences, grouped heads, a fused
    buffer, eight heads (the XCD-wise work mapping)."""
    lens = [[1, 2, 31, 32, 33], [63, 64, 65], [127, 128, 129], [200, 5], []]
    run(env, lens, chunk=64, H=2, seed=20 + d, d=d, check_repeat=True)
    run(env, [[700], [300, 260], [513]], chunk=128, H=3, seed=21 + d, d=d)
    run(env, [[300, 70], [129]], chunk=64, H=4, Hkv=2, seed=22 + d, d=d, fused=True)
    run(env, [[1000, 24]], chunk=256, H=8, seed=23 + d, d=d, max_pack_len=1024)


def test_random_sweep(env):
    """Seeded random calls: head dimensions 64 / 80 / 96 / 128, 1 to 8 key/value heads with groups of 1, 2 or 4 query
    heads, chunk sizes 16 to 256, up to four tasks of up to three sequences of up to 700 tokens, padded and dense
    tables, packs, separate and fused buffers."""
    rng = np.random.default_rng(777)
    for case in range(16):
        d = int(rng.choice([64, 80, 96, 128]))
        Hkv = int(rng.choice([1, 2, 3, 4, 8]))
        H = Hkv * int(rng.choice([1, 1, 2, 4]))
        chunk = int(rng.choice([16, 32, 64, 128, 256]))
        lens = [[int(v) for v in rng.integers(1, int(rng.choice([40, 200, 700])), size=int(rng.integers(0, 4)))]
                for _ in range(int(rng.integers(1, 5)))]
        if sum(len(l) for l in lens) == 0:
            lens[0] = [33]
        run(env, lens, chunk=chunk, H=H, Hkv=Hkv, seed=1000 + case, d=d, flags=int(rng.integers(0, 2)),
            fused=bool(rng.integers(0, 2)), max_pack_len=int(rng.choice([0, 0, 300])))


def test_argument_checks(env):
    mx, torch = env
    st = mx.mux_segtab_build([mx.TaskDesc(mx.MUX_ADAPTER_NONE, 0, 1.0, [64])], 64, 0, 0)
    dev = "cuda:0"
    nb = mx.mux_segtab_device_bytes(st)
    dtab = torch.zeros(nb, dtype=torch.uint8, device=dev)
    mx.mux_segtab_upload(st, dtab, nb)
    x = torch.zeros((64, 256), dtype=torch.bfloat16, device=dev)
    with pytest.raises(mx.MuxError):
        mx.mux_attn_forward(mx.AttnDesc(2, 48, 96, 96, 96, 96), st, dtab, x, x, x, x, None)           # head_dim 48
    with pytest.raises(mx.MuxError):
        mx.mux_attn_forward(mx.AttnDesc(2, 128, 128, 256, 256, 256), st, dtab, x, x, x, x, None)      # ldq too small
    x3 = torch.zeros((64, 384), dtype=torch.bfloat16, device=dev)
    with pytest.raises(mx.MuxError):
        mx.mux_attn_forward(mx.AttnDesc(3, 128, 384, 384, 384, 384, n_kv_heads=2), st, dtab, x3, x3, x3, x3, None)   # 2 does not divide 3
    with pytest.raises(mx.MuxError):
        mx.mux_attn_forward(mx.AttnDesc(2, 128, 256, 256, 256, 256), st, dtab, x, None, x, x, None)   # null K


def test_graph_capture_of_dispatch_and_attention(env):
    """Dispatch and the attention step allocate nothing and never synchronise: gather -> attention forward -> backward ->
    scatter captured into one HIP graph replays bit for bit, with eager work and synchronisations between the replays."""
    mx, torch = env
    d, H = 128, 2
    lens = [[150, 90], [257], [33]]
    st = mx.mux_segtab_build([mx.TaskDesc(mx.MUX_ADAPTER_NONE, 0, 1.0, l) for l in lens], 64, 0, 0)
    T = mx.mux_segtab_rows(st)
    dev = "cuda:0"
    nb = mx.mux_segtab_device_bytes(st)
    dtab = torch.zeros(nb, dtype=torch.uint8, device=dev)
    mx.mux_segtab_upload(st, dtab, nb)
    gen = torch.Generator(device=dev)
    gen.manual_seed(5)
    W = 3 * H * d
    packed = [torch.randn((sum(l), W), device=dev, generator=gen).to(torch.bfloat16) for l in lens]     # packed q|k|v rows
    qkv = torch.empty((T, W), dtype=torch.bfloat16, device=dev)
    dqkv = torch.empty_like(qkv)
    O = torch.empty((T, H * d), dtype=torch.bfloat16, device=dev)
    dO = torch.randn((T, H * d), device=dev, generator=gen).to(torch.bfloat16)
    outs = [torch.empty((sum(l), W), dtype=torch.bfloat16, device=dev) for l in lens]
    desc = mx.AttnDesc(H, d, W, W, W, H * d)
    saved = torch.zeros(max(mx.mux_attn_saved_bytes(desc, st), 256), dtype=torch.uint8, device=dev)
    wsb = mx.mux_attn_workspace_bytes(desc, st)
    ws = torch.zeros(max(wsb, 256), dtype=torch.uint8, device=dev)
    Q, K, V = qkv[:, :H * d], qkv[:, H * d:2 * H * d], qkv[:, 2 * H * d:]
    dQ, dK, dV = dqkv[:, :H * d], dqkv[:, H * d:2 * H * d], dqkv[:, 2 * H * d:]

    def chain(stream):
        mx.mux_dispatch_gather(st, dtab, packed, W, qkv, W, W, 2, stream)
        mx.mux_attn_forward(desc, st, dtab, Q, K, V, O, saved, stream)
        mx.mux_attn_backward(desc, st, dtab, Q, K, V, O, dO, saved, dQ, dK, dV, ws, wsb, stream)
        mx.mux_dispatch_scatter(st, dtab, dqkv, W, outs, W, W, 2, stream)

    chain(torch.cuda.current_stream())
    torch.cuda.synchronize()
    keep = [t.clone() for t in outs] + [O.clone()]
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        with torch.cuda.graph(graph, stream=stream):
            chain(stream)
    torch.cuda.synchronize()
    for rep in range(3):
        for t in outs + [O, qkv, dqkv]:
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(keep, outs + [O]):
            assert torch.equal(a.view(torch.int16), b.view(torch.int16)), f"replay {rep}"
        chain(torch.cuda.current_stream())               # eager work between the replays
        torch.cuda.synchronize()
