"""The pieces together: an attention sub-block of a transformer layer on the chunk-aligned batch of several tasks,
through the C ABI -- Dispatch (packed -> aligned), the multiplexed q / k / v projections with per-task adapters, causal
attention per sequence, the multiplexed o projection, and the whole chain backwards -- against the same chain built
from the oracles.  Activations that the GPU path stores in bf16 between the stages are rounded to bf16 at the same
places in the oracle chain, so that both sides feed every stage the same numbers up to that stage's own error."""
import numpy as np
import pytest

import mux_workloads as wlm
from oracle import attention as oatt
from oracle import dispatch as odisp
from oracle import segtab
from tests import mux_harness as hz
from tests.test_gpu_attention import bf16_round

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    import paper_2603_02885_amd as mx
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    mx.load_library()
    return mx, torch


def test_attention_block_forward_backward(env):
    import oracle
    mx, torch = env
    H, d = 2, 128
    C = H * d                                             # hidden size 256
    tasks = [wlm.Task(wlm.KIND_LORA, 16, 2.0, [100, 37]), wlm.Task(wlm.KIND_IA3, 0, 1.0, [70]),
             wlm.Task(wlm.KIND_NONE, 0, 1.0, [129]), wlm.Task(wlm.KIND_LORA, 8, 1.0, [5, 200]),
             wlm.Task(wlm.KIND_ADAPTER, 8, 0.5, [64])]
    wl = wlm.Workload(name="block", layers=[(n, C, C) for n in ("q", "k", "v", "o")], tasks=tasks, chunk=64,
                      sigma_w=0.06, sigma_ab=0.06)
    ot = segtab.build([t.seq_lens for t in tasks], wl.chunk)
    seqs = [(s[2], s[3]) for s in segtab.sequences(ot)]
    T, M = ot.T, len(tasks)
    kinds, ranks, scales = [t.kind for t in tasks], [t.rank for t in tasks], [t.scale for t in tasks]
    lts = [wlm.layer_tensors(wl, li, T, seed=40 + li, bf16=True, pad_rows=ot.row_task < 0, pad_fill=1e30) for li in range(4)]
    rng = np.random.default_rng(3)
    packed = [bf16_round(rng.standard_normal((t.tokens, C))) for t in tasks]           # every task's input tokens
    dYo = bf16_round(rng.standard_normal((T, C)))
    dYo[ot.row_task < 0] = np.nan                                                       # padding rows carry rubbish

    # ---- oracle chain
    r = lambda a: bf16_round(a).astype(np.float64)
    X = odisp.gather(packed, ot.row_task, C)
    lay = lambda li, x: oracle.forward(x, lts[li].W, ot.row_task, kinds, ranks, scales, lts[li].A, lts[li].B, lts[li].L)["Y"]
    Qo, Ko, Vo = (r(lay(li, X)) for li in range(3))
    Oo = r(oatt.forward(Qo, Ko, Vo, seqs, H)["O"])
    Yo = lay(3, Oo)
    bo = oracle.backward(Oo, dYo, lts[3].W, ot.row_task, kinds, ranks, scales, lts[3].A, lts[3].B, lts[3].L)
    dOo = r(bo["dX"])
    ba = oatt.backward(Qo, Ko, Vo, dOo, seqs, H)
    bq = [oracle.backward(X, r(ba[k]), lts[li].W, ot.row_task, kinds, ranks, scales, lts[li].A, lts[li].B, lts[li].L)
          for li, k in enumerate(("dQ", "dK", "dV"))]
    dXo = sum(r(b["dX"]) for b in bq)
    dx_packed = odisp.scatter(dXo, ot.row_task, M)

    # ---- the same chain through the library
    dev = "cuda:0"
    bf = torch.bfloat16
    st = mx.mux_segtab_build(hz.task_descs(mx, wl), wl.chunk, 0, 0)
    assert np.array_equal(mx.mux_segtab_serialize(st), ot.image)
    nb = mx.mux_segtab_device_bytes(st)
    dtab = torch.zeros(nb, dtype=torch.uint8, device=dev)
    mx.mux_segtab_upload(st, dtab, nb)
    up = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(dev).to(bf).contiguous()
    stream = torch.cuda.current_stream()
    tp = [up(p) for p in packed]
    Xg = torch.full((T, C), float("nan"), dtype=bf, device=dev)
    mx.mux_dispatch_gather(st, dtab, tp, C, Xg, C, C, 2, stream)
    layers = []
    for li in range(4):
        lt = lts[li]
        A, B, L = [up(a) for a in lt.A], [up(b) for b in lt.B], [up(l) for l in lt.L]
        W = up(lt.W)
        desc = mx.LayerDesc(C, C, mx.MUX_DT_BF16, W, M, A, B, L)
        saved = torch.zeros(max(mx.mux_lora_saved_bytes(desc, st), 256), dtype=torch.uint8, device=dev)
        wsb = mx.mux_lora_workspace_bytes(desc, st)
        ws = torch.zeros(max(wsb, 256), dtype=torch.uint8, device=dev)
        f32 = lambda ts: [None if t is None else torch.full(t.shape, float("nan"), dtype=torch.float32, device=dev) for t in ts]
        layers.append(dict(desc=desc, keep=(W, A, B, L), saved=saved, ws=ws, wsb=wsb, dA=f32(A), dB=f32(B), dL=f32(L)))
    nanbuf = lambda: torch.full((T, C), float("nan"), dtype=bf, device=dev)
    Qg, Kg, Vg, Og, Yg = nanbuf(), nanbuf(), nanbuf(), nanbuf(), nanbuf()
    for li, out in enumerate((Qg, Kg, Vg)):
        Ld = layers[li]
        mx.mux_lora_forward(Ld["desc"], st, dtab, Xg, out, Ld["saved"], Ld["ws"], Ld["wsb"], stream)
    adesc = mx.AttnDesc(H, d, C, C, C, C)
    asaved = torch.zeros(max(mx.mux_attn_saved_bytes(adesc, st), 256), dtype=torch.uint8, device=dev)
    awsb = mx.mux_attn_workspace_bytes(adesc, st)
    aws = torch.zeros(max(awsb, 256), dtype=torch.uint8, device=dev)
    mx.mux_attn_forward(adesc, st, dtab, Qg, Kg, Vg, Og, asaved, stream)
    Lo = layers[3]
    mx.mux_lora_forward(Lo["desc"], st, dtab, Og, Yg, Lo["saved"], Lo["ws"], Lo["wsb"], stream)
    dYg = up(dYo)
    dOg, dQg, dKg, dVg = nanbuf(), nanbuf(), nanbuf(), nanbuf()
    mx.mux_lora_backward(Lo["desc"], st, dtab, Og, dYg, Lo["saved"], dOg, Lo["dA"], Lo["dB"], Lo["dL"], 0, Lo["ws"], Lo["wsb"], stream)
    mx.mux_attn_backward(adesc, st, dtab, Qg, Kg, Vg, Og, dOg, asaved, dQg, dKg, dVg, aws, awsb, stream)
    dXs = []
    for li, g in enumerate((dQg, dKg, dVg)):
        Ld = layers[li]
        dx = nanbuf()
        mx.mux_lora_backward(Ld["desc"], st, dtab, Xg, g, Ld["saved"], dx, Ld["dA"], Ld["dB"], Ld["dL"], 0, Ld["ws"], Ld["wsb"], stream)
        dXs.append(dx)
    dXg = (dXs[0].float() + dXs[1].float() + dXs[2].float()).to(bf)          # the residual stream's sum (caller's job)
    outs = [torch.full((max(t.tokens, 1), C), float("nan"), dtype=bf, device=dev) for t in tasks]
    mx.mux_dispatch_scatter(st, dtab, dXg, C, outs, C, C, 2, stream)
    torch.cuda.synchronize()

    # ---- compare
    f = lambda t: t.float().cpu().numpy().astype(np.float64)
    errs = {"Q": hz.norm_err(f(Qg), Qo), "O": hz.norm_err(f(Og), Oo), "Y": hz.norm_err(f(Yg), Yo), "dO": hz.norm_err(f(dOg), dOo),
            "dQ": hz.norm_err(f(dQg), ba["dQ"]), "dK": hz.norm_err(f(dKg), ba["dK"]), "dV": hz.norm_err(f(dVg), ba["dV"])}
    for t in range(M):
        errs[f"dX[{t}]"] = hz.norm_err(f(outs[t])[:tasks[t].tokens], dx_packed[t])
    for li, b in enumerate(bq + [bo]):
        for name in ("dA", "dB", "dL"):
            for t, ref in enumerate(b[name]):
                if ref is not None:
                    errs[f"{name}[{li}][{t}]"] = hz.norm_err(f(layers[li][name][t]), ref)
    print({k: float(f"{v:.2e}") for k, v in errs.items()}, flush=True)
    bad = {k: v for k, v in errs.items() if not (v <= hz.TOL_BF16)}
    assert not bad, bad
