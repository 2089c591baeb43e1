#!/usr/bin/env python3
"""Benchmark of the multiplexed LoRA linear layer: fwd+bwd over every projection of one
synthetic multi-tenant workload, on ONE MI355X.

One "step" = forward + backward of all layer calls of the workload (7 projections of a
LLaMA-shaped block), inputs resident in HBM.  Default workload: configs[3] of the benchmark spec (LLaMA-13B shapes,
6 LoRA r16 + 2 IA3 tasks, about 20 k rows).  Prints one JSON line: value = valid tokens per second of the whole
step; roofline = the slower backbone GEMM kernel against the bf16 matrix-core peak, its duration from HIP events on
the launch stream; kernels = every kernel of the step; cpu_baseline = the fp64 oracle on a bounded sample.
`--gpus N` with N > 1 is refused: this build is single-GPU.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_MFMA = 2500.0    # TFLOP/s, MI355X dense bf16
PEAK_HBM = 8000.0          # GB/s


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", type=int, default=3,
                    help="index into BASELINE.json configs (default 3: the LLaMA-13B shapes with 6 LoRA + 2 IA3 tasks the "
                         "matrix-core target is stated on; 1: LLaMA-7B shapes); 5 / 6 = those shapes with two "
                         "Adapter-Tuning / Diff-Pruning tasks; 7 / 8 = the paper's Table 2 mixes A / B; 9 = mix A on GPT3-2.7B "
                         "shapes")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true",
                    help="leave out the extra measurement of the step replayed from a HIP graph")
    ap.add_argument("--no-mfma-probe", action="store_true",
                    help="leave out the two context probes of this box (register-only MFMA rate, plain HBM read stream)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="target CPU time of the oracle sample")
    ap.add_argument("--no-cpu-full", action="store_true",
                    help="leave out the oracle runs timed in full (tiny config, q projection of the LLaMA-7B config)")
    ap.add_argument("--compare-unmultiplexed", action="store_true",
                    help="also time the same tasks one at a time (one table and one set of calls per task, same shared "
                         "W, same rows), on one stream and alternating over two streams: what multiplexing buys")
    ap.add_argument("--two-streams", action="store_true",
                    help="also time the fully multiplexed step with its independent projections issued alternately on two "
                         "streams (kernels of the two streams overlap, so per-kernel times of a profiler run then differ "
                         "from the single-stream ones)")
    ap.add_argument("--tradeoff", action="store_true",
                    help="instead of the benchmark line: spatial against temporal multiplexing of m equal LoRA tasks "
                         "(micro-batch 8, sequence length 128 each) on the LLaMA-7B projections, m = 1..16, and "
                         "gradient accumulation over 4 micro-batches")
    ap.add_argument("--plan", action="store_true",
                    help="instead of the benchmark line: profile t_o(x), t_a(x), u_a(x) of the seven projections over "
                         "the token count, plan the fusion of 8 unequal LoRA tasks with the library's planner and compare "
                         "the cost model's predictions with measured steps")
    ap.add_argument("--attention", action="store_true",
                    help="instead of the benchmark line: the attention step between the q/k/v and o projections on the "
                         "sequences of the chosen workload (heads of --head-dim, as many as the q projection is wide)")
    ap.add_argument("--head-dim", type=int, default=128,
                    help="with --attention: head dimension (64, 80, 96 or 128); heads = projection width / head dimension")
    ap.add_argument("--dispatch", action="store_true",
                    help="instead of the benchmark line: Dispatch of the chosen workload's tokens (packed per task <-> "
                         "aligned batch) at the width of the first projection's input, in GB/s")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch a plain 512 MiB device copy (known traffic) for scaling rocprofv3 byte counters")
    return ap.parse_args()


class LayerState:
    pass


class Telemetry:
    """Clock and power of the GPU as the driver reports them (sysfs of the amdgpu card: hwmon freq1_input = shader
    clock in Hz, power1_average or power1_input in microwatts, power1_cap), polled by a thread every few milliseconds
    while a region runs.  Whatever cannot be read on the box is left out; the clock measured inside the kernels
    (mux_diag_set_clock_buffer) does not depend on it."""

    def __init__(self):
        import glob
        self.files = {}
        for dev in sorted(glob.glob("/sys/class/drm/card*/device")):
            try:
                if open(os.path.join(dev, "vendor")).read().strip() != "0x1002":
                    continue
            except OSError:
                continue
            for hw in sorted(glob.glob(os.path.join(dev, "hwmon", "hwmon*"))):
                for key, names in (("sclk_hz", ("freq1_input",)), ("power_uw", ("power1_average", "power1_input")),
                                   ("power_cap_uw", ("power1_cap",))):
                    for n in names:
                        f = os.path.join(hw, n)
                        if key not in self.files and os.access(f, os.R_OK):
                            self.files[key] = f
            for key, n in (("pp_dpm_sclk", "pp_dpm_sclk"), ("gpu_busy_percent", "gpu_busy_percent")):
                f = os.path.join(dev, n)
                if os.access(f, os.R_OK):
                    self.files[key] = f
            if self.files:
                break

    def _read(self, key):
        try:
            txt = open(self.files[key]).read()
        except (OSError, KeyError):
            return None
        if key == "pp_dpm_sclk":          # "1: 1878Mhz *" marks the current level
            for line in txt.splitlines():
                if line.rstrip().endswith("*"):
                    try:
                        return float(line.split(":")[1].strip().split("M")[0]) * 1e6
                    except (IndexError, ValueError):
                        return None
            return None
        try:
            return float(txt.strip())
        except ValueError:
            return None

    def sample_while(self, fn, period=0.004):
        """Runs fn() while a thread polls; returns (fn's result, summary of the samples)."""
        import threading
        stop = threading.Event()
        rows = {"sclk_hz": [], "power_uw": [], "pp_dpm_sclk": []}

        def poll():
            while not stop.is_set():
                for k in rows:
                    if k in self.files:
                        v = self._read(k)
                        if v is not None:
                            rows[k].append(v)
                stop.wait(period)
        th = threading.Thread(target=poll, daemon=True)
        th.start()
        try:
            res = fn()
        finally:
            stop.set()
            th.join()
        out = {"source": "sysfs", "samples": max(len(v) for v in rows.values()) if rows else 0}
        mean = lambda v: sum(v) / len(v)
        if rows["sclk_hz"]:
            out["sclk_mhz_mean"] = mean(rows["sclk_hz"]) / 1e6
            out["sclk_mhz_min"] = min(rows["sclk_hz"]) / 1e6
        elif rows["pp_dpm_sclk"]:
            out["sclk_mhz_mean"] = mean(rows["pp_dpm_sclk"]) / 1e6
            out["sclk_mhz_min"] = min(rows["pp_dpm_sclk"]) / 1e6
        if rows["power_uw"]:
            out["power_w_mean"] = mean(rows["power_uw"]) / 1e6
            out["power_w_max"] = max(rows["power_uw"]) / 1e6
        cap = self._read("power_cap_uw")
        if cap:
            out["power_cap_w"] = cap / 1e6
        if out["samples"] == 0:
            out["note"] = "no readable clock or power file under /sys/class/drm/card*/device on this box"
        return res, out


def clock_from_buffer(torch, buf):
    """MHz from the two counters the matrix-core kernels add to (shader cycles, 100 MHz ticks); None if unused."""
    torch.cuda.synchronize()
    c, r = int(buf[0].item()), int(buf[1].item())
    return (100.0 * c / r) if r > 0 else None


def hbm_read_probe(mx, torch):
    """Context for the HBM fractions of the adapter kernels: what one plain read stream draws on this machine.  Four
    buffers of 512 MiB read in turn, so that the 256 MB last-level cache cannot serve any of it."""
    dev = "cuda:0"
    nbytes = 512 << 20
    bufs = [torch.zeros(nbytes, dtype=torch.uint8, device=dev) for _ in range(4)]
    sink = torch.empty(mx.mux_probe_read_sink_bytes(), dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream()
    for b in bufs:
        mx.mux_probe_read(b, nbytes, sink, stream)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(3):
        for b in bufs:
            mx.mux_probe_read(b, nbytes, sink, stream)
    e1.record()
    torch.cuda.synchronize()
    gbps = 12 * nbytes / (e0.elapsed_time(e1) * 1e-3) / 1e9
    return {"unit": "GB/s", "read_stream": gbps, "frac_of_hbm_peak": gbps / PEAK_HBM, "bytes_per_launch": nbytes}


def mfma_probe(mx, torch, seed, tele=None, clkbuf=None):
    """Context for the roofline fraction: the rate the matrix cores sustain on this machine with bf16 operands that stay in
    registers (two waves per SIMD, independent MFMAs back to back), for operands that are all zero, N(0,1), and
    distributed like the benchmark's (activations N(0,1), weights N(0,0.02)).  The clock under dense MFMA load is set
    by power, hence by the data."""
    dev = "cuda:0"
    n = mx.mux_probe_mfma_operand_bytes() // 2
    sink = torch.empty(mx.mux_probe_mfma_sink_bytes(), dtype=torch.uint8, device=dev)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    rnd = torch.randn(n, device=dev, dtype=torch.float32, generator=gen)
    like = rnd.clone()
    like[n // 2:] *= 0.02                                # second half: the B operands, distributed like W
    kinds = {"zeros": torch.zeros(n, dtype=torch.bfloat16, device=dev),
             "normal": rnd.to(torch.bfloat16),            # both operands N(0,1)
             "like_benchmark": like.to(torch.bfloat16)}  # A ~ N(0,1) like X and dY, B ~ N(0,0.02) like W
    stream = torch.cuda.current_stream()
    out = {"unit": "TFLOP/s", "waves_per_simd": 2, "instruction": "v_mfma_f32_32x32x16_bf16"}
    iters = 4000                                         # about 10 ms a launch
    for name, ops in kinds.items():
        mx.mux_probe_mfma(ops, sink, iters, stream)      # warm-up, and the clock settles
        if clkbuf is not None:
            clkbuf.zero_()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

        def run():
            e0.record()
            flop = 0.0
            for _ in range(3):
                flop += mx.mux_probe_mfma(ops, sink, iters, stream)
            e1.record()
            torch.cuda.synchronize()
            return flop
        flop, smp = tele.sample_while(run) if tele is not None else (run(), None)
        out[name] = flop / (e0.elapsed_time(e1) * 1e-3) / 1e12
        if clkbuf is not None:
            mhz = clock_from_buffer(torch, clkbuf)
            if mhz:
                # the same box, the same instruction, every matrix pipe busy all the time: FLOP/s over the clock it
                # ran at gives the FLOP per cycle the part really delivers (nominal: 256 CUs x 4 SIMDs x 1024)
                out[name + "_clock_mhz"] = mhz
                out[name + "_flop_per_cycle"] = out[name] * 1e12 / (mhz * 1e6)
        if smp is not None and name == "like_benchmark":
            out["telemetry_like_benchmark"] = smp
    return out


def setup(mx, torch, wl, seed):
    """Allocates one LayerState per projection; values from torch's seeded device generator
    (same distributions as the parity workloads: X, dY ~ N(0,1); W, A, B ~ N(0, 0.02); l ~ N(1, 0.02))."""
    dev = "cuda:0"
    bf = torch.bfloat16
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    st = mx.mux_segtab_build([mx.TaskDesc(t.kind, t.rank, t.scale, t.seq_lens) for t in wl.tasks], wl.chunk,
                             wl.max_pack_len, 0)
    T = mx.mux_segtab_rows(st)
    nb = mx.mux_segtab_device_bytes(st)
    dtab = torch.zeros(nb, dtype=torch.uint8, device=dev)
    mx.mux_segtab_upload(st, dtab, nb)
    randn = lambda shape, sigma=1.0, mean=0.0: (torch.randn(shape, device=dev, dtype=torch.float32, generator=gen) * sigma + mean).to(bf)
    layers = []
    ws_bytes = 0
    for name, K, N in wl.layers:
        L = LayerState()
        L.name, L.K, L.N = name, K, N
        L.W = randn((K, N), 0.02)
        # LoRA: A [K, r], B [r, N]; Adapter-Tuning: D [N, r] in the A slot, U [r, N] in the B slot
        L.A = [randn((K if t.kind == 1 else N, t.rank), 0.02) if t.kind in (1, 3) else None for t in wl.tasks]
        L.B = [randn((t.rank, N), 0.02) if t.kind in (1, 3) else None for t in wl.tasks]
        L.L = [randn((N,), 0.02, 1.0) if t.kind == 2 else None for t in wl.tasks]
        # Diff-Pruning: a random mask of the stated density over W, values in the A slot
        L.masks = [None] * len(wl.tasks)
        for ti, t in enumerate(wl.tasks):
            if t.kind == 4:
                kn = torch.nonzero(torch.rand((K, N), device=dev, generator=gen) < t.density).cpu().numpy()
                L.masks[ti] = mx.SparseMask(kn[:, 0], kn[:, 1], K, N, lambda a: torch.from_numpy(a).to(dev))
                L.A[ti] = randn((L.masks[ti].nnz,), 0.02)
        L.X = randn((T, K))
        L.dY = randn((T, N))
        L.Y = torch.empty((T, N), device=dev, dtype=bf)
        L.dX = torch.empty((T, K), device=dev, dtype=bf)
        L.dA = [None if a is None else torch.zeros(a.shape, device=dev, dtype=torch.float32) for a in L.A]
        L.dB = [None if b is None else torch.zeros(b.shape, device=dev, dtype=torch.float32) for b in L.B]
        L.dL = [None if l is None else torch.zeros(l.shape, device=dev, dtype=torch.float32) for l in L.L]
        L.desc = mx.LayerDesc(K, N, mx.MUX_DT_BF16, L.W, len(wl.tasks), L.A, L.B, L.L,
                              masks=L.masks if any(m is not None for m in L.masks) else None)
        L.saved_bytes = mx.mux_lora_saved_bytes(L.desc, st)
        L.saved = torch.zeros(max(L.saved_bytes, 256), dtype=torch.uint8, device=dev)
        ws_bytes = max(ws_bytes, mx.mux_lora_workspace_bytes(L.desc, st))
        layers.append(L)
    ws = torch.zeros(max(ws_bytes, 256), dtype=torch.uint8, device=dev)
    return st, dtab, T, layers, ws, ws_bytes


def step(mx, st, dtab, layers, ws, ws_bytes, stream):
    for L in layers:
        mx.mux_lora_forward(L.desc, st, dtab, L.X, L.Y, L.saved, ws, ws_bytes, stream)
    for L in reversed(layers):
        mx.mux_lora_backward(L.desc, st, dtab, L.X, L.dY, L.saved, L.dX, L.dA, L.dB, L.dL, 0, ws, ws_bytes, stream)


def unmultiplexed(mx, torch, wl, st, layers, steps, warmup, n_groups=None):
    """The same tasks, rows and shared weights with less (or no) backbone multiplexing: the tasks are cut into
    `n_groups` groups of consecutive tasks (default: one task per group, the paper's spatial batching of section 3.2
    switched off); every group gets its own table and its own forward/backward calls per projection, i.e. the groups
    are multiplexed in time (section 3.3) and the tasks inside a group in space.  Rows of consecutive tasks are a
    contiguous block of the aligned batch, so a group's X, dY, Y, dX are views of the multiplexed buffers."""
    dev = "cuda:0"
    img = mx.mux_segtab_serialize(st)
    M = len(wl.tasks)
    G = M if n_groups is None else max(1, min(n_groups, M))
    bounds = [round(i * M / G) for i in range(G + 1)]
    per_task = []
    for gi in range(G):
        ts = list(range(bounds[gi], bounds[gi + 1]))
        if not ts:
            continue
        r0 = int(img[16 + 8 * ts[0] + 0])
        rc = sum(int(img[16 + 8 * t + 1]) for t in ts)
        if rc == 0:
            continue
        st1 = mx.mux_segtab_build([mx.TaskDesc(wl.tasks[t].kind, wl.tasks[t].rank, wl.tasks[t].scale, wl.tasks[t].seq_lens)
                                   for t in ts], wl.chunk, wl.max_pack_len, 0)
        assert mx.mux_segtab_rows(st1) == rc
        nb = mx.mux_segtab_device_bytes(st1)
        dtab1 = torch.zeros(nb, dtype=torch.uint8, device=dev)
        mx.mux_segtab_upload(st1, dtab1, nb)
        calls = []
        for L in layers:
            mk = [L.masks[t] for t in ts]
            desc = mx.LayerDesc(L.K, L.N, mx.MUX_DT_BF16, L.W, len(ts), [L.A[t] for t in ts], [L.B[t] for t in ts],
                                [L.L[t] for t in ts], masks=mk if any(m is not None for m in mk) else None)
            sb = mx.mux_lora_saved_bytes(desc, st1)
            calls.append((desc, L.X[r0:r0 + rc], L.dY[r0:r0 + rc], L.Y[r0:r0 + rc], L.dX[r0:r0 + rc],
                          torch.zeros(max(sb, 256), dtype=torch.uint8, device=dev), [L.dA[t] for t in ts],
                          [L.dB[t] for t in ts], [L.dL[t] for t in ts], mx.mux_lora_workspace_bytes(desc, st1)))
        per_task.append((st1, dtab1, calls))
    wsb = max(c[9] for _, _, calls in per_task for c in calls)
    wss = [torch.zeros(max(wsb, 256), dtype=torch.uint8, device=dev) for _ in range(2)]
    main = torch.cuda.current_stream()
    side = torch.cuda.Stream()        # default priority

    def one_step(streams):
        for i, (st1, dtab1, calls) in enumerate(per_task):
            sidx = i % len(streams)
            stream, ws = streams[sidx], wss[sidx]
            for (desc, X, dY, Y, dX, saved, dA, dB, dL, _) in calls:
                mx.mux_lora_forward(desc, st1, dtab1, X, Y, saved, ws, wsb, stream)
            for (desc, X, dY, Y, dX, saved, dA, dB, dL, _) in reversed(calls):
                mx.mux_lora_backward(desc, st1, dtab1, X, dY, saved, dX, dA, dB, dL, 0, ws, wsb, stream)

    res = {}
    for name, streams in (("one_stream", [main]), ("two_streams", [main, side])):
        side.wait_stream(main)
        for _ in range(warmup):
            one_step(streams)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            one_step(streams)
        torch.cuda.synchronize()
        res[name] = {"ms_per_step": (time.perf_counter() - t0) * 1e3 / steps}
    return res


def tradeoff(mx, torch, args):
    """Section 3.3, the spatial-temporal tradeoff on one GPU: m equal tasks (8 sequences of 128 tokens, LoRA rank 16)
    over the seven LLaMA-7B projections, (a) batched in space: one call per projection and pass; (b) interleaved in
    time: one call per task, projection and pass, on one stream and alternating over two; (c) batched in space with
    the batch cut into 4 micro-batches of 2 sequences per task whose adapter gradients accumulate."""
    import mux_workloads as wlm
    base = wlm.config(1)
    rows = []
    stream = torch.cuda.current_stream()

    def timed(fn):
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / args.steps

    for m in (1, 2, 4, 8, 16):
        mk = lambda seqs: wlm.Workload(name=f"tradeoff_{m}", layers=base.layers,
                                       tasks=[wlm.Task(wlm.KIND_LORA, 16, 2.0, [128] * seqs) for _ in range(m)], chunk=128)
        wl = mk(8)
        st, dtab, T, layers, ws, ws_bytes = setup(mx, torch, wl, args.seed)
        tokens = mx.mux_segtab_valid_tokens(st)
        ms_space = timed(lambda: step(mx, st, dtab, layers, ws, ws_bytes, stream))
        row = {"tasks": m, "tokens": tokens, "spatial_ms": ms_space, "spatial_tokens_per_s": tokens / (ms_space * 1e-3)}
        if m > 1:
            r = unmultiplexed(mx, torch, wl, st, layers, args.steps, args.warmup, None)
            row["temporal_one_stream_ms"] = r["one_stream"]["ms_per_step"]
            row["temporal_two_streams_ms"] = r["two_streams"]["ms_per_step"]
        # 4 micro-batches: the same table for each (2 sequences per task), gradients accumulate from the second on
        wl4 = mk(2)
        st4, dtab4, T4, layers4, ws4, ws_bytes4 = setup(mx, torch, wl4, args.seed)

        def step_mb():
            for c in range(4):
                for L in layers4:
                    mx.mux_lora_forward(L.desc, st4, dtab4, L.X, L.Y, L.saved, ws4, ws_bytes4, stream)
                for L in reversed(layers4):
                    mx.mux_lora_backward(L.desc, st4, dtab4, L.X, L.dY, L.saved, L.dX, L.dA, L.dB, L.dL, 1 if c else 0,
                                         ws4, ws_bytes4, stream)
        row["spatial_4_microbatches_ms"] = timed(step_mb)
        rows.append(row)
        print(f"tradeoff: {m} tasks done", file=sys.stderr, flush=True)
        del layers, layers4, ws, ws4
        torch.cuda.empty_cache()
    one = rows[0]["spatial_tokens_per_s"]
    for r in rows:
        r["spatial_gain_over_one_task"] = r["spatial_tokens_per_s"] / one
    return {"metric": "spatial against temporal multiplexing, fwd+bwd of 7 LLaMA-7B projections", "unit": "ms per step",
            "steps": args.steps, "warmup": args.warmup, "dtype": "bf16", "data": "synthetic", "rows": rows}


def plan(mx, torch, args):
    """Section 3.3 with S = 1, N_g = 1 on this GPU.  Offline profiling (section 5): for x tokens and each projection,
    the wall time of a forward + backward call pair with one task of x tokens, once without an adapter and once with a
    LoRA r16 adapter; t_o(x) = half the first (Eq. 3 counts one pass, Eq. 4 doubles it), t_a(x) = half the difference,
    u_a(x) = the adapter's token rate at x over its best token rate.  Then the planner cuts 8 unequal tasks into
    hybrid tasks, and three executions are timed against the model's prediction: the plan, everything in one hybrid
    task, and every task alone (hybrid tasks one after the other on one stream)."""
    import mux_workloads as wlm
    base = wlm.config(1)
    stream = torch.cuda.current_stream()
    xs = [128, 256, 512, 1024, 2048, 4096, 8192, 16384]
    reps = max(args.steps, 5)
    t_pair = {kind: [[0.0] * len(xs) for _ in base.layers] for kind in (wlm.KIND_NONE, wlm.KIND_LORA)}
    for xi, x in enumerate(xs):
        for kind in (wlm.KIND_NONE, wlm.KIND_LORA):
            wl = wlm.Workload(name="profile", layers=base.layers, tasks=[wlm.Task(kind, 16, 2.0, [x])], chunk=128)
            st, dtab, T, layers, ws, ws_bytes = setup(mx, torch, wl, args.seed)
            for li, L in enumerate(layers):
                def pair():
                    mx.mux_lora_forward(L.desc, st, dtab, L.X, L.Y, L.saved, ws, ws_bytes, stream)
                    mx.mux_lora_backward(L.desc, st, dtab, L.X, L.dY, L.saved, L.dX, L.dA, L.dB, L.dL, 0, ws, ws_bytes, stream)
                for _ in range(3):
                    pair()
                best = float("inf")
                for _ in range(4):              # the fastest of four batches: a profile, not a sample of the noise
                    torch.cuda.synchronize()
                    t0 = time.perf_counter()
                    for _ in range(reps):
                        pair()
                    torch.cuda.synchronize()
                    best = min(best, (time.perf_counter() - t0) * 1e3 / reps)
                t_pair[kind][li][xi] = best
            del layers, ws
            torch.cuda.empty_cache()
        print(f"plan: profiled {x} tokens", file=sys.stderr, flush=True)
    baseops, adapters = [], []
    for li in range(len(base.layers)):
        t_o = [v / 2.0 for v in t_pair[wlm.KIND_NONE][li]]
        t_a = [max((a - b) / 2.0, 1e-4) for a, b in zip(t_pair[wlm.KIND_LORA][li], t_pair[wlm.KIND_NONE][li])]
        rate = [x / t for x, t in zip(xs, t_a)]
        u_a = [min(1.0, r / max(rate)) for r in rate]
        baseops.append((xs, t_o))
        adapters.append(((xs, t_a), (xs, u_a)))
    stages = [{"n_gpus": 1, "baseops": baseops, "adapters": adapters}]
    model = mx.CostModel(stages, 1)
    tokens = [256, 8192, 512, 1024, 4096, 1024, 2048, 256]
    t0 = time.perf_counter()
    f_star, order, begins = mx.mux_plan_fusion(model, tokens)
    plan_seconds = time.perf_counter() - t0

    def groups_of(begins_):
        return [[order[i] for i in range(begins_[h], begins_[h + 1])] for h in range(len(begins_) - 1)]

    def measure(groups):
        runs = []
        for g in groups:
            wl = wlm.Workload(name="planned", layers=base.layers,
                              tasks=[wlm.Task(wlm.KIND_LORA, 16, 2.0, [tokens[t]]) for t in g], chunk=128)
            runs.append(setup(mx, torch, wl, args.seed))

        def one():
            for st, dtab, T, layers, ws, ws_bytes in runs:
                step(mx, st, dtab, layers, ws, ws_bytes, stream)
        for _ in range(args.warmup):
            one()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            one()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / args.steps
        del runs
        torch.cuda.empty_cache()
        return ms

    def predict(groups):
        return sum(mx.mux_plan_htask_latency(model, [tokens[t] for t in g]) for g in groups)

    M = len(tokens)
    candidates = {"planned": groups_of(begins), "one_hybrid_task": groups_of([0, M]),
                  "every_task_alone": groups_of(list(range(M + 1))),
                  "two_halves": groups_of([0, M // 2, M])}
    results = {}
    for name, groups in candidates.items():
        results[name] = {"hybrid_tasks": [[tokens[t] for t in g] for g in groups], "predicted_ms": predict(groups),
                         "measured_ms": measure(groups)}
        results[name]["predicted_over_measured"] = results[name]["predicted_ms"] / results[name]["measured_ms"]
        print(f"plan: measured {name}", file=sys.stderr, flush=True)
    # the same profiles as four equal pipeline stages with four micro-batches: what the planner would choose there
    # (prediction only: this build runs on one GPU)
    model4 = mx.CostModel([{"n_gpus": 1, "baseops": baseops, "adapters": adapters}] * 4, 4)
    f4, order4, begins4 = mx.mux_plan_fusion(model4, tokens)
    return {"metric": "task-fusion plan: cost model against measurement, fwd+bwd of 7 LLaMA-7B projections",
            "unit": "ms per step", "steps": args.steps, "warmup": args.warmup, "dtype": "bf16", "data": "synthetic",
            "profile": {"tokens": xs, "t_o_ms": {n: baseops[i][1] for i, (n, _, _) in enumerate(base.layers)},
                        "t_a_ms": {n: adapters[i][0][1] for i, (n, _, _) in enumerate(base.layers)},
                        "u_a": {n: adapters[i][1][1] for i, (n, _, _) in enumerate(base.layers)}},
            "tasks_tokens": tokens, "plan_seconds": plan_seconds, "F_star_ms": f_star, "executions": results,
            "four_stage_pipeline_prediction": {"C": 4, "F_star_ms": f4,
                                               "hybrid_tasks": [[tokens[order4[i]] for i in range(begins4[h], begins4[h + 1])]
                                                                for h in range(len(begins4) - 1)]}}


def attention(mx, torch, args):
    """Causal attention of every sequence of the workload's chunk-aligned batch (section 3.5), forward + backward, on
    the same table as the linear layers.  FLOPs counted on the visible (query, key) pairs only, n (n + 1) / 2 per
    sequence of n tokens and head: 2 products forward (4 d FLOP a pair), 5 backward (10 d FLOP a pair; the kernels
    recompute the scores and dO.V^T in both backward passes, which is not counted)."""
    import mux_workloads as wlm
    import numpy as np
    wl = wlm.config(args.workload, seed=args.seed)
    dev = "cuda:0"
    d = args.head_dim
    width = wl.layers[0][2]
    if d not in (64, 80, 96, 128) or width % d:
        raise SystemExit(f"--head-dim {d}: must be 64, 80, 96 or 128 and divide the projection width {width}")
    H = width // d
    st = mx.mux_segtab_build([mx.TaskDesc(t.kind, t.rank, t.scale, t.seq_lens) for t in wl.tasks], wl.chunk,
                             wl.max_pack_len, 0)
    T = mx.mux_segtab_rows(st)
    nb = mx.mux_segtab_device_bytes(st)
    dtab = torch.zeros(nb, dtype=torch.uint8, device=dev)
    mx.mux_segtab_upload(st, dtab, nb)
    gen = torch.Generator(device=dev)
    gen.manual_seed(args.seed)
    rnd = lambda: torch.randn((T, H * d), device=dev, dtype=torch.float32, generator=gen).to(torch.bfloat16)
    qkv = torch.cat([rnd(), rnd(), rnd()], dim=1).contiguous()         # the fused output of the q/k/v projections
    Q, K, V = qkv[:, :H * d], qkv[:, H * d:2 * H * d], qkv[:, 2 * H * d:]
    dqkv = torch.empty_like(qkv)
    dQ, dK, dV = dqkv[:, :H * d], dqkv[:, H * d:2 * H * d], dqkv[:, 2 * H * d:]
    O, dO = torch.empty((T, H * d), device=dev, dtype=torch.bfloat16), rnd()
    desc = mx.AttnDesc(H, d, 3 * H * d, 3 * H * d, 3 * H * d, H * d)
    saved = torch.zeros(max(mx.mux_attn_saved_bytes(desc, st), 256), dtype=torch.uint8, device=dev)
    wsb = mx.mux_attn_workspace_bytes(desc, st)
    ws = torch.zeros(max(wsb, 256), dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream()

    def one():
        mx.mux_attn_forward(desc, st, dtab, Q, K, V, O, saved, stream)
        mx.mux_attn_backward(desc, st, dtab, Q, K, V, O, dO, saved, dQ, dK, dV, ws, wsb, stream)
    for _ in range(args.warmup):
        one()
    torch.cuda.synchronize()
    mx.mux_profile_enable(1)
    mx.mux_profile_collect()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        one()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    prof = mx.mux_profile_collect()
    mx.mux_profile_enable(0)
    lens = [n for t in wl.tasks for n in t.seq_lens]
    pairs = float(sum(n * (n + 1) // 2 for n in lens)) * H
    flops = {"attn_fwd": 4.0 * d * pairs, "attn_bwd_kv": 6.0 * d * pairs, "attn_bwd_q": 4.0 * d * pairs}
    kernels = {}
    for e in prof:
        k = {"launches": e["launches"], "avg_us": e["total_ms"] * 1e3 / max(e["launches"], 1)}
        if e["name"] in flops:
            k["tflops"] = flops[e["name"]] / (k["avg_us"] * 1e-6) / 1e12
            k["frac_of_bf16_mfma_peak"] = k["tflops"] / PEAK_BF16_MFMA
        kernels[e["name"]] = k
    valid = mx.mux_segtab_valid_tokens(st)
    dom = max((n for n in kernels if n in flops), key=lambda n: kernels[n]["avg_us"])
    return {"metric": "chunk-aligned causal attention fwd+bwd tokens/s", "value": valid / (ms * 1e-3), "unit": "tokens/s",
            "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True,
            "dtype": "bf16", "data": "synthetic",
            "config": {"workload": f"configs[{args.workload}] {wl.name}: sequences of {wl.notes}; {H} heads of {d}",
                       "rows": T, "valid_tokens": valid, "sequences": len(lens), "longest": max(lens)},
            "tflops": 14.0 * d * pairs / (ms * 1e-3) / 1e12,
            "roofline": {"kernel": dom, "bound": "mfma", "achieved": kernels[dom]["tflops"], "peak": PEAK_BF16_MFMA,
                         "unit": "TFLOP/s", "frac": kernels[dom]["frac_of_bf16_mfma_peak"], "traffic": None},
            "kernels": kernels}


def dispatch(mx, torch, args):
    """Gather of every task's packed tokens onto the aligned batch and scatter back (section 3.2, Dispatch), bf16 rows
    of the first projection's input width.  Algorithmic bytes of one pass: every valid token read once and written once
    (plus the zero rows of the padding for the gather)."""
    import mux_workloads as wlm
    wl = wlm.config(args.workload, seed=args.seed)
    dev = "cuda:0"
    width = wl.layers[0][1]
    st = mx.mux_segtab_build([mx.TaskDesc(t.kind, t.rank, t.scale, t.seq_lens) for t in wl.tasks], wl.chunk,
                             wl.max_pack_len, 0)
    T = mx.mux_segtab_rows(st)
    valid = mx.mux_segtab_valid_tokens(st)
    nb = mx.mux_segtab_device_bytes(st)
    dtab = torch.zeros(nb, dtype=torch.uint8, device=dev)
    mx.mux_segtab_upload(st, dtab, nb)
    packed = [torch.randn((max(t.tokens, 1), width), device=dev, dtype=torch.float32).to(torch.bfloat16) for t in wl.tasks]
    ptrs = [p if t.tokens else None for p, t in zip(packed, wl.tasks)]
    back = [torch.empty_like(p) for p in packed]
    bptrs = [p if t.tokens else None for p, t in zip(back, wl.tasks)]
    aligned = torch.empty((T, width), device=dev, dtype=torch.bfloat16)
    stream = torch.cuda.current_stream()
    res = {}
    for name, fn in (("dispatch_gather", lambda: mx.mux_dispatch_gather(st, dtab, ptrs, width, aligned, width, width, 2, stream)),
                     ("dispatch_scatter", lambda: mx.mux_dispatch_scatter(st, dtab, aligned, width, bptrs, width, width, 2, stream))):
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        mx.mux_profile_enable(1)
        mx.mux_profile_collect()
        for _ in range(args.steps):
            fn()
        torch.cuda.synchronize()
        prof = mx.mux_profile_collect()
        mx.mux_profile_enable(0)
        us = sum(e["total_ms"] for e in prof) * 1e3 / args.steps
        nbytes = 2.0 * valid * width * 2 + (2.0 * (T - valid) * width if name == "dispatch_gather" else 0.0)
        res[name] = {"avg_us": us, "gbps": nbytes / (us * 1e-6) / 1e9, "frac_of_hbm_peak": nbytes / (us * 1e-6) / 1e9 / PEAK_HBM}
    ok = all(torch.equal(a[:t.tokens], b[:t.tokens]) for a, b, t in zip(packed, back, wl.tasks))
    return {"metric": "Dispatch packed <-> aligned", "unit": "GB/s", "steps": args.steps, "warmup": args.warmup,
            "dtype": "bf16", "data": "synthetic", "round_trip_bit_exact": bool(ok),
            "config": {"workload": f"configs[{args.workload}] {wl.name}", "rows": T, "valid_tokens": valid, "width": width},
            "kernels": res}


def cpu_baseline(wl, seconds, seed, full_runs=True):
    """The fp64 oracle, as it stands, timed on the host cores.  `value`: a bounded sample of the benchmarked workload --
    the first m tokens of every task, aligned by the workload's own rule (its chunk size and packing), through every
    projection forward + backward, m sized from a short calibration so that the run takes about `seconds`.  Beside it,
    timed in full: the tiny config and the q projection of the LLaMA-7B config (5120 tokens, 4096 x 4096)."""
    import numpy as np
    import mux_workloads as wlm
    import oracle
    from oracle import segtab

    def run(work, layer_ids, m=None):
        tasks = work.tasks if m is None else [
            wlm.Task(t.kind, t.rank, t.scale, [min(m, t.tokens)] if t.tokens > 0 else [], t.density) for t in work.tasks]
        sub = wlm.Workload(name=work.name + ("" if m is None else "_sample"), layers=work.layers, tasks=tasks,
                           chunk=work.chunk, max_pack_len=work.max_pack_len)
        ot = segtab.build([t.seq_lens for t in tasks], work.chunk, work.max_pack_len, 0)
        kinds, ranks, scales = [t.kind for t in tasks], [t.rank for t in tasks], [t.scale for t in tasks]
        total, flop = 0.0, 0.0
        for li in layer_ids:
            lt = wlm.layer_tensors(sub, li, ot.T, seed=seed)
            S = lt.masks if any(mk is not None for mk in lt.masks) else None
            t0 = time.perf_counter()
            oracle.forward(lt.X, lt.W, ot.row_task, kinds, ranks, scales, lt.A, lt.B, lt.L, S=S)
            oracle.backward(lt.X, lt.dY, lt.W, ot.row_task, kinds, ranks, scales, lt.A, lt.B, lt.L, S=S)
            total += time.perf_counter() - t0
            flop += 4.0 * ot.valid_total * lt.K * lt.N
        return ot.valid_total, total, flop

    all_layers = list(range(len(wl.layers)))
    run(wl, all_layers[:1], 1)              # warm up (library load, OpenMP pool)
    # two short runs give the fixed cost (outputs of the padded rows are still zeroed) and the cost per token
    n0, t0, _ = run(wl, all_layers, 2)
    n1, t1, _ = run(wl, all_layers, 12)
    per_tok = max((t1 - t0) / max(n1 - n0, 1), 1e-9)
    fixed = max(t0 - per_tok * n0, 0.0)
    m = int(max(2, min(4096, max(seconds - fixed, 0.2 * seconds) / per_tok / max(len(wl.tasks), 1))))
    n, t, flop = run(wl, all_layers, m)
    out = {"value": n / t, "unit": "tokens/s", "cores": oracle.max_threads(), "kind": "oracle",
           "gflops_backbone": flop / t / 1e9,
           "sample": f"first {m} tokens of each of the {len(wl.tasks)} tasks ({n} tokens), aligned with the workload's "
                     f"chunk size {wl.chunk}, through all {len(wl.layers)} projections fwd+bwd, fp64, {t:.1f} s"}
    if full_runs:
        full = {}
        for label, idx, lids in (("configs[0] tiny, in full", 0, None), ("configs[1] llama7b, q projection in full", 1, [0])):
            w = wlm.config(idx, seed=seed)
            nn, tt, ff = run(w, list(range(len(w.layers))) if lids is None else lids)
            full[label] = {"tokens": nn, "seconds": tt, "tokens_per_s": nn / tt, "gflops_backbone": ff / tt / 1e9}
        out["in_full"] = full
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print(f"bench.py: this build runs on exactly one GPU (got --gpus {args.gpus}); "
              "the layer has no multi-GPU path", file=sys.stderr)
        sys.exit(2)
    import torch
    import mux_workloads as wlm
    import paper_2603_02885_amd as mx

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    mx.load_library()
    if args.tradeoff:
        print(json.dumps(tradeoff(mx, torch, args)))
        return
    if args.plan:
        print(json.dumps(plan(mx, torch, args)))
        return
    if args.attention:
        print(json.dumps(attention(mx, torch, args)))
        return
    if args.dispatch:
        print(json.dumps(dispatch(mx, torch, args)))
        return
    wl = wlm.config(args.workload, seed=args.seed)
    st, dtab, T, layers, ws, ws_bytes = setup(mx, torch, wl, args.seed)
    stream = torch.cuda.current_stream()
    valid = mx.mux_segtab_valid_tokens(st)

    for _ in range(args.warmup):
        step(mx, st, dtab, layers, ws, ws_bytes, stream)
    torch.cuda.synchronize()

    # timed region: K steps; the backbone GEMM launches are bracketed by HIP events recorded by the library on
    # the launch stream (only those: an event pair costs microseconds, which matters for the 10-microsecond kernels).
    # Around it: the first workgroup of every GEMM launch adds its cycle and 100 MHz tick counts to a device buffer
    # (the clock the kernel really ran at), and a thread polls the driver's clock and power files.
    tele = Telemetry()
    clkbuf = torch.zeros(4, dtype=torch.int64, device="cuda:0")
    mx.mux_diag_set_clock_buffer(clkbuf)
    mx.mux_profile_enable(2)
    mx.mux_profile_collect()
    torch.cuda.synchronize()

    def timed_region():
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step(mx, st, dtab, layers, ws, ws_bytes, stream)
        torch.cuda.synchronize()
        return t0, time.perf_counter()
    (t0, t1), telemetry = tele.sample_while(timed_region)
    prof = mx.mux_profile_collect()
    gemm_clock_mhz = clock_from_buffer(torch, clkbuf)
    mx.mux_diag_set_clock_buffer(None)
    # after the timed region: a few more steps with every kernel bracketed, for the per-kernel table
    mx.mux_profile_enable(1)
    extra_steps = min(args.steps, 5)
    for _ in range(extra_steps):
        step(mx, st, dtab, layers, ws, ws_bytes, stream)
    torch.cuda.synchronize()
    prof_all = mx.mux_profile_collect()
    mx.mux_profile_enable(0)

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    tokens_per_s = valid / (ms_per_step * 1e-3)

    # algorithmic work of one step
    sumKN = sum(K * N for _, K, N in wl.layers)
    img = mx.mux_segtab_serialize(st)
    M = len(wl.tasks)
    task_rows = [int(img[16 + 8 * t + 1]) for t in range(M)]           # aligned rows per task
    sum_tr = sum(task_rows[t] * wl.tasks[t].rank for t in range(M) if wl.tasks[t].kind == 1)
    ia3_rows = sum(task_rows[t] for t in range(M) if wl.tasks[t].kind == 2)
    tune_rows = sum(task_rows[t] for t in range(M) if wl.tasks[t].kind == 3)
    sum_tune = sum(task_rows[t] * wl.tasks[t].rank for t in range(M) if wl.tasks[t].kind == 3)
    flops_backbone = 4.0 * T * sumKN
    flops_adapter = 6.0 * sum_tr * sum(K + N for _, K, N in wl.layers) + 12.0 * sum_tune * sum(N for _, K, N in wl.layers)
    gemm_flops = {  # per step, per kernel family (all layers): 2TKN + 2 sum T_t r_t N (fwd) / K (bwd)
        "gemm_nn": 2.0 * T * sumKN + 2.0 * sum_tr * sum(N for _, K, N in wl.layers),
        "gemm_nt": 2.0 * T * sumKN + 2.0 * sum_tr * sum(K for _, K, N in wl.layers),
    }
    kernels = {}
    for e in prof_all:      # every kernel, from the extra steps after the timed region
        kernels[e["name"]] = {"launches": e["launches"], "avg_us": e["total_ms"] * 1e3 / max(e["launches"], 1),
                              "total_ms_per_step": e["total_ms"] / extra_steps}
    for e in prof:          # the GEMM kernels, from the timed region itself
        kernels[e["name"]] = {"launches": e["launches"], "avg_us": e["total_ms"] * 1e3 / max(e["launches"], 1),
                              "total_ms_per_step": e["total_ms"] / args.steps, "timed_region": True}
    # HBM-bound adapter kernels: algorithmic bytes per step (bf16 = 2 B, fp32 gradients = 4 B), counted over the rows
    # each kernel really streams: the VALID rows of the tasks whose kind it serves (padding rows and the rows of other
    # kinds cost it no memory access), plus the small operands and what it writes.
    valid_rows = [int(img[16 + 8 * t + 2]) for t in range(M)]          # real tokens per task
    kinds = [t.kind for t in wl.tasks]
    v_lora = sum(valid_rows[t] for t in range(M) if kinds[t] == 1)
    v_rank = sum(valid_rows[t] for t in range(M) if kinds[t] in (1, 3))  # LoRA and Adapter-Tuning share down_g / the gradient pass
    v_ia3 = sum(valid_rows[t] for t in range(M) if kinds[t] == 2)
    v_tune = sum(valid_rows[t] for t in range(M) if kinds[t] == 3)
    ranked = [t.rank for t in wl.tasks if t.kind in (1, 3)]
    RP = ((max(ranked + [1]) + 15) // 16) * 16
    sum_r = sum(t.rank for t in wl.tasks if t.kind == 1)
    sum_r13 = sum(ranked)
    dims = [(K, N) for _, K, N in wl.layers]
    stream_bytes = {
        # Hs / Gs are written for every aligned row (zeros outside the kernel's tasks)
        "down_x": sum(2.0 * v_lora * K + 2.0 * K * sum_r + 2.0 * T * RP for K, N in dims),
        "down_g": sum(2.0 * v_rank * N + 2.0 * N * sum_r13 + 2.0 * T * RP for K, N in dims),
        # one pass over dY: Gs and dB_t together (reads Hs, writes Gs and the fp32 dB_t)
        "s4_dy_pass": sum(2.0 * v_rank * N + 2.0 * N * sum_r13 + 2.0 * v_rank * RP + 2.0 * T * RP + 4.0 * N * sum_r13 for K, N in dims),
        "grad_dbda": sum(2.0 * v_rank * (N + K) + 4.0 * v_rank * RP + 4.0 * (N + K) * sum_r13 for K, N in dims),
        "grad_da": sum(2.0 * v_rank * K + 2.0 * v_rank * RP + 4.0 * K * sum_r13 for K, N in dims),
        "grad_dl": sum(4.0 * v_ia3 * N + 4.0 * N * sum(1 for k in kinds if k == 2) for K, N in dims),
        # Adapter-Tuning steps: each streams the task's rows of z, dY or both once
        "tune_down": sum(2.0 * v_tune * N for K, N in dims),
        "tune_up": sum(4.0 * v_tune * N for K, N in dims),
        "tune_g": sum(2.0 * v_tune * N for K, N in dims),
        "tune_dz": sum(4.0 * v_tune * N for K, N in dims),
        "tune_grads": sum(4.0 * v_tune * N for K, N in dims),
    }
    # Diff-Pruning steps: the block-transposed copies move the task rows of X (or dY) once each way; the sparse update
    # reads the rows once, reads and writes the output rows and reads the lists of the mask (8 B an entry forward,
    # 4 B backward, 2 B a value); the masked gradient reads both row sets and the row listing, and writes 4 B an entry.
    diff_rows = sum(task_rows[t] for t in range(M) if wl.tasks[t].kind == 4)
    if diff_rows:
        nnz = [sum(m.nnz for m in L.masks if m is not None) for L in layers]
        stream_bytes.update({
            "diff_xt": sum(4.0 * diff_rows * K for K, N in dims),      # forward, when the sparse updates follow the product
            "diff_gxt": sum(4.0 * diff_rows * (K + N) for K, N in dims),   # backward: both copies in one launch
            "diff_fwd": sum(2.0 * diff_rows * K + 4.0 * diff_rows * N + 10.0 * z for (K, N), z in zip(dims, nnz)),
            "diff_bwd": sum(2.0 * diff_rows * N + 4.0 * diff_rows * K + 6.0 * z for (K, N), z in zip(dims, nnz)),
            "diff_grad": sum(2.0 * diff_rows * (K + N) + 8.0 * z for (K, N), z in zip(dims, nnz)),
        })
    for n, b in stream_bytes.items():
        if n in kernels and kernels[n]["total_ms_per_step"] > 0:
            kernels[n]["bound"] = "hbm"
            kernels[n]["algorithmic_bytes_per_launch"] = b / (kernels[n]["launches"] / extra_steps)
            kernels[n]["gbps"] = b / (kernels[n]["total_ms_per_step"] * 1e-3) / 1e9
            kernels[n]["frac_of_hbm_peak"] = kernels[n]["gbps"] / PEAK_HBM
    # kernels that exist only because of how the path is cut into launches (partial sums brought together, the task
    # table written): the method itself asks for none of their bytes, so they get the bytes they move, as the
    # library counts them at the launch, and the rate that gives
    for e in prof_all:
        k = kernels.get(e["name"])
        if k is not None and "gbps" not in k and e.get("bytes", 0.0) > 0 and k["total_ms_per_step"] > 0:
            k["bound"] = "hbm"
            k["algorithmic_bytes_per_launch"] = 0.0
            k["moved_bytes_per_launch"] = e["bytes"] / e["launches"]
            k["gbps_moved"] = e["bytes"] / extra_steps / (k["total_ms_per_step"] * 1e-3) / 1e9
            k["frac_of_hbm_peak"] = k["gbps_moved"] / PEAK_HBM
    gemm_names = [n for n in kernels if n in gemm_flops]
    dom = max(gemm_names, key=lambda n: kernels[n]["total_ms_per_step"]) if gemm_names else None
    roofline = None
    if dom:
        tf = gemm_flops[dom] / (kernels[dom]["total_ms_per_step"] * 1e-3) / 1e12
        roofline = {"kernel": dom, "bound": "mfma", "achieved": tf, "peak": PEAK_BF16_MFMA, "unit": "TFLOP/s",
                    "frac": tf / PEAK_BF16_MFMA, "traffic": None,
                    "launches_per_step": kernels[dom]["launches"] / args.steps, "avg_launch_us": kernels[dom]["avg_us"]}
        # The clock the GEMM kernels ran at in the timed region (cycles over 100 MHz ticks of their first workgroups)
        # and what the part could deliver at that clock with every matrix pipe busy all the time: 256 compute units x
        # 4 SIMDs x 1024 FLOP a cycle (the nominal peak is this at 2.4 GHz).
        if gemm_clock_mhz:
            roofline["clock_mhz_in_kernel"] = gemm_clock_mhz
            roofline["ceiling_at_clock"] = gemm_clock_mhz * 1e6 * 1024 * 1024 / 1e12
            roofline["achieved_over_ceiling_at_clock"] = tf / roofline["ceiling_at_clock"]
        roofline["telemetry"] = telemetry
    # HBM bytes per launch of that kernel from the committed rocprofv3 --pmc summary of this workload (two separate
    # counter runs, scaled by a plain copy of known size); null when no summary for this workload is there
    tpath = os.path.join(ROOT, "profiles", f"traffic_{wl.name}.txt")
    if roofline and os.path.exists(tpath):
        for line in open(tpath):
            f = line.split()
            if len(f) == 3 and f[0] == "traffic_bytes_per_launch" and f[1] == dom:
                roofline["traffic"] = float(f[2])
                roofline["algorithmic_bytes_per_launch"] = sum(2.0 * (T * K + K * N + T * N) for _, K, N in wl.layers) / len(wl.layers)
    for n in gemm_names:
        kernels[n]["tflops"] = gemm_flops[n] / (kernels[n]["total_ms_per_step"] * 1e-3) / 1e12
        kernels[n]["frac_of_bf16_mfma_peak"] = kernels[n]["tflops"] / PEAK_BF16_MFMA

    out = {
        "metric": "multiplexed LoRA-linear fwd+bwd tokens/s", "value": tokens_per_s, "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"configs[{args.workload}] {wl.name}: {wl.notes}; layers " +
                               ",".join(f"{n}:{K}x{N}" for n, K, N in wl.layers),
                   "rows": T, "valid_tokens": valid, "chunk": wl.chunk, "tasks": M},
        "tflops": (flops_backbone + flops_adapter) / (ms_per_step * 1e-3) / 1e12,
        "frac_of_bf16_mfma_peak": (flops_backbone + flops_adapter) / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_MFMA,
        "padded_rows_per_s": T / (ms_per_step * 1e-3),
        "valid_row_fraction": valid / max(T, 1),          # FLOP figures count every row of the aligned batch
        "roofline": roofline,
        "kernels": kernels,
    }
    mx.mux_profile_enable(0)
    mx.mux_profile_collect()
    if args.two_streams or args.compare_unmultiplexed:
        # fully multiplexed, but the (independent) projections issued alternately on two streams, each with its own
        # workspace: the second stream's kernels fill the compute units the first one's GEMM leaves idle in its last round
        side = torch.cuda.Stream()
        ws2 = torch.zeros_like(ws)
        main = torch.cuda.current_stream()

        def step2():
            for i, L in enumerate(layers):
                sx, wx = (main, ws) if i % 2 == 0 else (side, ws2)
                mx.mux_lora_forward(L.desc, st, dtab, L.X, L.Y, L.saved, wx, ws_bytes, sx)
            for i, L in reversed(list(enumerate(layers))):
                sx, wx = (main, ws) if i % 2 == 0 else (side, ws2)
                mx.mux_lora_backward(L.desc, st, dtab, L.X, L.dY, L.saved, L.dX, L.dA, L.dB, L.dL, 0, wx, ws_bytes, sx)

        side.wait_stream(main)
        for _ in range(args.warmup):
            step2()
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        for _ in range(args.steps):
            step2()
        torch.cuda.synchronize()
        ms2 = (time.perf_counter() - t2) * 1e3 / args.steps
        out["multiplexed_projections_on_two_streams"] = {"ms_per_step": ms2, "tokens_per_s": valid / (ms2 * 1e-3)}
    if args.compare_unmultiplexed:
        mx.mux_profile_enable(0)
        mx.mux_profile_collect()
        um = {}
        groups = sorted({g for g in (2, 4, M) if 1 < g <= M})
        for g in groups:          # g groups of tasks multiplexed in time, the tasks of a group in space
            r = unmultiplexed(mx, torch, wl, st, layers, args.steps, args.warmup, g)
            for v in r.values():
                v["tokens_per_s"] = valid / (v["ms_per_step"] * 1e-3)
                v["multiplexed_speedup"] = v["ms_per_step"] / ms_per_step
            um[f"groups_{g}" if g < M else "one_task_per_call"] = r
        out["unmultiplexed"] = um
    if args.calibrate_copy:
        src = torch.zeros(512 << 20, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        out["calibration_copy_bytes"] = int(src.numel())
    if not args.no_graph:
        # the same step captured once into a HIP graph and replayed: the launches then cost the host nothing and the
        # gaps between the 56 kernels shrink; `value` stays the eagerly launched figure
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step(mx, st, dtab, layers, ws, ws_bytes, torch.cuda.current_stream())
        for _ in range(max(2, args.warmup)):
            graph.replay()
        torch.cuda.synchronize()
        tg = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        msg = (time.perf_counter() - tg) * 1e3 / args.steps
        out["hip_graph_replay"] = {"ms_per_step": msg, "tokens_per_s": valid / (msg * 1e-3)}
    if not args.no_mfma_probe:
        out["hbm_read_probe"] = hbm_read_probe(mx, torch)
        mx.mux_diag_set_clock_buffer(clkbuf)
        out["mfma_probe"] = mfma_probe(mx, torch, args.seed, tele, clkbuf)
        mx.mux_diag_set_clock_buffer(None)
        if out["roofline"].get("achieved"):
            # the same kernel against what the matrix cores of this machine sustain on such operands from registers
            out["roofline"]["achieved_over_mfma_probe"] = out["roofline"]["achieved"] / out["mfma_probe"]["like_benchmark"]
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, args.cpu_seconds, args.seed, not args.no_cpu_full)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
