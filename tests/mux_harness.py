"""Helpers for the parity tests: run one layer call through the C ABI on the GPU and the same
seeded inputs through the fp64 oracle, and compare with the max-normalised error."""
from __future__ import annotations

from typing import Dict, List, Optional

import numpy as np

import mux_workloads as wlm

# Tolerances on E = max|gpu - ref| / max|ref| per tensor (each task's gradients separately):
# bf16 storage, fp32 accumulation on the matrix cores -> 2e-2; fp32 storage and arithmetic -> 1e-4.
TOL_BF16 = 2e-2
TOL_F32 = 1e-4


def norm_err(got: np.ndarray, ref: np.ndarray) -> float:
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    if not np.isfinite(got).all():
        return float("inf")
    scale = float(np.max(np.abs(ref)))
    d = float(np.max(np.abs(got - ref)))
    return d if scale == 0.0 else d / scale


def task_descs(mx, wl: wlm.Workload):
    return [mx.TaskDesc(t.kind, t.rank, t.scale, t.seq_lens) for t in wl.tasks]


class GpuLayer:
    """One layer call's device state (torch used for memory only)."""

    def __init__(self, mx, torch, wl: wlm.Workload, lt: wlm.LayerTensors, dtype: int, seg_flags: int = 0,
                 layer_flags: int = 0, max_pack_len: Optional[int] = None):
        self.mx, self.torch, self.wl, self.lt = mx, torch, wl, lt
        dev = "cuda:0"
        tdt = torch.bfloat16 if dtype == mx.MUX_DT_BF16 else torch.float32
        self.tdt = tdt
        self.st = mx.mux_segtab_build(task_descs(mx, wl), wl.chunk,
                                      wl.max_pack_len if max_pack_len is None else max_pack_len, seg_flags)
        self.T = mx.mux_segtab_rows(self.st)
        assert self.T == lt.X.shape[0]
        up = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(dev).to(tdt).contiguous()
        self.X, self.W, self.dY = up(lt.X), up(lt.W), up(lt.dY)
        self.A = [up(a) for a in lt.A]
        self.B = [up(b) for b in lt.B]
        self.L = [up(l) for l in lt.L]
        M = len(wl.tasks)
        todev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
        self.masks = [None if (not lt.masks or lt.masks[t] is None) else mx.SparseMask(lt.masks[t][0], lt.masks[t][1], lt.K, lt.N, todev)
                      for t in range(M)]
        self.layer = mx.LayerDesc(lt.K, lt.N, dtype, self.W, M, self.A, self.B, self.L, flags=layer_flags,
                                  masks=self.masks if any(m is not None for m in self.masks) else None)
        nb = mx.mux_segtab_device_bytes(self.st)
        self.dtab = torch.zeros(nb, dtype=torch.uint8, device=dev)
        mx.mux_segtab_upload(self.st, self.dtab, nb)
        self.saved_bytes = mx.mux_lora_saved_bytes(self.layer, self.st)
        self.ws_bytes = mx.mux_lora_workspace_bytes(self.layer, self.st)
        # poison scratch so that stale or unwritten data shows up
        self.saved = torch.full((max(self.saved_bytes, 256),), 0xFF, dtype=torch.uint8, device=dev)
        self.ws = torch.full((max(self.ws_bytes, 256),), 0xFF, dtype=torch.uint8, device=dev)
        self.Y = torch.full((self.T, lt.N), float("nan"), dtype=tdt, device=dev)
        self.dX = torch.full((self.T, lt.K), float("nan"), dtype=tdt, device=dev)
        self.dA = [None if a is None else torch.full(a.shape, float("nan"), dtype=torch.float32, device=dev) for a in lt.A]
        self.dB = [None if b is None else torch.full(b.shape, float("nan"), dtype=torch.float32, device=dev) for b in lt.B]
        self.dL = [None if l is None else torch.full(l.shape, float("nan"), dtype=torch.float32, device=dev) for l in lt.L]

    def forward(self):
        self.mx.mux_lora_forward(self.layer, self.st, self.dtab, self.X, self.Y, self.saved, self.ws, self.ws_bytes,
                                 self.torch.cuda.current_stream())

    def backward(self, accumulate: int = 0, want_dx: bool = True):
        self.mx.mux_lora_backward(self.layer, self.st, self.dtab, self.X, self.dY, self.saved,
                                  self.dX if want_dx else None, self.dA, self.dB, self.dL, accumulate, self.ws,
                                  self.ws_bytes, self.torch.cuda.current_stream())

    def results(self, cols=None, kcols=None) -> Dict[str, object]:
        """Outputs as float64 numpy; with cols / kcols only those columns of Y / dX are brought back."""
        torch = self.torch
        torch.cuda.synchronize()
        f = lambda t: None if t is None else t.float().cpu().numpy().astype(np.float64)
        Y, dX = self.Y, self.dX
        if cols is not None:
            Y = Y[:, torch.as_tensor(np.asarray(cols, dtype=np.int64), device=Y.device)]
        if kcols is not None:
            dX = dX[:, torch.as_tensor(np.asarray(kcols, dtype=np.int64), device=dX.device)]
        return {"Y": f(Y), "dX": f(dX), "dA": [f(t) for t in self.dA], "dB": [f(t) for t in self.dB],
                "dL": [f(t) for t in self.dL], "sampled": (cols is not None, kcols is not None)}


def oracle_results(wl: wlm.Workload, lt: wlm.LayerTensors, row_task: np.ndarray, cols=None, kcols=None):
    import oracle
    kinds = [t.kind for t in wl.tasks]
    ranks = [t.rank for t in wl.tasks]
    scales = [t.scale for t in wl.tasks]
    S = lt.masks if lt.masks else None
    f = oracle.forward(lt.X, lt.W, row_task, kinds, ranks, scales, lt.A, lt.B, lt.L, cols=cols, S=S)
    b = oracle.backward(lt.X, lt.dY, lt.W, row_task, kinds, ranks, scales, lt.A, lt.B, lt.L, kcols=kcols, cols=cols, S=S)
    return {"Y": f["Y"], "dX": b["dX"], "dA": b["dA"], "dB": b["dB"], "dL": b["dL"]}


def compare(got: Dict[str, object], ref: Dict[str, object], tol: float, cols=None, kcols=None, label: str = "") -> Dict[str, float]:
    """Asserts every tensor within tol; returns the errors found."""
    errs: Dict[str, float] = {}
    y_sampled, x_sampled = got.get("sampled", (False, False))
    gy = got["Y"] if (cols is None or y_sampled) else got["Y"][:, cols]
    gx = got["dX"] if (kcols is None or x_sampled) else got["dX"][:, kcols]
    errs["Y"] = norm_err(gy, ref["Y"])
    errs["dX"] = norm_err(gx, ref["dX"])
    for name in ("dA", "dB", "dL"):
        for t, r in enumerate(ref[name]):
            if r is None:
                continue
            g = got[name][t]
            if name == "dL" and cols is not None:
                g = g[cols]
            errs[f"{name}[{t}]"] = norm_err(g, r)
    bad = {k: v for k, v in errs.items() if not (v <= tol)}
    assert not bad, f"{label}: normalised error above {tol}: {bad}"
    return errs
