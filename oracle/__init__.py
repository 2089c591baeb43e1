"""TEST INFRASTRUCTURE -- fp64 CPU oracle of the multiplexed PEFT linear layer.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
package.  It never imports the HIP library or its binding.

`forward` / `backward` marshal numpy arrays into the plain-C routines of
`mux_oracle.c` (built by `oracle/build.py` with gcc); `segtab` is the oracle's own
chunk-alignment table builder.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

import numpy as np

from . import segtab  # noqa: F401
from .build import build_oracle, LIB_PATH

_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        override = os.environ.get("MUX_ORACLE_LIB")      # used only by the test that plants mistakes in a copy
        if override:
            _lib = ctypes.CDLL(override)
            _lib.mux_oracle_forward.restype = ctypes.c_int
            _lib.mux_oracle_backward.restype = ctypes.c_int
            _lib.mux_oracle_max_threads.restype = ctypes.c_int
            return _lib
        if not os.path.exists(LIB_PATH) or os.path.getmtime(LIB_PATH) < os.path.getmtime(
                os.path.join(os.path.dirname(__file__), "mux_oracle.c")):
            build_oracle()
        _lib = ctypes.CDLL(LIB_PATH)
        _lib.mux_oracle_forward.restype = ctypes.c_int
        _lib.mux_oracle_backward.restype = ctypes.c_int
        _lib.mux_oracle_max_threads.restype = ctypes.c_int
    return _lib


def max_threads() -> int:
    return int(lib().mux_oracle_max_threads())


_F = ctypes.POINTER(ctypes.c_float)
_D = ctypes.POINTER(ctypes.c_double)
_I = ctypes.POINTER(ctypes.c_int32)


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _ptrs_f(arrs: Sequence[Optional[np.ndarray]]):
    keep = [None if a is None else _f32(a) for a in arrs]
    arr = (_F * max(len(keep), 1))()
    for i, a in enumerate(keep):
        arr[i] = a.ctypes.data_as(_F) if a is not None else None
    return arr, keep


def _ptrs_d(arrs: Sequence[Optional[np.ndarray]]):
    arr = (_D * max(len(arrs), 1))()
    for i, a in enumerate(arrs):
        arr[i] = a.ctypes.data_as(_D) if a is not None else None
    return arr


def _cols(cols, n_full):
    if cols is None:
        return n_full, None, None
    c = np.ascontiguousarray(cols, dtype=np.int32)
    return int(c.size), c.ctypes.data_as(_I), c


def _sparse_args(S, M):
    """S: per task None or (k[nnz], n[nnz]) int arrays sorted by (k, n).  Returns the three C arguments and keep-alives."""
    S = S if S is not None else [None] * M
    nnz = np.zeros(M, dtype=np.int32)
    IP = ctypes.POINTER(ctypes.c_int32)
    kp = (IP * M)(); npp = (IP * M)()
    keep = []
    for t in range(M):
        if S[t] is None:
            continue
        k = np.ascontiguousarray(S[t][0], dtype=np.int32); n = np.ascontiguousarray(S[t][1], dtype=np.int32)
        assert k.shape == n.shape and k.ndim == 1
        nnz[t] = k.size
        kp[t] = k.ctypes.data_as(IP); npp[t] = n.ctypes.data_as(IP)
        keep += [k, n]
    return nnz.ctypes.data_as(_I), kp, npp, (nnz, keep)


def _task_arrays(kinds, ranks, scales):
    k = np.ascontiguousarray(kinds, dtype=np.int32)
    r = np.ascontiguousarray(ranks, dtype=np.int32)
    s = np.ascontiguousarray(scales, dtype=np.float64)
    return k, r, s


def forward(X, W, row_task, kinds, ranks, scales, A, B, L, cols=None, want_z=False, S=None):
    """Returns dict(Y[T,n_cols], H[T,r_max], Z or None), all float64."""
    X = _f32(X); W = _f32(W)
    T, K = X.shape
    K2, N = W.shape
    assert K == K2
    row_task = np.ascontiguousarray(row_task, dtype=np.int32)
    assert row_task.shape == (T,)
    k, r, s = _task_arrays(kinds, ranks, scales)
    M = len(k)
    r_max = int(max([int(r[t]) for t in range(M) if k[t] in (1, 3)] + [1]))
    n_cols, cptr, _ckeep = _cols(cols, N)
    Ap, _ka = _ptrs_f(A); Bp, _kb = _ptrs_f(B); Lp, _kl = _ptrs_f(L)
    sp = _sparse_args(S, M)
    Y = np.zeros((T, n_cols), dtype=np.float64)
    H = np.zeros((T, r_max), dtype=np.float64)
    Z = np.zeros((T, n_cols), dtype=np.float64) if want_z else None
    rc = lib().mux_oracle_forward(
        T, K, N, X.ctypes.data_as(_F), W.ctypes.data_as(_F), row_task.ctypes.data_as(_I),
        M, k.ctypes.data_as(_I), r.ctypes.data_as(_I), s.ctypes.data_as(_D),
        Ap, Bp, Lp, n_cols, cptr, r_max,
        Y.ctypes.data_as(_D), H.ctypes.data_as(_D),
        Z.ctypes.data_as(_D) if Z is not None else None, *sp[:3])
    if rc != 0:
        raise RuntimeError(f"mux_oracle_forward failed: {rc}")
    return {"Y": Y, "H": H, "Z": Z}


def backward(X, dY, W, row_task, kinds, ranks, scales, A, B, L, kcols=None, cols=None,
             want_dx=True, S=None):
    """Returns dict(dX[T,n_kcols], G[T,r_max], dA[list], dB[list], dL[list]), float64."""
    X = _f32(X); W = _f32(W); dY = _f32(dY)
    T, K = X.shape
    K2, N = W.shape
    assert K == K2 and dY.shape == (T, N)
    row_task = np.ascontiguousarray(row_task, dtype=np.int32)
    k, r, s = _task_arrays(kinds, ranks, scales)
    M = len(k)
    r_max = int(max([int(r[t]) for t in range(M) if k[t] in (1, 3)] + [1]))
    n_kcols, kptr, _kk = _cols(kcols, K)
    n_cols, cptr, _ck = _cols(cols, N)
    Ap, _ka = _ptrs_f(A); Bp, _kb = _ptrs_f(B); Lp, _kl = _ptrs_f(L)
    sp = _sparse_args(S, M)
    dX = np.zeros((T, n_kcols), dtype=np.float64) if want_dx else None
    G = np.zeros((T, r_max), dtype=np.float64)
    dA: List[Optional[np.ndarray]] = []
    dB: List[Optional[np.ndarray]] = []
    dL: List[Optional[np.ndarray]] = []
    for t in range(M):
        if k[t] == 1:
            dA.append(np.zeros((K, int(r[t])), dtype=np.float64))
            dB.append(np.zeros((int(r[t]), N), dtype=np.float64))
            dL.append(None)
        elif k[t] == 4:     # selective kind: one gradient value per masked entry
            dA.append(np.zeros((int(np.asarray(S[t][0]).size),), dtype=np.float64))
            dB.append(None); dL.append(None)
        elif k[t] == 3:     # additive kind: D [N, r] in the A slot, U [r, N] in the B slot
            dA.append(np.zeros((N, int(r[t])), dtype=np.float64))
            dB.append(np.zeros((int(r[t]), N), dtype=np.float64))
            dL.append(None)
        elif k[t] == 2:
            dA.append(None); dB.append(None)
            dL.append(np.zeros((n_cols,), dtype=np.float64))
        else:
            dA.append(None); dB.append(None); dL.append(None)
    rc = lib().mux_oracle_backward(
        T, K, N, X.ctypes.data_as(_F), dY.ctypes.data_as(_F), W.ctypes.data_as(_F),
        row_task.ctypes.data_as(_I), M, k.ctypes.data_as(_I), r.ctypes.data_as(_I),
        s.ctypes.data_as(_D), Ap, Bp, Lp, n_kcols, kptr, n_cols, cptr, r_max,
        dX.ctypes.data_as(_D) if dX is not None else None, G.ctypes.data_as(_D),
        _ptrs_d(dA), _ptrs_d(dB), _ptrs_d(dL), *sp[:3])
    if rc != 0:
        raise RuntimeError(f"mux_oracle_backward failed: {rc}")
    return {"dX": dX, "G": G, "dA": dA, "dB": dB, "dL": dL}
