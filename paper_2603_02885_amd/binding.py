"""ctypes binding of libmuxlora.so: same names as include/mux.h, argument marshalling only.

Every step of the layer runs in the library's HIP kernels; there is no Python or CPU
fallback.  PyTorch tensors (or raw integers) are accepted wherever a device pointer is
expected; torch is used by callers for device memory and streams only.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, c_char_p, c_float, c_int, c_int32, c_int64, c_size_t, c_uint32, c_void_p
from typing import List, Optional, Sequence

import numpy as np

__all__ = [
    "MUX_OK", "MUX_ADAPTER_NONE", "MUX_ADAPTER_LORA", "MUX_ADAPTER_IA3_OUT", "MUX_ADAPTER_TUNING", "MUX_ADAPTER_DIFF", "SparseMask", "MUX_DT_BF16", "MUX_DT_F32",
    "MUX_SEGTAB_DENSE", "MUX_LAYER_REFERENCE_KERNELS", "MUX_MAX_RANK", "MuxError", "TaskDesc", "LayerDesc", "SegTab",
    "library_path", "load_library", "mux_choose_chunk_size", "mux_segtab_build", "mux_segtab_free",
    "mux_segtab_rows", "mux_segtab_n_chunks", "mux_segtab_n_tasks", "mux_segtab_valid_tokens",
    "mux_segtab_serialized_bytes", "mux_segtab_serialize", "mux_segtab_row_task", "mux_segtab_device_bytes",
    "mux_segtab_upload", "mux_sparse_mask_layout", "mux_sparse_mask_tile_layout", "mux_lora_saved_bytes", "mux_lora_workspace_bytes", "mux_lora_forward",
    "mux_lora_backward", "mux_lora_backward_static_ws", "MUX_STATIC_WS_BYTES", "mux_last_error", "mux_version", "mux_profile_enable", "mux_profile_collect",
    "CostModel", "mux_plan_stage_latency", "mux_plan_htask_latency", "mux_plan_fusion",
    "mux_dispatch_gather", "mux_dispatch_scatter",
    "AttnDesc", "mux_attn_saved_bytes", "mux_attn_workspace_bytes", "mux_attn_forward", "mux_attn_backward",
    "mux_probe_mfma_operand_bytes", "mux_probe_mfma_sink_bytes", "mux_probe_mfma",
    "mux_probe_read_sink_bytes", "mux_probe_read", "mux_diag_set_clock_buffer",
]

MUX_OK = 0
MUX_ADAPTER_NONE, MUX_ADAPTER_LORA, MUX_ADAPTER_IA3_OUT, MUX_ADAPTER_TUNING, MUX_ADAPTER_DIFF = 0, 1, 2, 3, 4
MUX_DT_BF16, MUX_DT_F32 = 0, 1
MUX_SEGTAB_DENSE = 1
MUX_LAYER_REFERENCE_KERNELS = 1
MUX_MAX_RANK = 64
MUX_STATIC_WS_BYTES = 32 << 20

_STATUS_NAMES = {1: "MUX_ERR_INVALID_ARG", 2: "MUX_ERR_SHAPE", 3: "MUX_ERR_UNSUPPORTED", 4: "MUX_ERR_WORKSPACE",
                 5: "MUX_ERR_HOST_NOMEM", 6: "MUX_ERR_DEVICE"}


class MuxError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"{_STATUS_NAMES.get(status, status)}: {text}")
        self.status = status


class _TaskDescC(ctypes.Structure):
    _fields_ = [("kind", c_int32), ("rank", c_int32), ("scale", c_float), ("n_seqs", c_int32),
                ("seq_lens", POINTER(c_int32))]


class _SparseMaskC(ctypes.Structure):
    _fields_ = [("nnz", c_int32), ("row_ptr", c_void_p), ("col_idx", c_void_p), ("col_ptr", c_void_p),
                ("col_ent", c_void_p), ("fwd_ptr", c_void_p), ("fwd_ent", c_void_p), ("bwd_ptr", c_void_p),
                ("bwd_ent", c_void_p)]


class _LayerDescC(ctypes.Structure):
    _fields_ = [("K", c_int32), ("N", c_int32), ("dtype", c_int32), ("flags", c_uint32), ("W", c_void_p),
                ("ldw", c_int64), ("n_tasks", c_int32), ("A", POINTER(c_void_p)), ("B", POINTER(c_void_p)),
                ("L", POINTER(c_void_p)), ("masks", POINTER(POINTER(_SparseMaskC)))]


class _ProfileEntryC(ctypes.Structure):
    _fields_ = [("name", c_char_p), ("launches", c_int32), ("total_ms", ctypes.c_double), ("bytes", ctypes.c_double)]


class _AttnDescC(ctypes.Structure):
    _fields_ = [("n_heads", c_int32), ("n_kv_heads", c_int32), ("head_dim", c_int32), ("dtype", c_int32),
                ("scale", c_float), ("ldq", c_int64), ("ldk", c_int64), ("ldv", c_int64), ("ldo", c_int64)]


class AttnDesc:
    """mux_attn_desc (include/mux_attn.h)."""

    def __init__(self, n_heads: int, head_dim: int, ldq: int, ldk: int, ldv: int, ldo: int, scale: float = 0.0,
                 n_kv_heads: Optional[int] = None, dtype: int = MUX_DT_BF16):
        self.c = _AttnDescC(int(n_heads), int(n_heads if n_kv_heads is None else n_kv_heads), int(head_dim), int(dtype),
                            float(scale), int(ldq), int(ldk), int(ldv), int(ldo))


class _CurveC(ctypes.Structure):
    _fields_ = [("n_points", c_int32), ("tokens", POINTER(c_int64)), ("value", POINTER(ctypes.c_double))]


class _StageModelC(ctypes.Structure):
    _fields_ = [("n_gpus", c_int32), ("n_baseops", c_int32), ("baseop_latency", POINTER(_CurveC)),
                ("n_adapters", c_int32), ("adapter_latency", POINTER(_CurveC)), ("adapter_util", POINTER(_CurveC))]


class _CostModelC(ctypes.Structure):
    _fields_ = [("n_stages", c_int32), ("stages", POINTER(_StageModelC)), ("n_microbatches", c_int32)]


class CostModel:
    """mux_cost_model (include/mux_plan.h) laid out from plain Python data:
    stages = [{"n_gpus": N_g, "baseops": [(tokens, values), ...], "adapters": [((tokens, t_a), (tokens, u_a)), ...]}, ...],
    C = number of micro-batches.  Marshalling only; the arrays stay alive with the object."""

    def __init__(self, stages, C: int):
        self._keep = []

        def curves(items):
            arr = (_CurveC * max(len(items), 1))()
            for i, (xs, ys) in enumerate(items):
                tx = (c_int64 * max(len(xs), 1))(*[int(v) for v in xs])
                ty = (ctypes.c_double * max(len(ys), 1))(*[float(v) for v in ys])
                self._keep += [tx, ty]
                arr[i] = _CurveC(min(len(xs), len(ys)), ctypes.cast(tx, POINTER(c_int64)),
                                 ctypes.cast(ty, POINTER(ctypes.c_double)))
            self._keep.append(arr)
            return ctypes.cast(arr, POINTER(_CurveC))

        sarr = (_StageModelC * max(len(stages), 1))()
        for i, st in enumerate(stages):
            sarr[i] = _StageModelC(int(st["n_gpus"]), len(st["baseops"]), curves(list(st["baseops"])),
                                   len(st["adapters"]), curves([a[0] for a in st["adapters"]]),
                                   curves([a[1] for a in st["adapters"]]))
        self._keep.append(sarr)
        self.c = _CostModelC(len(stages), ctypes.cast(sarr, POINTER(_StageModelC)), int(C))


class TaskDesc:
    """Host description of one task: adapter kind, rank, scale and its sequence lengths."""

    def __init__(self, kind: int, rank: int, scale: float, seq_lens: Sequence[int]):
        self.kind, self.rank, self.scale = int(kind), int(rank), float(scale)
        self.seq_lens = [int(v) for v in seq_lens]


def library_path() -> str:
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "libmuxlora.so")


_lib = None


def load_library() -> ctypes.CDLL:
    """Loads the in-tree HIP library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it with `python -m paper_2603_02885_amd.build` "
                          "(or __graft_entry__.build()); there is no fallback path")
    lib = ctypes.CDLL(path)
    vp = c_void_p
    sig = {
        "mux_choose_chunk_size": (c_int, [POINTER(c_int32), c_int32, c_int32, POINTER(c_int32)]),
        "mux_segtab_build": (c_int, [POINTER(_TaskDescC), c_int32, c_int32, c_int32, c_uint32, POINTER(vp)]),
        "mux_segtab_free": (None, [vp]),
        "mux_segtab_rows": (c_int32, [vp]),
        "mux_segtab_n_chunks": (c_int32, [vp]),
        "mux_segtab_n_tasks": (c_int32, [vp]),
        "mux_segtab_valid_tokens": (c_int32, [vp]),
        "mux_segtab_serialized_bytes": (c_size_t, [vp]),
        "mux_segtab_serialize": (c_int, [vp, vp, c_size_t]),
        "mux_segtab_row_task": (c_int, [vp, POINTER(c_int32), c_size_t]),
        "mux_segtab_device_bytes": (c_size_t, [vp]),
        "mux_segtab_upload": (c_int, [vp, vp, c_size_t, vp]),
        "mux_sparse_mask_layout": (c_int, [POINTER(c_int32), POINTER(c_int32), c_int32, c_int32, c_int32, POINTER(c_int32),
                                           POINTER(c_int32), POINTER(c_int32), POINTER(c_int32)]),
        "mux_sparse_mask_tile_layout": (c_int, [POINTER(c_int32), POINTER(c_int32), c_int32, c_int32, c_int32,
                                                POINTER(c_int32), POINTER(c_int32), POINTER(c_int32), POINTER(c_int32)]),
        "mux_lora_saved_bytes": (c_size_t, [POINTER(_LayerDescC), vp]),
        "mux_lora_workspace_bytes": (c_size_t, [POINTER(_LayerDescC), vp]),
        "mux_lora_forward": (c_int, [POINTER(_LayerDescC), vp, vp, vp, vp, vp, vp, c_size_t, vp]),
        "mux_lora_backward": (c_int, [POINTER(_LayerDescC), vp, vp, vp, vp, vp, vp, POINTER(vp), POINTER(vp),
                                      POINTER(vp), c_int, vp, c_size_t, vp]),
        "mux_lora_backward_static_ws": (c_int, [POINTER(_LayerDescC), vp, vp, vp, vp, vp, vp, POINTER(vp), POINTER(vp),
                                                POINTER(vp), c_int, vp]),
        "mux_profile_enable": (c_int, [c_int]),
        "mux_profile_collect": (c_int, [POINTER(_ProfileEntryC), c_int32, POINTER(c_int32)]),
        "mux_last_error": (c_char_p, []),
        "mux_version": (c_char_p, []),
        "mux_probe_mfma_operand_bytes": (c_size_t, []),
        "mux_probe_mfma_sink_bytes": (c_size_t, []),
        "mux_probe_mfma": (c_int, [vp, vp, c_int32, vp, POINTER(ctypes.c_double)]),
        "mux_probe_read_sink_bytes": (c_size_t, []),
        "mux_probe_read": (c_int, [vp, c_size_t, vp, vp]),
        "mux_diag_set_clock_buffer": (c_int, [vp]),
        "mux_dispatch_gather": (c_int, [vp, vp, POINTER(vp), c_int64, vp, c_int64, c_int32, c_int32, vp]),
        "mux_dispatch_scatter": (c_int, [vp, vp, vp, c_int64, POINTER(vp), c_int64, c_int32, c_int32, vp]),
        "mux_attn_saved_bytes": (c_size_t, [POINTER(_AttnDescC), vp]),
        "mux_attn_workspace_bytes": (c_size_t, [POINTER(_AttnDescC), vp]),
        "mux_attn_forward": (c_int, [POINTER(_AttnDescC), vp, vp, vp, vp, vp, vp, vp, vp]),
        "mux_attn_backward": (c_int, [POINTER(_AttnDescC), vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, c_size_t, vp]),
        "mux_plan_stage_latency": (c_int, [POINTER(_CostModelC), c_int32, c_int32, POINTER(c_int64), POINTER(ctypes.c_double)]),
        "mux_plan_htask_latency": (c_int, [POINTER(_CostModelC), c_int32, POINTER(c_int64), POINTER(ctypes.c_double)]),
        "mux_plan_fusion": (c_int, [POINTER(_CostModelC), c_int32, POINTER(c_int64), c_int32, POINTER(c_int32),
                                    POINTER(c_int32), POINTER(c_int32), POINTER(ctypes.c_double)]),
    }
    for name, (res, args) in sig.items():
        f = getattr(lib, name)
        f.restype = res
        f.argtypes = args
    _lib = lib
    return lib


def _check(status: int) -> None:
    if status != MUX_OK:
        raise MuxError(status, load_library().mux_last_error().decode())


def _ptr(x) -> Optional[int]:
    """Device (or host) address of a tensor / array / int / None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if hasattr(x, "data_ptr"):
        return int(x.data_ptr())
    if isinstance(x, np.ndarray):
        return int(x.ctypes.data)
    raise TypeError(f"cannot take the address of {type(x)}")


def _stream(stream) -> Optional[int]:
    if stream is None:
        return None
    if isinstance(stream, int):
        return stream
    return int(stream.cuda_stream)      # torch.cuda.Stream


def _ptr_array(items: Optional[Sequence], n: int):
    arr = (c_void_p * max(n, 1))()
    if items is not None:
        if len(items) != n:
            raise ValueError("per-task pointer list has the wrong length")
        for i, it in enumerate(items):
            arr[i] = _ptr(it)
    return arr


class SegTab:
    """Owner of a host mux_segtab handle (freed with the object)."""

    def __init__(self, handle: int):
        self.handle = handle

    def __del__(self):
        h, self.handle = getattr(self, "handle", None), None
        if h and _lib is not None:
            _lib.mux_segtab_free(h)


def mux_sparse_mask_layout(k, n, K: int, N: int):
    """The two listings of a mask as host arrays (row_ptr [K+1], col_idx [nnz], col_ptr [N+1], col_ent [2 nnz]), laid
    out by the library from the entries (k[e], n[e]) sorted by (k, n)."""
    k = np.ascontiguousarray(k, dtype=np.int32)
    n = np.ascontiguousarray(n, dtype=np.int32)
    if k.shape != n.shape or k.ndim != 1:
        raise ValueError("k and n must be one-dimensional arrays of the same length")
    nnz = int(k.size)
    row_ptr = np.zeros(K + 1, dtype=np.int32)
    col_ptr = np.zeros(N + 1, dtype=np.int32)
    col_idx = np.zeros(max(nnz, 1), dtype=np.int32)
    col_ent = np.zeros(max(2 * nnz, 2), dtype=np.int32)
    ip = lambda a: a.ctypes.data_as(POINTER(c_int32))
    _check(load_library().mux_sparse_mask_layout(ip(k), ip(n), nnz, int(K), int(N), ip(row_ptr), ip(col_idx),
                                                 ip(col_ptr), ip(col_ent)))
    return row_ptr, col_idx, col_ptr, col_ent


def mux_sparse_mask_tile_layout(k, n, K: int, N: int):
    """The listing by tiles of a mask as host arrays (fwd_ptr, fwd_ent [2 nnz], bwd_ptr, bwd_ent [2 nnz]), laid out by
    the library from the entries (k[e], n[e]) sorted by (k, n)."""
    k = np.ascontiguousarray(k, dtype=np.int32)
    n = np.ascontiguousarray(n, dtype=np.int32)
    if k.shape != n.shape or k.ndim != 1:
        raise ValueError("k and n must be one-dimensional arrays of the same length")
    nnz = int(k.size)
    fwd_ptr = np.zeros(((K + 63) // 64) * ((N + 127) // 128) + 1, dtype=np.int32)
    bwd_ptr = np.zeros(((N + 63) // 64) * ((K + 127) // 128) + 1, dtype=np.int32)
    fwd_ent = np.zeros(max(2 * nnz, 2), dtype=np.int32)
    bwd_ent = np.zeros(max(2 * nnz, 2), dtype=np.int32)
    ip = lambda a: a.ctypes.data_as(POINTER(c_int32))
    _check(load_library().mux_sparse_mask_tile_layout(ip(k), ip(n), nnz, int(K), int(N), ip(fwd_ptr), ip(fwd_ent),
                                                      ip(bwd_ptr), ip(bwd_ent)))
    return fwd_ptr, fwd_ent, bwd_ptr, bwd_ent


class SparseMask:
    """Mirror of mux_sparse_mask.  Built from the masked entries (k[nnz], n[nnz]) sorted by (k, n): the library lays the
    row-major listing (row_ptr, col_idx), the column-by-column listing (col_ptr, col_ent) and, unless `tiles` is False,
    the listing by tiles out on the host (mux_sparse_mask_layout, mux_sparse_mask_tile_layout); `to_device` is a
    callable that turns an int32 numpy array into an object with a device pointer (for instance
    lambda a: torch.from_numpy(a).cuda())."""

    def __init__(self, k, n, K: int, N: int, to_device, tiles: bool = True):
        row_ptr, col_idx, col_ptr, col_ent = mux_sparse_mask_layout(k, n, K, N)
        self.nnz = int(np.asarray(k).size)
        self._bufs = [to_device(row_ptr), to_device(col_idx), to_device(col_ptr), to_device(col_ent)]
        self.c = _SparseMaskC(nnz=self.nnz, row_ptr=_ptr(self._bufs[0]), col_idx=_ptr(self._bufs[1]),
                              col_ptr=_ptr(self._bufs[2]), col_ent=_ptr(self._bufs[3]))
        if tiles:
            self._bufs += [to_device(a) for a in mux_sparse_mask_tile_layout(k, n, K, N)]
            self.c.fwd_ptr, self.c.fwd_ent = _ptr(self._bufs[4]), _ptr(self._bufs[5])
            self.c.bwd_ptr, self.c.bwd_ent = _ptr(self._bufs[6]), _ptr(self._bufs[7])


class LayerDesc:
    """Mirror of mux_layer_desc; keeps the pointer arrays alive."""

    def __init__(self, K: int, N: int, dtype: int, W, n_tasks: int, A=None, B=None, L=None, ldw: Optional[int] = None,
                 flags: int = 0, masks=None):
        self._A = _ptr_array(A, n_tasks)
        self._B = _ptr_array(B, n_tasks)
        self._L = _ptr_array(L, n_tasks)
        self._keep = (W, A, B, L, masks)
        self._masks = (POINTER(_SparseMaskC) * max(n_tasks, 1))()
        if masks is not None:
            for t in range(n_tasks):
                if masks[t] is not None:
                    self._masks[t] = ctypes.pointer(masks[t].c)
        self.c = _LayerDescC(K=int(K), N=int(N), dtype=int(dtype), flags=int(flags), W=_ptr(W),
                             ldw=int(N if ldw is None else ldw), n_tasks=int(n_tasks),
                             A=ctypes.cast(self._A, POINTER(c_void_p)), B=ctypes.cast(self._B, POINTER(c_void_p)),
                             L=ctypes.cast(self._L, POINTER(c_void_p)),
                             masks=ctypes.cast(self._masks, POINTER(POINTER(_SparseMaskC))) if masks is not None else None)
        self.n_tasks = int(n_tasks)


# ------------------------------------------------------------------ same names as the header

def mux_last_error() -> str:
    return load_library().mux_last_error().decode()


def mux_version() -> str:
    return load_library().mux_version().decode()


def mux_probe_mfma_operand_bytes() -> int:
    return int(load_library().mux_probe_mfma_operand_bytes())


def mux_probe_mfma_sink_bytes() -> int:
    return int(load_library().mux_probe_mfma_sink_bytes())


def mux_probe_read_sink_bytes() -> int:
    return int(load_library().mux_probe_read_sink_bytes())


def mux_diag_set_clock_buffer(dev_four_u64) -> None:
    """Device buffer of four zeroed 64-bit words the matrix-core kernels add their cycle and 100 MHz tick counts to
    (None switches it off)."""
    _check(load_library().mux_diag_set_clock_buffer(_ptr(dev_four_u64)))


def mux_probe_read(dev_buf, nbytes: int, dev_sink, stream=None) -> None:
    """Launches the plain read stream over nbytes bytes of dev_buf."""
    _check(load_library().mux_probe_read(_ptr(dev_buf), int(nbytes), _ptr(dev_sink), _stream(stream)))


def mux_probe_mfma(dev_operands, dev_sink, iters: int, stream=None) -> float:
    """Launches the register-only MFMA loop; returns the floating-point operations of the launch."""
    flop = ctypes.c_double(0.0)
    _check(load_library().mux_probe_mfma(_ptr(dev_operands), _ptr(dev_sink), int(iters), _stream(stream), ctypes.byref(flop)))
    return float(flop.value)


def mux_choose_chunk_size(lens: Sequence[int], floor_: int = 64) -> int:
    arr = (c_int32 * max(len(lens), 1))(*[int(v) for v in lens])
    out = c_int32(0)
    _check(load_library().mux_choose_chunk_size(arr, len(lens), int(floor_), ctypes.byref(out)))
    return int(out.value)


def mux_segtab_build(tasks: Sequence[TaskDesc], chunk: int, max_pack_len: int = 0, flags: int = 0) -> SegTab:
    n = len(tasks)
    descs = (_TaskDescC * max(n, 1))()
    keep = []
    for i, t in enumerate(tasks):
        lens = (c_int32 * max(len(t.seq_lens), 1))(*t.seq_lens)
        keep.append(lens)
        descs[i] = _TaskDescC(t.kind, t.rank, t.scale, len(t.seq_lens), ctypes.cast(lens, POINTER(c_int32)))
    out = c_void_p(None)
    _check(load_library().mux_segtab_build(descs, n, int(chunk), int(max_pack_len), int(flags), ctypes.byref(out)))
    return SegTab(out.value)


def mux_segtab_free(st: SegTab) -> None:
    h, st.handle = st.handle, None
    if h:
        load_library().mux_segtab_free(h)


def mux_segtab_rows(st: SegTab) -> int:
    return int(load_library().mux_segtab_rows(st.handle))


def mux_segtab_n_chunks(st: SegTab) -> int:
    return int(load_library().mux_segtab_n_chunks(st.handle))


def mux_segtab_n_tasks(st: SegTab) -> int:
    return int(load_library().mux_segtab_n_tasks(st.handle))


def mux_segtab_valid_tokens(st: SegTab) -> int:
    return int(load_library().mux_segtab_valid_tokens(st.handle))


def mux_segtab_serialized_bytes(st: SegTab) -> int:
    return int(load_library().mux_segtab_serialized_bytes(st.handle))


def mux_segtab_serialize(st: SegTab) -> np.ndarray:
    n = mux_segtab_serialized_bytes(st)
    out = np.zeros(n // 4, dtype="<i4")
    _check(load_library().mux_segtab_serialize(st.handle, out.ctypes.data, n))
    return out


def mux_segtab_row_task(st: SegTab) -> np.ndarray:
    T = mux_segtab_rows(st)
    out = np.zeros(max(T, 1), dtype=np.int32)
    _check(load_library().mux_segtab_row_task(st.handle, out.ctypes.data_as(POINTER(c_int32)), out.size))
    return out[:T]


def mux_segtab_device_bytes(st: SegTab) -> int:
    return int(load_library().mux_segtab_device_bytes(st.handle))


def mux_segtab_upload(st: SegTab, dev_dst, cap: int, stream=None) -> None:
    _check(load_library().mux_segtab_upload(st.handle, _ptr(dev_dst), int(cap), _stream(stream)))


def mux_lora_saved_bytes(layer: LayerDesc, st: SegTab) -> int:
    return int(load_library().mux_lora_saved_bytes(ctypes.byref(layer.c), st.handle))


def mux_lora_workspace_bytes(layer: LayerDesc, st: SegTab) -> int:
    return int(load_library().mux_lora_workspace_bytes(ctypes.byref(layer.c), st.handle))


def mux_lora_forward(layer: LayerDesc, st: SegTab, dev_segtab, X, Y, saved, ws, ws_bytes: int, stream=None) -> None:
    _check(load_library().mux_lora_forward(ctypes.byref(layer.c), st.handle, _ptr(dev_segtab), _ptr(X), _ptr(Y),
                                           _ptr(saved), _ptr(ws), int(ws_bytes), _stream(stream)))


def mux_lora_backward(layer: LayerDesc, st: SegTab, dev_segtab, X, dY, saved, dX, dA, dB, dL, accumulate: int,
                      ws, ws_bytes: int, stream=None) -> None:
    n = layer.n_tasks
    pa, pb, pl = _ptr_array(dA, n), _ptr_array(dB, n), _ptr_array(dL, n)
    _check(load_library().mux_lora_backward(
        ctypes.byref(layer.c), st.handle, _ptr(dev_segtab), _ptr(X), _ptr(dY), _ptr(saved), _ptr(dX),
        ctypes.cast(pa, POINTER(c_void_p)), ctypes.cast(pb, POINTER(c_void_p)), ctypes.cast(pl, POINTER(c_void_p)),
        int(accumulate), _ptr(ws), int(ws_bytes), _stream(stream)))


def mux_lora_backward_static_ws(layer: LayerDesc, st: SegTab, dev_segtab, X, dY, saved, dX, dA, dB, dL, accumulate: int,
                                stream=None) -> None:
    n = layer.n_tasks
    pa, pb, pl = _ptr_array(dA, n), _ptr_array(dB, n), _ptr_array(dL, n)
    _check(load_library().mux_lora_backward_static_ws(
        ctypes.byref(layer.c), st.handle, _ptr(dev_segtab), _ptr(X), _ptr(dY), _ptr(saved), _ptr(dX),
        ctypes.cast(pa, POINTER(c_void_p)), ctypes.cast(pb, POINTER(c_void_p)), ctypes.cast(pl, POINTER(c_void_p)),
        int(accumulate), _stream(stream)))


def mux_profile_enable(on) -> None:
    """0/False off, 1/True every kernel, 2 backbone GEMM kernels only."""
    _check(load_library().mux_profile_enable(int(on)))


def mux_profile_collect(cap: int = 64) -> List[dict]:
    """Per-kernel [{name, launches, total_ms}] since the last collect (waits for the events)."""
    arr = (_ProfileEntryC * cap)()
    n = c_int32(0)
    _check(load_library().mux_profile_collect(arr, cap, ctypes.byref(n)))
    return [{"name": arr[i].name.decode(), "launches": int(arr[i].launches), "total_ms": float(arr[i].total_ms),
             "bytes": float(arr[i].bytes)}
            for i in range(min(n.value, cap))]


def _tokens_c(tokens: Sequence[int]):
    return (c_int64 * max(len(tokens), 1))(*[int(v) for v in tokens])


def mux_plan_stage_latency(model: CostModel, stage: int, tokens: Sequence[int]) -> float:
    out = ctypes.c_double(0.0)
    _check(load_library().mux_plan_stage_latency(ctypes.byref(model.c), int(stage), len(tokens), _tokens_c(tokens),
                                                 ctypes.byref(out)))
    return float(out.value)


def mux_plan_htask_latency(model: CostModel, tokens: Sequence[int]) -> float:
    out = ctypes.c_double(0.0)
    _check(load_library().mux_plan_htask_latency(ctypes.byref(model.c), len(tokens), _tokens_c(tokens), ctypes.byref(out)))
    return float(out.value)


def mux_plan_fusion(model: CostModel, tokens: Sequence[int], max_htasks: int = 0):
    """Returns (latency, order, htask_begin): hybrid task h holds the tasks order[htask_begin[h]:htask_begin[h+1]]."""
    n = len(tokens)
    order = (c_int32 * max(n, 1))()
    begins = (c_int32 * (n + 1))()
    nh = c_int32(0)
    lat = ctypes.c_double(0.0)
    _check(load_library().mux_plan_fusion(ctypes.byref(model.c), n, _tokens_c(tokens), int(max_htasks), order, begins,
                                          ctypes.byref(nh), ctypes.byref(lat)))
    return float(lat.value), [int(order[i]) for i in range(n)], [int(begins[i]) for i in range(nh.value + 1)]


def mux_attn_saved_bytes(desc: AttnDesc, st: SegTab) -> int:
    return int(load_library().mux_attn_saved_bytes(ctypes.byref(desc.c), st.handle))


def mux_attn_workspace_bytes(desc: AttnDesc, st: SegTab) -> int:
    return int(load_library().mux_attn_workspace_bytes(ctypes.byref(desc.c), st.handle))


def mux_attn_forward(desc: AttnDesc, st: SegTab, dev_segtab, Q, K, V, O, saved, stream=None) -> None:
    _check(load_library().mux_attn_forward(ctypes.byref(desc.c), st.handle, _ptr(dev_segtab), _ptr(Q), _ptr(K), _ptr(V),
                                           _ptr(O), _ptr(saved), _stream(stream)))


def mux_attn_backward(desc: AttnDesc, st: SegTab, dev_segtab, Q, K, V, O, dO, saved, dQ, dK, dV, ws, ws_bytes: int,
                      stream=None) -> None:
    _check(load_library().mux_attn_backward(ctypes.byref(desc.c), st.handle, _ptr(dev_segtab), _ptr(Q), _ptr(K), _ptr(V),
                                            _ptr(O), _ptr(dO), _ptr(saved), _ptr(dQ), _ptr(dK), _ptr(dV), _ptr(ws),
                                            int(ws_bytes), _stream(stream)))


def mux_dispatch_gather(st: SegTab, dev_segtab, task_ptrs: Sequence, ld_task: int, aligned, ld_aligned: int, width: int,
                        elem_bytes: int, stream=None) -> None:
    arr = _ptr_array(task_ptrs, len(task_ptrs))
    _check(load_library().mux_dispatch_gather(st.handle, _ptr(dev_segtab), ctypes.cast(arr, POINTER(c_void_p)), int(ld_task),
                                              _ptr(aligned), int(ld_aligned), int(width), int(elem_bytes), _stream(stream)))


def mux_dispatch_scatter(st: SegTab, dev_segtab, aligned, ld_aligned: int, task_ptrs: Sequence, ld_task: int, width: int,
                         elem_bytes: int, stream=None) -> None:
    arr = _ptr_array(task_ptrs, len(task_ptrs))
    _check(load_library().mux_dispatch_scatter(st.handle, _ptr(dev_segtab), _ptr(aligned), int(ld_aligned),
                                               ctypes.cast(arr, POINTER(c_void_p)), int(ld_task), int(width),
                                               int(elem_bytes), _stream(stream)))
