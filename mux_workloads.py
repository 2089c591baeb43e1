"""Seeded synthetic inputs for the multiplexed PEFT linear layer.

This module only *describes* workloads (shapes, task lists, sequence lengths) and
draws their tensor values.  It holds none of the layer's arithmetic and none of the
chunk-alignment logic: both the CPU oracle and the HIP library consume what it
returns, each with its own table builder and its own kernels.

Workloads stand in for the multi-tenant PEFT mixes the paper evaluates (several
LoRA tasks with independent, variable-length batches on one frozen backbone, §2.1
"Characteristics" and Table 2): a linear layer sees shapes and value
distributions only, so no dataset is needed.

Tensor values: numpy's Philox counter-based generator keyed by (seed, tensor id),
float32 standard normals scaled by the stated sigma, then (bf16 mode) rounded to
bfloat16 with round-to-nearest-even and returned as float32 holding exactly
representable bf16 values.
"""
from __future__ import annotations

import zlib
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

KIND_NONE = 0
KIND_LORA = 1
KIND_IA3 = 2
KIND_DIFF = 4      # selective kind (Diff-Pruning): trainable values on a fixed sparse mask over W; values in the A slot
KIND_ADAPTER = 3   # additive bottleneck after the BaseOp (Adapter-Tuning): D [N, r] in the A slot, U [r, N] in the B slot


@dataclass
class Task:
    kind: int
    rank: int
    scale: float
    seq_lens: List[int]
    density: float = 0.0       # KIND_DIFF: fraction of the entries of W that are trainable

    @property
    def tokens(self) -> int:
        return int(sum(self.seq_lens))


@dataclass
class Workload:
    name: str
    layers: List[Tuple[str, int, int]]          # (name, K, N): Y[T,N] = X[T,K] W[K,N]
    tasks: List[Task]
    chunk: int
    max_pack_len: int = 0
    sigma_w: float = 0.02
    sigma_ab: float = 0.02
    notes: str = ""

    @property
    def valid_tokens(self) -> int:
        return sum(t.tokens for t in self.tasks)


# --------------------------------------------------------------------------- values

def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """float32 -> nearest bfloat16 (ties to even), returned as float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    nan = np.isnan(x)
    if nan.any():
        r = np.where(nan, np.uint32(0x7FC00000), r)
    return r.view(np.float32)


def _key(seed: int, tensor_id: str) -> List[int]:
    return [int(seed) & 0xFFFFFFFFFFFFFFFF, zlib.crc32(tensor_id.encode()) | (1 << 40)]


def normal(seed: int, tensor_id: str, shape: Sequence[int], sigma: float = 1.0,
           mean: float = 0.0, bf16: bool = True) -> np.ndarray:
    """Seeded N(mean, sigma) float32 tensor; values depend only on (seed, tensor_id, shape)."""
    gen = np.random.Generator(np.random.Philox(key=_key(seed, tensor_id)))
    out = gen.standard_normal(size=tuple(int(s) for s in shape), dtype=np.float32)
    if sigma != 1.0:
        out *= np.float32(sigma)
    if mean != 0.0:
        out += np.float32(mean)
    return round_to_bf16(out) if bf16 else out


def integers(seed: int, tensor_id: str, low: int, high_incl: int, n: int) -> np.ndarray:
    gen = np.random.Generator(np.random.Philox(key=_key(seed, tensor_id)))
    return gen.integers(low, high_incl + 1, size=n, dtype=np.int64)


def lognormal_lengths(seed: int, tensor_id: str, n: int, median: float, sigma: float,
                      cap: int) -> np.ndarray:
    gen = np.random.Generator(np.random.Philox(key=_key(seed, tensor_id)))
    z = gen.standard_normal(size=n)
    l = np.rint(np.exp(np.log(median) + sigma * z)).astype(np.int64)
    return np.clip(l, 1, cap)


# --------------------------------------------------------------------------- workloads

def _llama_layers(h: int, mlp: int) -> List[Tuple[str, int, int]]:
    return [("q", h, h), ("k", h, h), ("v", h, h), ("o", h, h),
            ("gate", h, mlp), ("up", h, mlp), ("down", mlp, h)]


def config(idx: int, seed: int = 0) -> Workload:
    """The five benchmark workloads (index 0..4), and an extra one for the additive kind (5)."""
    if idx == 0:
        return Workload(
            name="tiny", layers=[("w", 256, 256)], chunk=64,
            tasks=[Task(KIND_LORA, 8, 2.0, [100]), Task(KIND_LORA, 8, 2.0, [150])],
            notes="2 LoRA r8 tasks, 100+150 tokens, chunk 64")
    if idx == 1:
        return Workload(
            name="llama7b", layers=_llama_layers(4096, 11008), chunk=512,
            tasks=[Task(KIND_LORA, 16, 2.0, [n]) for n in (2048, 1536, 1024, 512)],
            notes="4 LoRA r16 tasks, 5120 tokens, chunk 512")
    if idx == 2:
        tasks = []
        for t in range(16):
            r = (8, 16, 32, 64)[t // 4]
            lens = lognormal_lengths(seed, f"c3.len.{t}", 8, 128.0, 0.7, 1024)
            tasks.append(Task(KIND_LORA, r, 2.0, [int(v) for v in lens]))
        return Workload(
            name="small_ops", layers=_llama_layers(4096, 11008), chunk=256, tasks=tasks,
            notes="16 LoRA tasks ranks 8/16/32/64, 8 lognormal sequences each, chunk 256")
    if idx == 3:
        toks = integers(seed, "c4.tokens", 1024, 4096, 8)
        tasks = [Task(KIND_LORA if t < 6 else KIND_IA3, 16 if t < 6 else 0, 2.0, [int(toks[t])])
                 for t in range(8)]
        return Workload(
            name="llama13b", layers=_llama_layers(5120, 13824), chunk=512, tasks=tasks,
            notes="6 LoRA r16 + 2 IA3 tasks, tokens U[1024,4096], chunk 512")
    if idx == 4:
        total = 32768
        lens: List[int] = []
        got = 0
        draw = lognormal_lengths(seed, "c5.len", 4096, 512.0, 0.7, total)
        for v in draw:
            v = int(min(int(v), total - got))
            lens.append(v)
            got += v
            if got == total:
                break
        per_task: List[List[int]] = [[] for _ in range(32)]
        for i, v in enumerate(lens):
            per_task[i % 32].append(v)
        tasks = [Task(KIND_LORA, 16, 2.0, l) for l in per_task]
        layers = [("q", 8192, 1024), ("k", 8192, 1024), ("v", 8192, 1024), ("o", 1024, 8192),
                  ("gate", 8192, 3584), ("up", 8192, 3584), ("down", 3584, 8192)]
        return Workload(
            name="llama70b_tp8_share", layers=layers, chunk=1024, tasks=tasks,
            notes="32 LoRA r16 tasks, 32768 tokens lognormal(512), chunk 1024, 1/8 TP shard shapes")
    if idx == 5:
        # not one of the benchmark configs: the LLaMA-7B shapes with two of the four tasks switched to the additive
        # bottleneck kind (bottleneck width 64, the usual size of that method), to measure that kind's kernels
        kinds = (KIND_LORA, KIND_ADAPTER, KIND_LORA, KIND_ADAPTER)
        tasks = [Task(k, 16 if k == KIND_LORA else 64, 2.0 if k == KIND_LORA else 1.0, [n])
                 for k, n in zip(kinds, (2048, 1536, 1024, 512))]
        return Workload(
            name="llama7b_tuning", layers=_llama_layers(4096, 11008), chunk=512, tasks=tasks,
            notes="2 LoRA r16 + 2 Adapter-Tuning r64 tasks, 5120 tokens, chunk 512")
    if idx == 6:
        # not one of the benchmark configs either: two of the four tasks switched to the selective kind, 0.5 % of the
        # entries of every W trainable (the sparsity that method reports), to measure that kind's kernels
        tasks = [Task(KIND_LORA, 16, 2.0, [2048]), Task(KIND_DIFF, 0, 1.0, [1536], density=0.005),
                 Task(KIND_LORA, 16, 2.0, [1024]), Task(KIND_DIFF, 0, 1.0, [512], density=0.005)]
        return Workload(
            name="llama7b_diff", layers=_llama_layers(4096, 11008), chunk=512, tasks=tasks,
            notes="2 LoRA r16 + 2 Diff-Pruning (0.5 % of W) tasks, 5120 tokens, chunk 512")
    if idx in (7, 8):
        # not benchmark configs: the small-batch regime of the paper's own workload mixes (Table 2: eight tasks of 2-8
        # sequences padded to 64, 128 or 256 tokens), all seven LLaMA-7B projections, LoRA rank 16
        w = table2_workload("A" if idx == 7 else "B", 64 if idx == 7 else 128)
        return Workload(name=w.name, layers=_llama_layers(4096, 11008), chunk=w.chunk, tasks=w.tasks,
                        notes=f"Table 2 mix {'A' if idx == 7 else 'B'}: 8 LoRA r16 tasks, {sum(t.tokens for t in w.tasks)} tokens, chunk {w.chunk}")
    if idx == 9:
        # Table 2's mix A on the backbone the paper runs it on (GPT3-2.7B, Table 3: hidden 2560, 32 heads): the four
        # attention projections and the two matrices of its MLP (4 x hidden)
        w = table2_workload("A", 64)
        layers = [("q", 2560, 2560), ("k", 2560, 2560), ("v", 2560, 2560), ("o", 2560, 2560),
                  ("fc1", 2560, 10240), ("fc2", 10240, 2560)]
        return Workload(name="gpt2p7b_mixA", layers=layers, chunk=w.chunk, tasks=w.tasks,
                        notes=f"Table 2 mix A on GPT3-2.7B shapes: 8 LoRA r16 tasks, {sum(t.tokens for t in w.tasks)} tokens, chunk {w.chunk}")
    raise ValueError(f"no config {idx}")


def table2_workload(which: str, chunk: int, rank: int = 16) -> Workload:
    """Token-count shapes of the paper's Table 2 mixes (batch x padded length), LLaMA-7B shapes.

    Only the shapes are used: task i has `batch` sequences of one padded length
    (64, 128 or 256 tokens, §5.1 "Workloads")."""
    batch = (4, 2, 4, 4, 8, 2, 4, 4)
    length = {"A": (64, 128, 128, 64, 64, 64, 128, 128),
              "B": (256, 64, 256, 64, 64, 256, 256, 256)}[which]
    tasks = [Task(KIND_LORA, rank, 2.0, [l] * b) for b, l in zip(batch, length)]
    return Workload(name=f"table2_{which}_c{chunk}", layers=[("q", 4096, 4096)], chunk=chunk,
                    tasks=tasks, notes="Table 2 shapes")


# --------------------------------------------------------------------------- tensors

@dataclass
class LayerTensors:
    K: int
    N: int
    W: np.ndarray
    A: List[Optional[np.ndarray]]
    B: List[Optional[np.ndarray]]
    L: List[Optional[np.ndarray]]
    X: np.ndarray
    dY: np.ndarray
    extra: Dict[str, np.ndarray] = field(default_factory=dict)
    masks: List[Optional[Tuple[np.ndarray, np.ndarray]]] = field(default_factory=list)   # KIND_DIFF: (k[nnz], n[nnz]) by (k, n)


def layer_tensors(wl: Workload, layer: int, T: int, seed: int = 0, bf16: bool = True,
                  pad_rows: Optional[np.ndarray] = None, pad_fill: Optional[float] = None
                  ) -> LayerTensors:
    """Draw W, adapters, X[T,K] and dY[T,N] for one layer call.

    `pad_rows` (bool[T]) with `pad_fill` overwrites padding rows of X and dY with a
    sentinel, to show that their contents are ignored."""
    name, K, N = wl.layers[layer]
    tag = f"{wl.name}.{name}"
    W = normal(seed, f"{tag}.W", (K, N), wl.sigma_w, bf16=bf16)
    A: List[Optional[np.ndarray]] = []
    B: List[Optional[np.ndarray]] = []
    L: List[Optional[np.ndarray]] = []
    masks: List[Optional[Tuple[np.ndarray, np.ndarray]]] = [None] * len(wl.tasks)
    for t, task in enumerate(wl.tasks):
        if task.kind == KIND_LORA:
            A.append(normal(seed, f"{tag}.A{t}", (K, task.rank), wl.sigma_ab, bf16=bf16))
            B.append(normal(seed, f"{tag}.B{t}", (task.rank, N), wl.sigma_ab, bf16=bf16))
            L.append(None)
        elif task.kind == KIND_ADAPTER:
            A.append(normal(seed, f"{tag}.D{t}", (N, task.rank), wl.sigma_ab, bf16=bf16))
            B.append(normal(seed, f"{tag}.U{t}", (task.rank, N), wl.sigma_ab, bf16=bf16))
            L.append(None)
        elif task.kind == KIND_DIFF:
            # unstructured mask: every entry of W independently with probability `density`, listed by (k, n)
            rng = np.random.Generator(np.random.Philox(key=_key(seed, f"{tag}.M{t}")))
            flat = np.flatnonzero(rng.random(K * N) < task.density).astype(np.int64)
            masks[t] = ((flat // N).astype(np.int32), (flat % N).astype(np.int32))
            A.append(normal(seed, f"{tag}.V{t}", (flat.size,), wl.sigma_ab, bf16=bf16))
            B.append(None)
            L.append(None)
        elif task.kind == KIND_IA3:
            A.append(None)
            B.append(None)
            L.append(normal(seed, f"{tag}.L{t}", (N,), 0.02, mean=1.0, bf16=bf16))
        else:
            A.append(None); B.append(None); L.append(None)
    X = normal(seed, f"{tag}.X", (T, K), 1.0, bf16=bf16)
    dY = normal(seed, f"{tag}.dY", (T, N), 1.0, bf16=bf16)
    if pad_rows is not None and pad_fill is not None:
        X[pad_rows] = np.float32(pad_fill)
        dY[pad_rows] = np.float32(pad_fill)
    return LayerTensors(K=K, N=N, W=W, A=A, B=B, L=L, X=X, dY=dY, masks=masks)
