"""TEST INFRASTRUCTURE -- fp64 oracle of the attention step of a chunk-aligned batch (section 3.5).

The aligned batch holds each task's sequences packed one after the other and cut along the chunk grid; a pack longer
than a chunk continues in the next chunks and its later chunks reuse the keys and values of its earlier ones.  What is
computed is therefore plain causal attention of every sequence on its own: a token attends to the tokens of its own
sequence up to itself, never to another sequence of the pack, to another task or to padding.  That definition is
written out here with numpy matmuls in double precision, one (sequence, head) at a time.

Q, dO, O: [T, H * d] (head h in columns h*d .. (h+1)*d - 1); K, V: [T, Hkv * d] with Hkv dividing H (grouped-query
attention: query head h reads key/value head h // (H / Hkv); Hkv = H unless given); seqs: (first_row, len) pairs;
padding rows of the results are zero.  scale = 1 / sqrt(d) unless given.
"""
from __future__ import annotations

from typing import Dict, Optional, Sequence, Tuple

import numpy as np


def _probabilities(q: np.ndarray, k: np.ndarray, scale: float) -> Tuple[np.ndarray, np.ndarray]:
    """Row-wise softmax of the causally masked scores of one sequence and head; also the log of each row's sum."""
    n = q.shape[0]
    s = scale * (q @ k.T)
    s = np.where(np.tril(np.ones((n, n), dtype=bool)), s, -np.inf)       # key j is visible to query i iff j <= i
    m = s.max(axis=1, keepdims=True)
    e = np.exp(s - m)
    z = e.sum(axis=1, keepdims=True)
    return e / z, (m + np.log(z))[:, 0]


def forward(Q, K, V, seqs: Sequence[Tuple[int, int]], n_heads: int, scale: Optional[float] = None,
            n_kv_heads: Optional[int] = None) -> Dict[str, np.ndarray]:
    Q, K, V = (np.asarray(a, dtype=np.float64) for a in (Q, K, V))
    T, HD = Q.shape
    d = HD // n_heads
    group = n_heads // (n_heads if n_kv_heads is None else n_kv_heads)
    scale = 1.0 / np.sqrt(d) if scale is None else float(scale)
    O = np.zeros((T, HD))
    lse = np.zeros((n_heads, T))
    for first, n in seqs:
        r = slice(first, first + n)
        for h in range(n_heads):
            c = slice(h * d, (h + 1) * d)
            ck = slice((h // group) * d, (h // group + 1) * d)
            p, l = _probabilities(Q[r, c], K[r, ck], scale)
            O[r, c] = p @ V[r, ck]
            lse[h, r] = l
    return {"O": O, "lse": lse}


def backward(Q, K, V, dO, seqs: Sequence[Tuple[int, int]], n_heads: int, scale: Optional[float] = None,
             n_kv_heads: Optional[int] = None) -> Dict[str, np.ndarray]:
    """Gradients of sum(O * dO): with P the probabilities, dV = P^T dO, dP = dO V^T,
    dS = P * (dP - rowsum(dP * P)) (softmax), dQ = scale dS K, dK = scale dS^T Q; a key/value head collects the
    contributions of every query head of its group."""
    Q, K, V, dO = (np.asarray(a, dtype=np.float64) for a in (Q, K, V, dO))
    T, HD = Q.shape
    d = HD // n_heads
    group = n_heads // (n_heads if n_kv_heads is None else n_kv_heads)
    scale = 1.0 / np.sqrt(d) if scale is None else float(scale)
    dQ, dK, dV = np.zeros((T, HD)), np.zeros(K.shape), np.zeros(V.shape)
    for first, n in seqs:
        r = slice(first, first + n)
        for h in range(n_heads):
            c = slice(h * d, (h + 1) * d)
            ck = slice((h // group) * d, (h // group + 1) * d)
            p, _ = _probabilities(Q[r, c], K[r, ck], scale)
            dV[r, ck] += p.T @ dO[r, c]
            dp = dO[r, c] @ V[r, ck].T
            ds = p * (dp - (dp * p).sum(axis=1, keepdims=True))
            dQ[r, c] = scale * (ds @ K[r, ck])
            dK[r, ck] += scale * (ds.T @ Q[r, c])
    return {"dQ": dQ, "dK": dK, "dV": dV}
