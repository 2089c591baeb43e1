"""Pins of the attention oracle (oracle/attention.py): a hand-worked example, closed forms, explicit double loops on
tiny inputs, finite differences, and the properties the chunk-aligned layout must keep (section 3.5)."""
import json
import math
import os

import numpy as np
import pytest

from oracle import attention, segtab

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "attention_hand_example.json")


def loops_forward(Q, K, V, seqs, H, scale):
    """The definition with explicit sums, one output element at a time."""
    T, HD = Q.shape
    d = HD // H
    O = np.zeros((T, HD))
    for first, n in seqs:
        for h in range(H):
            for i in range(n):
                w = [math.exp(scale * sum(Q[first + i, h * d + c] * K[first + j, h * d + c] for c in range(d)))
                     for j in range(i + 1)]
                z = sum(w)
                for c in range(d):
                    O[first + i, h * d + c] = sum(w[j] * V[first + j, h * d + c] for j in range(i + 1)) / z
    return O


def check_pins(att):
    g = json.load(open(GOLDEN))
    seqs = [tuple(s) for s in g["seqs"]]
    f = att.forward(g["Q"], g["K"], g["V"], seqs, g["n_heads"], g["scale"])
    assert np.allclose(f["O"], g["O"], rtol=1e-13, atol=1e-13) and np.allclose(f["lse"], g["lse"], rtol=1e-13, atol=1e-13)
    b = att.backward(g["Q"], g["K"], g["V"], g["dO"], seqs, g["n_heads"], g["scale"])
    for k in ("dQ", "dK", "dV"):
        assert np.allclose(b[k], g[k], rtol=1e-13, atol=1e-13), k
    rng = np.random.default_rng(5)
    H, d = 2, 3
    seqs = [(1, 4), (5, 1), (8, 5)]                         # rows 0, 6, 7, 13 are padding
    T = 14
    Q, K, V, dO = (rng.standard_normal((T, H * d)) for _ in range(4))
    f = att.forward(Q, K, V, seqs, H)
    assert np.allclose(f["O"], loops_forward(Q, K, V, seqs, H, 1.0 / math.sqrt(d)), rtol=1e-12, atol=1e-13)
    pad = [0, 6, 7, 13]
    b = att.backward(Q, K, V, dO, seqs, H)
    assert np.all(f["O"][pad] == 0) and all(np.all(b[k][pad] == 0) for k in b)
    # closed forms: all-zero queries weigh every visible key equally -> running means of V; a sequence of one token
    # returns its own V and passes dO to dV
    f0 = att.forward(np.zeros_like(Q), K, V, seqs, H)
    for first, n in seqs:
        assert np.allclose(f0["O"][first:first + n], np.cumsum(V[first:first + n], axis=0) / np.arange(1, n + 1)[:, None])
    assert np.allclose(f["O"][5], V[5]) and np.allclose(b["dV"][5], dO[5]) and np.all(b["dQ"][5] == 0) and np.all(b["dK"][5] == 0)
    # the explicit scale is used as given
    f2 = att.forward(Q, K, V, seqs, H, scale=0.25)
    assert np.allclose(f2["O"], loops_forward(Q, K, V, seqs, H, 0.25), rtol=1e-12, atol=1e-13)
    # central differences of sum(O * dO) in every input
    base = {"Q": Q, "K": K, "V": V}
    for name, gname in (("Q", "dQ"), ("K", "dK"), ("V", "dV")):
        for _ in range(12):
            i, j = int(rng.integers(T)), int(rng.integers(H * d))
            hstep = 1e-5
            vals = []
            for sgn in (+1, -1):
                a = {k: v.copy() for k, v in base.items()}
                a[name][i, j] += sgn * hstep
                vals.append(float((att.forward(a["Q"], a["K"], a["V"], seqs, H)["O"] * dO).sum()))
            fd = (vals[0] - vals[1]) / (2 * hstep)
            want = b[gname][i, j] if i not in pad else 0.0
            assert abs(fd - want) <= 1e-7 * max(1.0, abs(want)), (name, i, j, fd, want)
    # causality: a later token changes nothing before it; isolation: another sequence (or padding) changes nothing
    K2, V2 = K.copy(), V.copy()
    K2[11] += 3.0; V2[11] -= 2.0; K2[0] = np.nan; V2[6] = np.inf
    f3 = att.forward(Q, K2, V2, seqs, H)
    assert np.array_equal(f3["O"][:11], f["O"][:11]) and not np.allclose(f3["O"][11:13], f["O"][11:13])
    # heads are independent
    Q4 = Q.copy(); Q4[:, d:] *= -1.5
    f4 = att.forward(Q4, K, V, seqs, H)
    assert np.array_equal(f4["O"][:, :d], f["O"][:, :d])
    # a sequence gives the same rows wherever the table puts it: alone, packed behind another one, cut by small chunks
    lens = [[5, 3], [4]]
    ref = {}
    for chunk, mpl in ((16, 0), (2, 0), (4, 5)):
        st = segtab.build(lens, chunk, mpl)
        sq = segtab.sequences(st)
        r2 = np.random.default_rng(11)
        per_seq = [tuple(r2.standard_normal((3, n, H * d))) for n in (5, 3, 4)]
        Qa, Ka, Va = (np.full((st.T, H * d), np.nan) for _ in range(3))
        for (t, p, first, n), (q, k, v) in zip(sq, per_seq):
            Qa[first:first + n], Ka[first:first + n], Va[first:first + n] = q, k, v
        out = att.forward(Qa, Ka, Va, [(s[2], s[3]) for s in sq], H)["O"]
        for si, (t, p, first, n) in enumerate(sq):
            if si in ref:
                assert np.array_equal(out[first:first + n], ref[si])
            ref[si] = out[first:first + n]


def check_gqa(att):
    """Grouped-query heads: the same as ordinary heads on keys and values repeated for every query head of a group,
    with the key/value gradients of the copies added up."""
    rng = np.random.default_rng(21)
    H, Hkv, d = 4, 2, 3
    seqs = [(0, 5), (6, 3)]
    T = 10
    Q, dO = rng.standard_normal((T, H * d)), rng.standard_normal((T, H * d))
    K, V = rng.standard_normal((T, Hkv * d)), rng.standard_normal((T, Hkv * d))
    rep = lambda a: np.concatenate([a[:, (h // 2) * d:(h // 2 + 1) * d] for h in range(H)], axis=1)
    f = att.forward(Q, K, V, seqs, H, n_kv_heads=Hkv)
    fr = att.forward(Q, rep(K), rep(V), seqs, H)
    assert np.array_equal(f["O"], fr["O"]) and np.array_equal(f["lse"], fr["lse"])
    b = att.backward(Q, K, V, dO, seqs, H, n_kv_heads=Hkv)
    br = att.backward(Q, rep(K), rep(V), dO, seqs, H)
    assert np.array_equal(b["dQ"], br["dQ"])
    fold = lambda a: np.concatenate([a[:, (2 * g) * d:(2 * g + 1) * d] + a[:, (2 * g + 1) * d:(2 * g + 2) * d] for g in range(Hkv)], axis=1)
    assert np.allclose(b["dK"], fold(br["dK"]), rtol=1e-13, atol=1e-13) and np.allclose(b["dV"], fold(br["dV"]), rtol=1e-13, atol=1e-13)
    assert not np.allclose(b["dK"][:, :d], br["dK"][:, :d])          # really a sum over the group
    bm = att.backward(Q, rep(K), rep(V), dO, seqs, H, n_kv_heads=H)
    assert all(np.array_equal(bm[k], br[k]) for k in br)             # Hkv = H is the ordinary case


def test_attention_oracle_gqa():
    check_gqa(attention)


def test_attention_oracle_pins():
    check_pins(attention)


MUTATIONS = [
    ("s = scale * (q @ k.T)", "s = (q @ k.T)"),                                              # scale dropped
    ("np.tril(np.ones((n, n), dtype=bool))", "np.tril(np.ones((n, n), dtype=bool), -1) | np.eye(n, dtype=bool) * (np.arange(n) == 0)[:, None]"),
    ("np.tril(np.ones((n, n), dtype=bool))", "np.ones((n, n), dtype=bool)"),                 # not causal
    ("lse[h, r] = l", "lse[h, r] = l - np.log(n)"),
    ("ds = p * (dp - (dp * p).sum(axis=1, keepdims=True))", "ds = p * dp"),                  # softmax slope without its sum term
    ("dQ[r, c] = scale * (ds @ K[r, ck])", "dQ[r, c] = (ds @ K[r, ck])"),
    ("dK[r, ck] += scale * (ds.T @ Q[r, c])", "dK[r, ck] += scale * (ds @ Q[r, c])"),            # transposed operand
    ("dV[r, ck] += p.T @ dO[r, c]", "dV[r, ck] += p @ dO[r, c]"),
    ("dp = dO[r, c] @ V[r, ck].T", "dp = dO[r, c] @ K[r, ck].T"),
    ("O[r, c] = p @ V[r, ck]", "O[r, c] = p @ K[r, ck]"),
    ("dV[r, ck] += p.T @ dO[r, c]", "dV[r, ck] = p.T @ dO[r, c]"),                             # last head of a group wins
    ("ck = slice((h // group) * d, (h // group + 1) * d)\n            p, l =", "ck = slice((h % (n_heads // group)) * d, (h % (n_heads // group) + 1) * d)\n            p, l ="),
]


@pytest.mark.parametrize("idx", range(len(MUTATIONS)))
def test_attention_pins_catch_planted_mistakes(idx):
    import types
    old, new = MUTATIONS[idx]
    src = open(attention.__file__).read()
    assert src.count(old) == 1, old
    mod = types.ModuleType("attention_mutant")
    exec(compile(src.replace(old, new), "attention_mutant", "exec"), mod.__dict__)
    with pytest.raises((AssertionError, ValueError, FloatingPointError)):
        with np.errstate(all="ignore"):
            check_pins(mod)
            check_gqa(mod)
