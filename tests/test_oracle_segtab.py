"""Pins of the oracle's chunk-alignment table (paper section 3.5 and section 5.4)."""
import json
import os

import numpy as np
import pytest

import mux_workloads as wlm
from oracle import segtab


def sections(img):
    h = img[:segtab.HEADER_INTS]
    M, n_chunks, n_packs, n_segs, n_seqs = int(h[3]), int(h[6]), int(h[9]), int(h[10]), int(h[11])
    o = segtab.HEADER_INTS
    out = {"header": h}
    for name, n, w in (("tasks", M, segtab.TASK_INTS), ("packs", n_packs, segtab.PACK_INTS),
                       ("chunks", n_chunks, segtab.CHUNK_INTS), ("segments", n_segs, segtab.SEG_INTS),
                       ("seqs", n_seqs, segtab.SEQ_INTS)):
        out[name] = img[o:o + n * w].reshape(n, w)
        o += n * w
    assert o == img.size
    return out


def test_hand_laid_example(golden_dir):
    g = json.load(open(os.path.join(golden_dir, "segtab_hand_example.json")))
    for mode, flags in (("default", 0), ("dense", segtab.FLAG_DENSE)):
        st = segtab.build(g["tasks"], g["chunk"], g["max_pack_len"], flags)
        e = g[mode]
        exp = sum([e["header"]] + e["tasks"] + e["packs"] + e["chunks"] + e["segments"] + e["seqs"], [])
        assert list(st.image) == exp
        assert list(st.row_task) == e["row_task"]


def test_paper_alignment_cases():
    """Section 5.4: with chunk 64 and sequence lengths 64 / 128 (workload A of Table 2) no
    chunk is padded; with chunk 128, 64-token tasks get intra-chunk zero padding only when
    their packed length is not a multiple of 128."""
    wa = wlm.table2_workload("A", 64)
    st = segtab.build([t.seq_lens for t in wa.tasks], 64)
    assert st.T == st.valid_total == sum(t.tokens for t in wa.tasks) == 2944
    assert np.all(st.row_task >= 0)
    # one 64-token sequence per pack, chunk 128: half of every chunk is padding
    st = segtab.build([[64], [64], [128]], 128, max_pack_len=64)
    s = sections(st.image)
    assert list(s["chunks"][:, 0]) == [64, 64, 128]
    assert st.T == 384 and st.valid_total == 256


def test_config1_has_five_chunks_by_default_and_four_dense():
    wl = wlm.config(0)
    st = segtab.build([t.seq_lens for t in wl.tasks], 64)
    assert (st.n_chunks, st.T, st.valid_total) == (5, 320, 250)
    s = sections(st.image)
    assert list(s["chunks"][:, 0]) == [64, 36, 64, 64, 22]
    st = segtab.build([t.seq_lens for t in wl.tasks], 64, 0, segtab.FLAG_DENSE)
    assert (st.n_chunks, st.T, st.valid_total) == (4, 256, 250)
    s = sections(st.image)
    assert list(s["chunks"][:, 2]) == [1, 2, 1, 1]      # the second chunk holds both tasks


def test_chunk_size_rule():
    """Section 3.5: greatest power-of-two divisor of all lengths, floor 64."""
    assert segtab.choose_chunk_size([64, 128, 256]) == 64
    assert segtab.choose_chunk_size([128, 256]) == 128
    assert segtab.choose_chunk_size([96, 160]) == 64       # divisor 32 is below the floor
    assert segtab.choose_chunk_size([512, 1024, 1536]) == 512
    assert segtab.choose_chunk_size([96, 160], floor=16) == 32
    assert segtab.choose_chunk_size([]) == 64


@pytest.mark.parametrize("seed", range(40))
def test_invariants_on_random_cases(seed):
    rng = np.random.default_rng(seed)
    M = int(rng.integers(1, 7))
    tasks = [[int(v) for v in rng.integers(1, 40, size=int(rng.integers(0, 5)))] for _ in range(M)]
    c = int(2 ** rng.integers(0, 6))
    P = int(rng.choice([0, 0, 16, 50]))
    for flags in (0, segtab.FLAG_DENSE):
        st = segtab.build(tasks, c, P, flags)
        s = sections(st.image)
        assert st.T == st.n_chunks * c
        assert st.valid_total == sum(sum(t) for t in tasks) == int((st.row_task >= 0).sum())
        assert int(s["chunks"][:, 0].sum()) == st.valid_total
        # rows of a chunk are a valid prefix followed by padding
        for ch in range(st.n_chunks):
            rt = st.row_task[ch * c:(ch + 1) * c]
            v = int(s["chunks"][ch, 0])
            assert np.all(rt[:v] >= 0) and np.all(rt[v:] < 0)
            if flags == 0:
                assert len(set(rt[:v].tolist())) <= 1       # one task per chunk
        # a pack's chunks are consecutive, its padding is less than one chunk
        for p in range(len(s["packs"])):
            task, row_begin, valid, chunk_begin, chunk_count, seg_begin = [int(v) for v in s["packs"][p]]
            segs = s["segments"][seg_begin:seg_begin + chunk_count]
            assert list(segs[:, 2]) == list(range(chunk_begin, chunk_begin + chunk_count))
            assert list(segs[:, 5]) == list(range(chunk_count))
            assert int(segs[:, 4].sum()) == valid
            assert np.all(segs[:, 1] == p) and np.all(segs[:, 0] == task)
            if flags == 0:
                assert chunk_count == -(-valid // c) and row_begin == chunk_begin * c
            if P > 0:
                lens = [int(q[3]) for q in s["seqs"] if int(q[1]) == p]
                assert sum(lens) == valid and (valid <= P or len(lens) == 1)
        # tasks in caller order, rows ascending, token order preserved
        pos = 0
        for t in range(M):
            rows = st.task_rows[t]
            assert len(rows) == sum(tasks[t])
            if len(rows):
                assert rows[0] >= pos
                pos = rows[-1] + 1
        if flags == segtab.FLAG_DENSE:
            assert np.all(st.row_task[:st.valid_total] >= 0) and st.T - st.valid_total < c


def test_rejects_bad_arguments():
    with pytest.raises(ValueError):
        segtab.build([[3]], 12)
    with pytest.raises(ValueError):
        segtab.build([[0]], 16)


def test_dispatch_oracle_hand_example_and_round_trip():
    """Dispatch places a task's packed tokens on its valid rows in order (pinned on the hand-laid table of the paper's
    alignment example: Task1's 8 tokens on rows 0-5, 8, 9, Task2's 3 tokens on rows 12-14, zeros elsewhere) and
    scatter is its inverse on the valid rows."""
    import json
    import os
    from oracle import dispatch
    g = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "segtab_hand_example.json")))
    st = segtab.build(g["tasks"], g["chunk"], g["max_pack_len"], 0)
    a = np.arange(1, 9, dtype=np.float64)[:, None] * np.array([[1.0, 10.0]])        # task 1: tokens 1..8
    b = -np.arange(1, 4, dtype=np.float64)[:, None] * np.array([[1.0, 10.0]])       # task 2: tokens -1..-3
    X = dispatch.gather([a, b], st.row_task, 2)
    want = np.zeros((16, 2))
    for tok, row in enumerate([0, 1, 2, 3, 4, 5, 8, 9]):
        want[row] = a[tok]
    for tok, row in enumerate([12, 13, 14]):
        want[row] = b[tok]
    assert np.array_equal(X, want)
    back = dispatch.scatter(X, st.row_task, 2)
    assert np.array_equal(back[0], a) and np.array_equal(back[1], b)
    # the dense table of the same example: same tokens, other rows
    sd = segtab.build(g["tasks"], g["chunk"], g["max_pack_len"], 1)
    Xd = dispatch.gather([a, b], sd.row_task, 2)
    assert np.array_equal(Xd[:8], a) and np.array_equal(Xd[8:11], b) and np.all(Xd[11] == 0)
    # a token keeps its place inside its sequence: the rows of a sequence are consecutive and in order
    for t, p, first, n in segtab.sequences(st):
        src = a if t == 0 else b
        off = sum(s[3] for s in segtab.sequences(st) if s[0] == t and s[2] < first)
        assert np.array_equal(X[first:first + n], src[off:off + n])
