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
