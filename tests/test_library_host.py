"""CPU-side checks of the library: it loads, exports every declared symbol, and its table
builder agrees with the oracle's byte for byte.  No compute call needs a GPU here."""
import ctypes
import os
import re

import numpy as np
import pytest

import mux_workloads as wlm
from oracle import segtab

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def mx():
    import paper_2603_02885_amd as m
    if not os.path.exists(m.library_path()):
        from paper_2603_02885_amd.build import build_library
        build_library()
    m.load_library()
    return m


def test_exports_every_declared_symbol(mx):
    hdr = "".join(open(os.path.join(ROOT, "include", f)).read() for f in sorted(os.listdir(os.path.join(ROOT, "include")))
                  if f.endswith(".h"))
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)          # declarations only, not prose
    names = set(re.findall(r"\b(mux_[a-z0-9_]+)\s*\(", hdr))
    assert {"mux_lora_forward", "mux_lora_backward", "mux_segtab_build", "mux_segtab_upload", "mux_plan_fusion"} <= names
    lib = ctypes.CDLL(mx.library_path())
    for n in sorted(names):
        assert hasattr(lib, n), n
    # the binding carries the same names
    for n in sorted(names):
        assert hasattr(mx, n), n


@pytest.mark.parametrize("idx", range(5))
@pytest.mark.parametrize("flags", [0, 1])
def test_benchmark_config_tables_bit_exact(mx, idx, flags):
    wl = wlm.config(idx)
    st = mx.mux_segtab_build([mx.TaskDesc(t.kind, t.rank, t.scale, t.seq_lens) for t in wl.tasks], wl.chunk, 0, flags)
    o = segtab.build([t.seq_lens for t in wl.tasks], wl.chunk, 0, flags)
    assert mx.mux_segtab_serialize(st).tobytes() == o.image.tobytes()
    assert np.array_equal(mx.mux_segtab_row_task(st), o.row_task)
    assert mx.mux_segtab_rows(st) == o.T and mx.mux_segtab_n_chunks(st) == o.n_chunks
    assert mx.mux_segtab_valid_tokens(st) == o.valid_total == wl.valid_tokens


def test_random_tables_bit_exact(mx):
    rng = np.random.default_rng(99)
    for case in range(1000):
        M = int(rng.integers(0, 9))
        tasks = [[int(v) for v in rng.integers(1, 70, size=int(rng.integers(0, 6)))] for _ in range(M)]
        c = int(2 ** rng.integers(0, 8))
        P = int(rng.choice([0, 0, 10, 64, 100]))
        flags = int(rng.integers(0, 2))
        st = mx.mux_segtab_build([mx.TaskDesc(1, 4, 1.0, t) for t in tasks], c, P, flags)
        o = segtab.build(tasks, c, P, flags)
        assert mx.mux_segtab_serialize(st).tobytes() == o.image.tobytes(), (case, tasks, c, P, flags)
        assert np.array_equal(mx.mux_segtab_row_task(st), o.row_task)


def test_table2_shapes(mx):
    """Workloads A/B of Table 2 as token-count shapes: chunk 64 leaves no padding for A."""
    for which, chunk in (("A", 64), ("B", 64), ("B", 128)):
        wl = wlm.table2_workload(which, chunk)
        st = mx.mux_segtab_build([mx.TaskDesc(t.kind, t.rank, t.scale, t.seq_lens) for t in wl.tasks], chunk)
        o = segtab.build([t.seq_lens for t in wl.tasks], chunk)
        assert mx.mux_segtab_serialize(st).tobytes() == o.image.tobytes()
        assert mx.mux_segtab_rows(st) == mx.mux_segtab_valid_tokens(st)


def test_chunk_size_rule(mx):
    for lens, floor in (([64, 128, 256], 64), ([96, 160], 64), ([96, 160], 16), ([512, 1024, 1536], 64), ([], 64),
                        ([7, 9], 1)):
        assert mx.mux_choose_chunk_size(lens, floor) == segtab.choose_chunk_size(lens, floor)


def test_argument_errors(mx):
    with pytest.raises(mx.MuxError) as e:
        mx.mux_segtab_build([mx.TaskDesc(1, 4, 1.0, [5])], 12)
    assert e.value.status == 1 and "power of two" in str(e.value)
    with pytest.raises(mx.MuxError):
        mx.mux_segtab_build([mx.TaskDesc(1, 0, 1.0, [5])], 16)          # LoRA rank 0
    with pytest.raises(mx.MuxError):
        mx.mux_segtab_build([mx.TaskDesc(1, 65, 1.0, [5])], 16)         # rank above the maximum
    with pytest.raises(mx.MuxError):
        mx.mux_segtab_build([mx.TaskDesc(7, 4, 1.0, [5])], 16)          # unknown kind
    with pytest.raises(mx.MuxError):
        mx.mux_segtab_build([mx.TaskDesc(1, 4, 1.0, [0])], 16)          # empty sequence
    st = mx.mux_segtab_build([mx.TaskDesc(1, 4, 1.0, [5])], 16)
    layer = mx.LayerDesc(8, 8, mx.MUX_DT_BF16, 0x1000, 2, [1, 1], [1, 1], None)   # 2 tasks vs table's 1
    with pytest.raises(mx.MuxError) as e:
        mx.mux_lora_forward(layer, st, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 1 << 30)
    assert e.value.status == 2
    layer = mx.LayerDesc(8, 8, mx.MUX_DT_BF16, 0x1000, 1, [None], [None], None)   # LoRA task without A/B
    with pytest.raises(mx.MuxError) as e:
        mx.mux_lora_forward(layer, st, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 1 << 30)
    assert e.value.status == 1
    layer = mx.LayerDesc(8, 8, mx.MUX_DT_BF16, 0x1000, 1, [0x1000], [0x1000], None)
    assert mx.mux_lora_workspace_bytes(layer, st) > 0
    with pytest.raises(mx.MuxError) as e:                                          # workspace too small
        mx.mux_lora_forward(layer, st, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 8)
    assert e.value.status == 4


def test_empty_table(mx):
    st = mx.mux_segtab_build([], 64)
    assert mx.mux_segtab_rows(st) == 0 and mx.mux_segtab_n_chunks(st) == 0
    st = mx.mux_segtab_build([mx.TaskDesc(1, 8, 1.0, [])], 64)
    assert mx.mux_segtab_rows(st) == 0
    o = segtab.build([[]], 64)
    assert mx.mux_segtab_serialize(st).tobytes() == o.image.tobytes()


def test_sparse_mask_layout_against_a_direct_listing(mx):
    """mux_sparse_mask_layout and mux_sparse_mask_tile_layout against the listings written down directly from the
    entries (pure Python), on random masks with empty rows and columns, and shapes with several buckets of 64 x 128 and
    ragged last ones; unsorted, duplicated and out-of-range entries are refused."""
    import ctypes
    rng = np.random.default_rng(5)

    class Keep:
        def __init__(self, a):
            self.a = a

        def data_ptr(self):
            return self.a.ctypes.data

    for K, N, dens in ((7, 5, 0.4), (33, 64, 0.05), (16, 9, 0.0), (5, 300, 0.3), (200, 300, 0.02), (130, 129, 0.1)):
        flat = np.flatnonzero(rng.random(K * N) < dens)
        k, n = (flat // N).astype(np.int32), (flat % N).astype(np.int32)
        held = []
        m = mx.SparseMask(k, n, K, N, lambda a: held.append(Keep(a.copy())) or held[-1])
        row_ptr, col_idx, col_ptr, col_ent, fwd_ptr, fwd_ent, bwd_ptr, bwd_ent = (h.a for h in held)
        assert m.nnz == flat.size
        by_row = [[int(n[e]) for e in range(flat.size) if k[e] == r] for r in range(K)]
        assert list(row_ptr) == [sum(len(x) for x in by_row[:r]) for r in range(K + 1)]
        assert list(col_idx[:flat.size]) == [c for x in by_row for c in x]
        by_col = [[(int(k[e]), e) for e in range(flat.size) if n[e] == c] for c in range(N)]
        assert list(col_ptr) == [sum(len(x) for x in by_col[:c]) for c in range(N + 1)]
        assert list(col_ent[:2 * flat.size]) == [v for x in by_col for pair in x for v in pair]
        # by tiles: forward buckets (k / 64, n / 128), backward buckets (n / 64, k / 128), (k, n) order inside a bucket
        nbn, nbk = (N + 127) // 128, (K + 127) // 128
        fwd = [[] for _ in range(((K + 63) // 64) * nbn)]
        bwd = [[] for _ in range(((N + 63) // 64) * nbk)]
        for e in range(flat.size):
            fwd[(k[e] // 64) * nbn + n[e] // 128] += [e, (int(k[e]) % 64) << 7 | int(n[e]) % 128]
            bwd[(n[e] // 64) * nbk + k[e] // 128] += [e, (int(n[e]) % 64) << 7 | int(k[e]) % 128]
        assert list(fwd_ptr) == [sum(len(x) // 2 for x in fwd[:b]) for b in range(len(fwd) + 1)]
        assert list(bwd_ptr) == [sum(len(x) // 2 for x in bwd[:b]) for b in range(len(bwd) + 1)]
        assert list(fwd_ent[:2 * flat.size]) == [v for x in fwd for v in x]
        assert list(bwd_ent[:2 * flat.size]) == [v for x in bwd for v in x]
    for k, n in (([1, 0], [0, 0]), ([0, 0], [2, 2]), ([0], [9]), ([-1], [0])):
        with pytest.raises(mx.MuxError):
            mx.SparseMask(np.array(k), np.array(n), 4, 4, lambda a: Keep(a))
