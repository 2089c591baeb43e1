"""Pins of the fp64 oracle against what the paper and the mathematics fix.

Each test names the mistake it would catch.  None of them retypes the oracle's own loops:
they compare with numpy's float64 matmul on special cases, with the merged-weight closed
form (which goes through the dense X^T dY the method itself never forms), with exact
finite differences of a loss that is linear in each argument, with hand-worked numbers,
and with the isolation properties of section 3.2.
"""
import json
import os

import numpy as np
import pytest

import mux_workloads as wlm
import oracle
from oracle import segtab

RNG = np.random.default_rng(1234)


def small_problem(seed=0, K=24, N=20, c=4, bf16=True, with_ia3=True, with_none=True):
    """Three or four tasks with uneven token counts, ragged padding."""
    tasks = [wlm.Task(wlm.KIND_LORA, 3, 2.0, [5, 2]),
             wlm.Task(wlm.KIND_LORA, 5, 0.5, [6])]
    if with_ia3:
        tasks.append(wlm.Task(wlm.KIND_IA3, 0, 1.0, [3, 3]))
    if with_none:
        tasks.append(wlm.Task(wlm.KIND_NONE, 0, 1.0, [2]))
    wl = wlm.Workload(name=f"small{seed}", layers=[("w", K, N)], tasks=tasks, chunk=c,
                      sigma_w=0.5, sigma_ab=0.5)
    st = segtab.build([t.seq_lens for t in tasks], c)
    lt = wlm.layer_tensors(wl, 0, st.T, seed=seed, bf16=bf16)
    return wl, st, lt


def run_fwd(wl, st, lt, **kw):
    return oracle.forward(lt.X, lt.W, st.row_task, [t.kind for t in wl.tasks],
                          [t.rank for t in wl.tasks], [t.scale for t in wl.tasks],
                          lt.A, lt.B, lt.L, **kw)


def run_bwd(wl, st, lt, **kw):
    return oracle.backward(lt.X, lt.dY, lt.W, st.row_task, [t.kind for t in wl.tasks],
                           [t.rank for t in wl.tasks], [t.scale for t in wl.tasks],
                           lt.A, lt.B, lt.L, **kw)


def masked(a, row_task):
    a = np.array(a, dtype=np.float64)
    a[row_task < 0] = 0.0
    return a


# ----------------------------------------------------------------- hand-worked numbers

def test_hand_worked_example(golden_dir):
    """A wrong sign, a dropped scale, a transposed A/B or W, or a leaking pad row changes
    at least one of these pencil-computed values."""
    g = json.load(open(os.path.join(golden_dir, "layer_hand_example.json")))
    tk = g["tasks"]
    A = [np.array(t["A"], dtype=np.float32) if "A" in t else None for t in tk]
    B = [np.array(t["B"], dtype=np.float32) if "B" in t else None for t in tk]
    L = [np.array(t["L"], dtype=np.float32) if "L" in t else None for t in tk]
    args = (np.array(g["row_task"]), [t["kind"] for t in tk], [t["rank"] for t in tk],
            [t["scale"] for t in tk], A, B, L)
    X = np.array(g["X"], dtype=np.float32)
    W = np.array(g["W"], dtype=np.float32)
    dY = np.array(g["dY"], dtype=np.float32)
    f = oracle.forward(X, W, *args)
    b = oracle.backward(X, dY, W, *args)
    e = g["expect"]
    assert np.array_equal(f["Y"], np.array(e["Y"], dtype=np.float64))
    assert np.array_equal(f["H"], np.array(e["H"], dtype=np.float64))
    assert np.array_equal(b["dX"], np.array(e["dX"], dtype=np.float64))
    assert np.array_equal(b["G"], np.array(e["G"], dtype=np.float64))
    assert np.array_equal(b["dA"][0], np.array(e["dA0"], dtype=np.float64))
    assert np.array_equal(b["dB"][0], np.array(e["dB0"], dtype=np.float64))
    assert np.array_equal(b["dL"][1], np.array(e["dL1"], dtype=np.float64))


# ----------------------------------------------------------------- special cases -> library matmul

def test_zero_B_reduces_to_backbone_gemm():
    """B_t = 0: Y is the plain GEMM of Eq. 1, dX the plain GEMM of Eq. 2, dA_t = 0 exactly."""
    wl, st, lt = small_problem(with_ia3=False)
    lt.B = [None if b is None else np.zeros_like(b) for b in lt.B]
    f = run_fwd(wl, st, lt)
    b = run_bwd(wl, st, lt)
    Xm = masked(lt.X, st.row_task)
    Gm = masked(lt.dY, st.row_task)
    W = lt.W.astype(np.float64)
    np.testing.assert_allclose(f["Y"], Xm @ W, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(b["dX"], Gm @ W.T, rtol=1e-13, atol=1e-13)
    for t, task in enumerate(wl.tasks):
        if task.kind == wlm.KIND_LORA:
            assert np.all(b["dA"][t] == 0.0)
            assert np.any(b["dB"][t] != 0.0)


def test_zero_A_gives_zero_dB_and_plain_output():
    wl, st, lt = small_problem(with_ia3=False)
    lt.A = [None if a is None else np.zeros_like(a) for a in lt.A]
    f = run_fwd(wl, st, lt)
    b = run_bwd(wl, st, lt)
    W = lt.W.astype(np.float64)
    np.testing.assert_allclose(f["Y"], masked(lt.X, st.row_task) @ W, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(b["dX"], masked(lt.dY, st.row_task) @ W.T, rtol=1e-13, atol=1e-13)
    for t, task in enumerate(wl.tasks):
        if task.kind == wlm.KIND_LORA:
            assert np.all(b["dB"][t] == 0.0)
            assert np.any(b["dA"][t] != 0.0)


def test_unit_ia3_vector_is_plain_gemm():
    wl, st, lt = small_problem()
    lt.L = [None if l is None else np.ones_like(l) for l in lt.L]
    f = run_fwd(wl, st, lt)
    b = run_bwd(wl, st, lt)
    W = lt.W.astype(np.float64)
    rows = st.task_rows[2]
    np.testing.assert_allclose(f["Y"][rows], lt.X[rows].astype(np.float64) @ W, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(b["dX"][rows], lt.dY[rows].astype(np.float64) @ W.T, rtol=1e-13, atol=1e-13)


# ----------------------------------------------------------------- closed form through merged weights

@pytest.mark.parametrize("seed", [0, 1])
def test_merged_weight_closed_form(seed):
    """LoRA is a low-rank reparameterisation of the weight (section 2.1): per task,
    Y_t = X_t (W + s A B), dX_t = dY_t (W + s A B)^T, and with D = X_t^T dY_t (the dense
    weight gradient the method avoids) dA = s D B^T, dB = s A^T D.  For the output-scale
    kind: Y = X (W diag l), dX = dY (W diag l)^T, dl = diag(W^T D)."""
    wl, st, lt = small_problem(seed=seed)
    f = run_fwd(wl, st, lt, want_z=True)
    b = run_bwd(wl, st, lt)
    W = lt.W.astype(np.float64)
    for t, task in enumerate(wl.tasks):
        rows = st.task_rows[t]
        Xt = lt.X[rows].astype(np.float64)
        Gt = lt.dY[rows].astype(np.float64)
        D = Xt.T @ Gt
        if task.kind == wlm.KIND_LORA:
            A = lt.A[t].astype(np.float64); B = lt.B[t].astype(np.float64)
            Weff = W + task.scale * (A @ B)
            np.testing.assert_allclose(b["dA"][t], task.scale * D @ B.T, rtol=1e-11, atol=1e-11)
            np.testing.assert_allclose(b["dB"][t], task.scale * A.T @ D, rtol=1e-11, atol=1e-11)
            np.testing.assert_allclose(f["H"][rows][:, :task.rank], Xt @ A, rtol=1e-12, atol=1e-12)
            np.testing.assert_allclose(b["G"][rows][:, :task.rank], Gt @ B.T, rtol=1e-12, atol=1e-12)
        elif task.kind == wlm.KIND_IA3:
            l = lt.L[t].astype(np.float64)
            Weff = W * l[None, :]
            np.testing.assert_allclose(b["dL"][t], np.einsum("kn,kn->n", W, D), rtol=1e-11, atol=1e-11)
            np.testing.assert_allclose(f["Z"][rows], Xt @ W, rtol=1e-12, atol=1e-12)
        else:
            Weff = W
        np.testing.assert_allclose(f["Y"][rows], Xt @ Weff, rtol=1e-11, atol=1e-11)
        np.testing.assert_allclose(b["dX"][rows], Gt @ Weff.T, rtol=1e-11, atol=1e-11)
    pad = st.row_task < 0
    assert pad.any()
    assert np.all(f["Y"][pad] == 0) and np.all(b["dX"][pad] == 0)
    assert np.all(f["H"][pad] == 0) and np.all(b["G"][pad] == 0)


def test_config1_against_numpy():
    """Benchmark config 1 in full against numpy float64 (library routine), both table modes."""
    wl = wlm.config(0)
    for flags in (0, segtab.FLAG_DENSE):
        st = segtab.build([t.seq_lens for t in wl.tasks], wl.chunk, 0, flags)
        assert st.n_chunks == (5 if flags == 0 else 4)
        lt = wlm.layer_tensors(wl, 0, st.T, seed=0)
        f = run_fwd(wl, st, lt)
        b = run_bwd(wl, st, lt)
        W = lt.W.astype(np.float64)
        for t, task in enumerate(wl.tasks):
            rows = st.task_rows[t]
            assert len(rows) == task.tokens
            Xt = lt.X[rows].astype(np.float64); Gt = lt.dY[rows].astype(np.float64)
            A = lt.A[t].astype(np.float64); B = lt.B[t].astype(np.float64)
            np.testing.assert_allclose(f["Y"][rows], Xt @ W + task.scale * (Xt @ A) @ B, rtol=1e-11, atol=1e-12)
            np.testing.assert_allclose(b["dX"][rows], Gt @ W.T + task.scale * (Gt @ B.T) @ A.T, rtol=1e-11, atol=1e-12)
            np.testing.assert_allclose(b["dA"][t], task.scale * Xt.T @ (Gt @ B.T), rtol=1e-11, atol=1e-12)
            np.testing.assert_allclose(b["dB"][t], task.scale * (Xt @ A).T @ Gt, rtol=1e-11, atol=1e-12)


# ----------------------------------------------------------------- exact finite differences

def _loss(wl, st, lt):
    f = run_fwd(wl, st, lt)
    return float(np.sum(f["Y"] * masked(lt.dY, st.row_task)))


def test_finite_differences_are_exact():
    """With L = sum(Y * dY), L is linear in each of X, A_t, B_t, l_t taken alone, so a
    central difference has no truncation error; fp32 storage of the perturbed entry is kept
    exact by choosing power-of-two values and steps."""
    wl, st, lt = small_problem(seed=3, bf16=True)
    b = run_bwd(wl, st, lt)
    eps = 2.0 ** -6
    rng = np.random.default_rng(7)

    def fd(arr, idx):
        old = arr[idx]
        arr[idx] = np.float32(old + eps); lp = _loss(wl, st, lt)
        arr[idx] = np.float32(old - eps); lm = _loss(wl, st, lt)
        arr[idx] = old
        return (lp - lm) / (2 * eps)

    # X (valid rows) and pad rows (gradient must be zero and value ignored)
    for _ in range(12):
        i = int(rng.integers(0, st.T)); k = int(rng.integers(0, lt.K))
        g = fd(lt.X, (i, k))
        assert abs(g - b["dX"][i, k]) <= 1e-9 * max(1.0, abs(g))
        if st.row_task[i] < 0:
            assert g == 0.0
    for t, task in enumerate(wl.tasks):
        if task.kind == wlm.KIND_LORA:
            for _ in range(6):
                k = int(rng.integers(0, lt.K)); j = int(rng.integers(0, task.rank)); n = int(rng.integers(0, lt.N))
                g = fd(lt.A[t], (k, j))
                assert abs(g - b["dA"][t][k, j]) <= 1e-9 * max(1.0, abs(g))
                g = fd(lt.B[t], (j, n))
                assert abs(g - b["dB"][t][j, n]) <= 1e-9 * max(1.0, abs(g))
        elif task.kind == wlm.KIND_IA3:
            for n in range(0, lt.N, 3):
                g = fd(lt.L[t], (n,))
                assert abs(g - b["dL"][t][n]) <= 1e-9 * max(1.0, abs(g))


# ----------------------------------------------------------------- isolation (section 3.2)

def test_task_alone_equals_its_rows_in_the_multiplexed_run():
    """Eq. 1 / Eq. 2: the batched result restricted to a task's rows is that task run alone
    (bitwise here: same per-row code, same order)."""
    wl, st, lt = small_problem(seed=5)
    f = run_fwd(wl, st, lt); b = run_bwd(wl, st, lt)
    for t, task in enumerate(wl.tasks):
        rows = st.task_rows[t]
        alone_rt = np.zeros(len(rows), dtype=np.int32)
        fa = oracle.forward(lt.X[rows], lt.W, alone_rt, [task.kind], [task.rank], [task.scale],
                            [lt.A[t]], [lt.B[t]], [lt.L[t]])
        ba = oracle.backward(lt.X[rows], lt.dY[rows], lt.W, alone_rt, [task.kind], [task.rank],
                             [task.scale], [lt.A[t]], [lt.B[t]], [lt.L[t]])
        assert np.array_equal(fa["Y"], f["Y"][rows])
        assert np.array_equal(ba["dX"], b["dX"][rows])
        for name in ("dA", "dB", "dL"):
            if b[name][t] is not None:
                assert np.array_equal(ba[name][0], b[name][t])


def test_task_permutation_only_permutes():
    wl, st, lt = small_problem(seed=6)
    f = run_fwd(wl, st, lt); b = run_bwd(wl, st, lt)
    perm = [2, 0, 3, 1]
    tasks2 = [wl.tasks[p] for p in perm]
    st2 = segtab.build([t.seq_lens for t in tasks2], wl.chunk)
    X2 = np.zeros((st2.T, lt.K), dtype=np.float32); dY2 = np.zeros((st2.T, lt.N), dtype=np.float32)
    for new, old in enumerate(perm):
        X2[st2.task_rows[new]] = lt.X[st.task_rows[old]]
        dY2[st2.task_rows[new]] = lt.dY[st.task_rows[old]]
    args = ([t.kind for t in tasks2], [t.rank for t in tasks2], [t.scale for t in tasks2],
            [lt.A[p] for p in perm], [lt.B[p] for p in perm], [lt.L[p] for p in perm])
    f2 = oracle.forward(X2, lt.W, st2.row_task, *args)
    b2 = oracle.backward(X2, dY2, lt.W, st2.row_task, *args)
    for new, old in enumerate(perm):
        assert np.array_equal(f2["Y"][st2.task_rows[new]], f["Y"][st.task_rows[old]])
        assert np.array_equal(b2["dX"][st2.task_rows[new]], b["dX"][st.task_rows[old]])
        for name in ("dA", "dB", "dL"):
            if b[name][old] is not None:
                assert np.array_equal(b2[name][new], b[name][old])


def test_other_tasks_data_and_nan_do_not_leak():
    """Changing or poisoning task j's data, adapters and the padding rows leaves every other
    task's outputs and gradients bit-identical and finite (section 3.2: numerical failures of
    one task do not propagate)."""
    wl, st, lt = small_problem(seed=8)
    f = run_fwd(wl, st, lt); b = run_bwd(wl, st, lt)
    j = 1
    lt2 = wlm.layer_tensors(wl, 0, st.T, seed=8)
    rows_j = st.task_rows[j]
    lt2.X[rows_j] = np.nan
    lt2.dY[rows_j] = np.inf
    lt2.A[j][:] = np.nan
    lt2.B[j][:] = np.nan
    pad = st.row_task < 0
    lt2.X[pad] = np.nan
    lt2.dY[pad] = 1e30
    f2 = run_fwd(wl, st, lt2); b2 = run_bwd(wl, st, lt2)
    for t in range(len(wl.tasks)):
        if t == j:
            continue
        rows = st.task_rows[t]
        assert np.array_equal(f2["Y"][rows], f["Y"][rows]) and np.isfinite(f2["Y"][rows]).all()
        assert np.array_equal(b2["dX"][rows], b["dX"][rows])
        for name in ("dA", "dB", "dL"):
            if b[name][t] is not None:
                assert np.array_equal(b2[name][t], b[name][t])
                assert np.isfinite(b2[name][t]).all()
    assert np.all(f2["Y"][pad] == 0) and np.all(b2["dX"][pad] == 0)


def test_column_sampling_matches_full():
    wl, st, lt = small_problem(seed=9)
    f = run_fwd(wl, st, lt); b = run_bwd(wl, st, lt)
    cols = np.array([1, 7, 19, 4], dtype=np.int32)
    kcols = np.array([0, 23, 5], dtype=np.int32)
    fs = run_fwd(wl, st, lt, cols=cols)
    bs = run_bwd(wl, st, lt, cols=cols, kcols=kcols)
    assert np.array_equal(fs["Y"], f["Y"][:, cols])
    assert np.array_equal(bs["dX"], b["dX"][:, kcols])
    assert np.array_equal(bs["dL"][2], b["dL"][2][cols])
    assert np.array_equal(bs["dA"][0], b["dA"][0]) and np.array_equal(bs["dB"][1], b["dB"][1])


def test_thread_count_does_not_change_results():
    import subprocess, sys, textwrap
    code = textwrap.dedent("""
        import sys, numpy as np
        sys.path.insert(0, %r)
        from tests.test_oracle_pins import small_problem, run_fwd, run_bwd
        wl, st, lt = small_problem(seed=11)
        f = run_fwd(wl, st, lt); b = run_bwd(wl, st, lt)
        import hashlib
        h = hashlib.sha256()
        for a in [f['Y'], b['dX'], b['dA'][0], b['dB'][1], b['dL'][2]]:
            h.update(a.tobytes())
        print(h.hexdigest())
    """) % os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    outs = []
    for n in ("1", "5"):
        env = dict(os.environ, OMP_NUM_THREADS=n)
        outs.append(subprocess.check_output([sys.executable, "-c", code], env=env).strip())
    assert outs[0] == outs[1]


# ----------------------------------------------------------------- additive bottleneck kind

def adapter_problem(seed=0, K=12, N=10, c=4, bf16=True):
    """One additive-bottleneck task between a LoRA task and a plain one, ragged padding."""
    tasks = [wlm.Task(wlm.KIND_LORA, 3, 2.0, [5]),
             wlm.Task(wlm.KIND_ADAPTER, 4, 1.5, [6, 3]),
             wlm.Task(wlm.KIND_NONE, 0, 1.0, [2]),
             wlm.Task(wlm.KIND_ADAPTER, 2, 0.5, [5])]
    wl = wlm.Workload(name=f"adp{seed}", layers=[("w", K, N)], tasks=tasks, chunk=c, sigma_w=0.5, sigma_ab=0.5)
    st = segtab.build([t.seq_lens for t in tasks], c)
    lt = wlm.layer_tensors(wl, 0, st.T, seed=seed, bf16=bf16)
    return wl, st, lt


def test_adapter_hand_worked_row():
    """One token, K = 2, N = 2, r = 1, numbers a pencil can follow: z = x W = (1, 2);
    u = z D = 1*0.5 + 2*0.25 = 1; gelu(1) = (1 + erf(1/sqrt 2))/2 = Phi(1), the standard normal cdf at 1
    (0.8413447460685429, a tabulated constant); y = z + s gelu(u) U = (1 + 2*Phi(1)*1, 2 + 2*Phi(1)*(-1)).
    Backward with g = (1, 1): g U^T = 0, so p = 0, dX = g W^T = (1*1 + 1*0, 1*0 + 1*2) = (1, 2),
    dD = 0, dU = s gelu(u) g = (2 Phi(1), 2 Phi(1)).  A wrong aggregate, a dropped scale, D and U exchanged
    or a transposed W changes one of these."""
    phi1 = 0.8413447460685429
    X = np.array([[1.0, 1.0]], dtype=np.float32)
    W = np.array([[1.0, 0.0], [0.0, 2.0]], dtype=np.float32)
    D = np.array([[0.5], [0.25]], dtype=np.float32)
    U = np.array([[1.0, -1.0]], dtype=np.float32)
    dY = np.array([[1.0, 1.0]], dtype=np.float32)
    rt = np.array([0], dtype=np.int32)
    f = oracle.forward(X, W, rt, [wlm.KIND_ADAPTER], [1], [2.0], [D], [U], [None])
    assert np.allclose(f["Y"], [[1 + 2 * phi1, 2 - 2 * phi1]], rtol=0, atol=1e-15)
    assert np.allclose(f["H"], [[1.0]], rtol=0, atol=0)
    b = oracle.backward(X, dY, W, rt, [wlm.KIND_ADAPTER], [1], [2.0], [D], [U], [None])
    assert np.allclose(b["dX"], [[1.0, 2.0]], rtol=0, atol=1e-15)
    assert np.allclose(b["dA"][0], [[0.0], [0.0]], rtol=0, atol=1e-15)
    assert np.allclose(b["dB"][0], [[2 * phi1, 2 * phi1]], rtol=0, atol=1e-15)
    # second output gradient, g = (1, 0): g U^T = 1, p = s * 1 * gelu'(1), gelu'(1) = Phi(1) + pdf(1),
    # pdf(1) = exp(-1/2)/sqrt(2 pi) = 0.24197072451914337; dz = g + p D^T; dX = dz W^T = (dz0, 2 dz1); dD = z^T p
    gp = phi1 + 0.24197072451914337
    dY2 = np.array([[1.0, 0.0]], dtype=np.float32)
    b = oracle.backward(X, dY2, W, rt, [wlm.KIND_ADAPTER], [1], [2.0], [D], [U], [None])
    p = 2.0 * gp
    assert np.allclose(b["G"], [[p]], rtol=1e-15, atol=0)
    assert np.allclose(b["dX"], [[1 + p * 0.5, 2 * (p * 0.25)]], rtol=1e-15, atol=0)
    assert np.allclose(b["dA"][0], [[1 * p], [2 * p]], rtol=1e-15, atol=0)
    assert np.allclose(b["dB"][0], [[2 * phi1, 0.0]], rtol=1e-15, atol=0)


def test_adapter_zero_up_projection_is_plain_gemm():
    """U = 0: the bottleneck adds nothing, Y = X W, dX = dY W^T, dD = 0 (numpy matmul as the routine)."""
    wl, st, lt = adapter_problem(seed=1)
    for t, task in enumerate(wl.tasks):
        if task.kind == wlm.KIND_ADAPTER:
            lt.B[t][:] = 0
    f = run_fwd(wl, st, lt); b = run_bwd(wl, st, lt)
    X64, W64, g64 = lt.X.astype(np.float64), lt.W.astype(np.float64), lt.dY.astype(np.float64)
    for t, task in enumerate(wl.tasks):
        if task.kind != wlm.KIND_ADAPTER:
            continue
        rows = st.row_task == t
        assert np.allclose(f["Y"][rows], X64[rows] @ W64, rtol=1e-13, atol=1e-13)
        assert np.allclose(b["dX"][rows], g64[rows] @ W64.T, rtol=1e-13, atol=1e-13)
        assert np.all(b["dA"][t] == 0)


def test_adapter_zero_down_projection():
    """D = 0: u = 0, gelu(0) = 0, so Y = X W and dU = 0; gelu'(0) = 1/2, so p = s/2 g U^T,
    dD = (X W)^T p and dX = dY W^T (p D^T vanishes) -- all through numpy matmul."""
    wl, st, lt = adapter_problem(seed=2)
    for t, task in enumerate(wl.tasks):
        if task.kind == wlm.KIND_ADAPTER:
            lt.A[t][:] = 0
    f = run_fwd(wl, st, lt); b = run_bwd(wl, st, lt)
    X64, W64, g64 = lt.X.astype(np.float64), lt.W.astype(np.float64), lt.dY.astype(np.float64)
    for t, task in enumerate(wl.tasks):
        if task.kind != wlm.KIND_ADAPTER:
            continue
        rows = st.row_task == t
        z = X64[rows] @ W64
        assert np.allclose(f["Y"][rows], z, rtol=1e-13, atol=1e-13)
        assert np.all(b["dB"][t] == 0)
        p = 0.5 * task.scale * (g64[rows] @ lt.B[t].astype(np.float64).T)
        assert np.allclose(b["dA"][t], z.T @ p, rtol=1e-12, atol=1e-12)
        assert np.allclose(b["dX"][rows], g64[rows] @ W64.T, rtol=1e-13, atol=1e-13)


def test_adapter_large_preactivation_is_linear():
    """For u >> 0, gelu(u) = u to double precision: the bottleneck becomes the linear low-rank
    update z -> z + s (z D) U, i.e. Y = X W (I + s D U) -- the merged closed form through numpy."""
    K, N, r = 6, 5, 2
    rng = np.random.default_rng(5)
    X = np.abs(rng.standard_normal((7, K))).astype(np.float32) + 1
    W = np.abs(rng.standard_normal((K, N))).astype(np.float32) + 1
    D = (np.abs(rng.standard_normal((N, r))) * 4 + 4).astype(np.float32)      # u in the hundreds
    U = rng.standard_normal((r, N)).astype(np.float32)
    dY = rng.standard_normal((7, N)).astype(np.float32)
    rt = np.zeros(7, dtype=np.int32)
    f = oracle.forward(X, W, rt, [wlm.KIND_ADAPTER], [r], [0.75], [D], [U], [None])
    b = oracle.backward(X, dY, W, rt, [wlm.KIND_ADAPTER], [r], [0.75], [D], [U], [None])
    M = np.eye(N) + 0.75 * D.astype(np.float64) @ U.astype(np.float64)
    Wm = W.astype(np.float64) @ M
    assert np.min(f["H"]) > 40
    assert np.allclose(f["Y"], X.astype(np.float64) @ Wm, rtol=1e-13, atol=0)
    assert np.allclose(b["dX"], dY.astype(np.float64) @ Wm.T, rtol=1e-13, atol=0)
    z = X.astype(np.float64) @ W.astype(np.float64)
    assert np.allclose(b["dB"][0], 0.75 * (z @ D.astype(np.float64)).T @ dY.astype(np.float64), rtol=1e-13, atol=0)
    assert np.allclose(b["dA"][0], 0.75 * z.T @ (dY.astype(np.float64) @ U.astype(np.float64).T), rtol=1e-13, atol=0)


def test_adapter_finite_differences():
    """L = sum(Y * dY) is linear in U (exact central difference) and smooth in X and D:
    a central difference with step h has error O(h^2) and must agree to 1e-6 relative."""
    wl, st, lt = adapter_problem(seed=3, bf16=False)
    b = run_bwd(wl, st, lt)
    rng = np.random.default_rng(11)
    h = 2.0 ** -9

    def fd(arr, idx, step):
        old = arr[idx]
        arr[idx] = np.float32(old + step); lp = _loss(wl, st, lt)
        arr[idx] = np.float32(old - step); lm = _loss(wl, st, lt)
        hp = float(np.float32(old + step)) - float(np.float32(old - step))
        arr[idx] = old
        return (lp - lm) / hp

    for t, task in enumerate(wl.tasks):
        if task.kind != wlm.KIND_ADAPTER:
            continue
        rows = np.nonzero(st.row_task == t)[0]
        for _ in range(6):
            i = int(rng.choice(rows)); k = int(rng.integers(0, lt.K))
            g = fd(lt.X, (i, k), h)
            assert abs(g - b["dX"][i, k]) <= 2e-5 * max(1.0, abs(g)), (g, b["dX"][i, k])
            n = int(rng.integers(0, lt.N)); j = int(rng.integers(0, task.rank))
            g = fd(lt.A[t], (n, j), h)
            assert abs(g - b["dA"][t][n, j]) <= 2e-5 * max(1.0, abs(g)), (g, b["dA"][t][n, j])
            g = fd(lt.B[t], (j, n), 2.0 ** -6)
            assert abs(g - b["dB"][t][j, n]) <= 1e-9 * max(1.0, abs(g))


def test_adapter_isolation_and_padding():
    """The additive task alone gives bit-identical rows and gradients; NaN in other tasks' rows and in
    padding rows changes nothing (section 3.2)."""
    wl, st, lt = adapter_problem(seed=4)
    f = run_fwd(wl, st, lt); b = run_bwd(wl, st, lt)
    t = 1
    rows = st.row_task == t
    rt = np.where(rows, 0, -1).astype(np.int32)
    f1 = oracle.forward(lt.X, lt.W, rt, [wl.tasks[t].kind], [wl.tasks[t].rank], [wl.tasks[t].scale], [lt.A[t]], [lt.B[t]], [None])
    b1 = oracle.backward(lt.X, lt.dY, lt.W, rt, [wl.tasks[t].kind], [wl.tasks[t].rank], [wl.tasks[t].scale], [lt.A[t]], [lt.B[t]], [None])
    assert np.array_equal(f1["Y"][rows], f["Y"][rows]) and np.array_equal(b1["dX"][rows], b["dX"][rows])
    assert np.array_equal(b1["dA"][0], b["dA"][t]) and np.array_equal(b1["dB"][0], b["dB"][t])
    lt2 = wlm.layer_tensors(wl, 0, st.T, seed=4)
    lt2.X[~rows] = np.nan; lt2.dY[~rows] = np.nan
    f2 = run_fwd(wl, st, lt2); b2 = run_bwd(wl, st, lt2)
    assert np.array_equal(f2["Y"][rows], f["Y"][rows]) and np.array_equal(b2["dX"][rows], b["dX"][rows])
    assert np.array_equal(b2["dA"][t], b["dA"][t]) and np.array_equal(b2["dB"][t], b["dB"][t])
    pad = st.row_task < 0
    assert np.all(f2["Y"][pad] == 0) and np.all(b2["dX"][pad] == 0)


# ----------------------------------------------------------------- selective kind (masked sparse update of W)

def diff_problem(seed=0, K=14, N=11, c=4, bf16=True, density=0.2):
    tasks = [wlm.Task(wlm.KIND_LORA, 3, 2.0, [5]),
             wlm.Task(wlm.KIND_DIFF, 0, 1.0, [6, 3], density=density),
             wlm.Task(wlm.KIND_NONE, 0, 1.0, [2]),
             wlm.Task(wlm.KIND_DIFF, 0, 1.0, [5], density=density / 2)]
    wl = wlm.Workload(name=f"diff{seed}", layers=[("w", K, N)], tasks=tasks, chunk=c, sigma_w=0.5, sigma_ab=0.5)
    st = segtab.build([t.seq_lens for t in tasks], c)
    lt = wlm.layer_tensors(wl, 0, st.T, seed=seed, bf16=bf16)
    return wl, st, lt


def _kw(lt):
    return {"S": lt.masks}


def test_diff_hand_worked_row():
    """x = (1, 2, 3), W = [[1,0],[0,1],[1,1]], mask entries (0,1) and (2,0) with values 10 and -1:
    W' = [[1,10],[0,1],[0,1]], y = x W' = (1, 10 + 2 + 3) = (1, 15).  With g = (1, 2): dX = g W'^T = (21, 2, 2);
    d delta = (x_0 g_1, x_2 g_0) = (2, 3).  A transposed mask index or an unmasked gradient entry changes these."""
    X = np.array([[1.0, 2.0, 3.0]], dtype=np.float32)
    W = np.array([[1.0, 0.0], [0.0, 1.0], [1.0, 1.0]], dtype=np.float32)
    k = np.array([0, 2], dtype=np.int32); n = np.array([1, 0], dtype=np.int32)
    v = np.array([10.0, -1.0], dtype=np.float32)
    dY = np.array([[1.0, 2.0]], dtype=np.float32)
    rt = np.array([0], dtype=np.int32)
    f = oracle.forward(X, W, rt, [wlm.KIND_DIFF], [0], [1.0], [v], [None], [None], S=[(k, n)])
    assert np.array_equal(f["Y"], [[1.0, 15.0]])
    b = oracle.backward(X, dY, W, rt, [wlm.KIND_DIFF], [0], [1.0], [v], [None], [None], S=[(k, n)])
    assert np.array_equal(b["dX"], [[21.0, 2.0, 2.0]])
    assert np.array_equal(b["dA"][0], [2.0, 3.0])


@pytest.mark.parametrize("seed", [0, 1])
def test_diff_against_dense_weights(seed):
    """The definition through dense matrices and numpy: W_t = W + scatter(mask, delta), Y = X W_t, dX = dY W_t^T,
    and the gradient is the masked slice of the dense X^T dY -- the weight gradient the rest of the method never forms."""
    wl, st, lt = diff_problem(seed=seed)
    f = run_fwd(wl, st, lt, **_kw(lt)); b = run_bwd(wl, st, lt, **_kw(lt))
    X64, W64, g64 = lt.X.astype(np.float64), lt.W.astype(np.float64), lt.dY.astype(np.float64)
    for t, task in enumerate(wl.tasks):
        if task.kind != wlm.KIND_DIFF:
            continue
        rows = st.row_task == t
        k, n = lt.masks[t]
        assert k.size > 0 and np.all(np.diff(k.astype(np.int64) * lt.N + n) > 0)      # sorted by (k, n), no duplicates
        Wt = W64.copy(); Wt[k, n] += lt.A[t].astype(np.float64)
        assert np.allclose(f["Y"][rows], X64[rows] @ Wt, rtol=1e-13, atol=1e-13)
        assert np.allclose(b["dX"][rows], g64[rows] @ Wt.T, rtol=1e-13, atol=1e-13)
        dense = X64[rows].T @ g64[rows]
        assert np.allclose(b["dA"][t], dense[k, n], rtol=1e-13, atol=1e-13)


def test_diff_empty_mask_is_plain_gemm():
    wl, st, lt = diff_problem(seed=2, density=0.0)
    f = run_fwd(wl, st, lt, **_kw(lt)); b = run_bwd(wl, st, lt, **_kw(lt))
    rows = st.row_task == 1
    assert lt.masks[1][0].size == 0
    assert np.allclose(f["Y"][rows], lt.X[rows].astype(np.float64) @ lt.W.astype(np.float64), rtol=1e-13, atol=1e-13)
    assert b["dA"][1].shape == (0,)


def test_diff_finite_differences_are_exact():
    """L = sum(Y * dY) is linear in the masked values and in X: central differences have no truncation error."""
    wl, st, lt = diff_problem(seed=3)
    b = run_bwd(wl, st, lt, **_kw(lt))
    eps = 2.0 ** -6
    rng = np.random.default_rng(3)

    def loss():
        return float(np.sum(run_fwd(wl, st, lt, **_kw(lt))["Y"] * masked(lt.dY, st.row_task)))

    def fd(arr, idx):
        old = arr[idx]
        arr[idx] = np.float32(old + eps); lp = loss()
        arr[idx] = np.float32(old - eps); lm = loss()
        arr[idx] = old
        return (lp - lm) / (2 * eps)

    for t, task in enumerate(wl.tasks):
        if task.kind != wlm.KIND_DIFF:
            continue
        rows = np.nonzero(st.row_task == t)[0]
        for e in range(0, lt.A[t].size, max(1, lt.A[t].size // 6)):
            g = fd(lt.A[t], (e,))
            assert abs(g - b["dA"][t][e]) <= 1e-9 * max(1.0, abs(g))
        for _ in range(6):
            i = int(rng.choice(rows)); k = int(rng.integers(0, lt.K))
            g = fd(lt.X, (i, k))
            assert abs(g - b["dX"][i, k]) <= 1e-9 * max(1.0, abs(g))


def test_diff_isolation_and_column_sampling():
    """NaN in the other tasks' rows and in the padding rows changes nothing; sampled columns equal the full run."""
    wl, st, lt = diff_problem(seed=4)
    f = run_fwd(wl, st, lt, **_kw(lt)); b = run_bwd(wl, st, lt, **_kw(lt))
    rows = st.row_task == 1
    lt2 = wlm.layer_tensors(wl, 0, st.T, seed=4)
    lt2.X[~rows] = np.nan; lt2.dY[~rows] = np.nan
    f2 = run_fwd(wl, st, lt2, **_kw(lt2)); b2 = run_bwd(wl, st, lt2, **_kw(lt2))
    assert np.array_equal(f2["Y"][rows], f["Y"][rows]) and np.array_equal(b2["dX"][rows], b["dX"][rows])
    assert np.array_equal(b2["dA"][1], b["dA"][1])
    cols = np.array([1, 4, 9], dtype=np.int32); kcols = np.array([0, 5, 13], dtype=np.int32)
    fs = run_fwd(wl, st, lt, cols=cols, **_kw(lt)); bs = run_bwd(wl, st, lt, cols=cols, kcols=kcols, **_kw(lt))
    assert np.array_equal(fs["Y"], f["Y"][:, cols]) and np.array_equal(bs["dX"], b["dX"][:, kcols])
