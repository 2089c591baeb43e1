"""The pins must catch plausible mistakes: each case plants one mistake in a COPY of the oracle's C source
(on the CPU, in a temporary directory), builds it, and runs the pin tests against it in a subprocess; the
run has to fail.  The unmodified copy has to pass."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "mux_oracle.c")

MUTATIONS = {
    "forward_drops_scale": ("y[c] += scale[t] * u;", "y[c] += u;"),
    "forward_pad_row_leaks": ("        if (t < 0) continue;                       /* padding row: zero token in, zero out */", ""),
    "forward_B_columns_reversed": ("for (int j = 0; j < r; ++j) u += hh[j] * (double)Bt[(size_t)j * N + n];",
                                   "for (int j = 0; j < r; ++j) u += hh[j] * (double)Bt[(size_t)j * N + (N - 1 - n)];"),
    "forward_ia3_adds_instead_of_multiplies": ("y[c] *= (double)l[col_of(cols, c)];", "y[c] += (double)l[col_of(cols, c)];"),
    "backward_adapter_sign": ("dx[c] = s + scale[t] * u;", "dx[c] = s - scale[t] * u;"),
    "backward_ia3_forgets_l": ("s += ((double)g[n] * (double)l[n]) * (double)W[(size_t)k * N + n];",
                               "s += ((double)g[n]) * (double)W[(size_t)k * N + n];"),
    "dA_uses_h_instead_of_q": ("const double* q = Qf + (size_t)i * r_max;\n                        for (int k = k0; k < k1; ++k)",
                               "const double* q = Hf + (size_t)i * r_max;\n                        for (int k = k0; k < k1; ++k)"),
    "dB_without_scale": ("for (int n = n0; n < n1; ++n) db[(size_t)j * N + n] *= scale[t];", ";"),
    "dA_sums_rows_of_other_tasks": ("                    for (int i = 0; i < T; ++i) {\n                        if (row_task[i] != t) continue;\n                        const float* x = X + (size_t)i * K;\n                        const double* q",
                                    "                    for (int i = 0; i < T; ++i) {\n                        if (row_task[i] < 0) continue;\n                        const float* x = X + (size_t)i * K;\n                        const double* q"),
    "dl_uses_scaled_output": ("dl[c] += (double)dY[(size_t)i * N + col_of(cols, c)] * z[c - c0];",
                              "dl[c] += (double)dY[(size_t)i * N + col_of(cols, c)] * z[c - c0] * (double)L[t][col_of(cols, c)];"),
    "additive_forward_drops_scale": ("y[c] += scale[t] * v;", "y[c] += v;"),
    "additive_forward_without_activation": ("for (int j = 0; j < r; ++j) aa[j] = gelu(uu[j]);", "for (int j = 0; j < r; ++j) aa[j] = uu[j];"),
    "additive_backward_drops_activation_slope": ("pp[j] = scale[t] * da * gelu_prime(u);", "pp[j] = scale[t] * da;"),
    "additive_backward_forgets_residual": ("dz[n] = (double)g[n] + v;", "dz[n] = v;"),
    "additive_dD_uses_activation_instead_of_z": ("for (int j = 0; j < r; ++j) dd[(size_t)n * r + j] += zf[n] * pp[j];",
                                                 "for (int j = 0; j < r; ++j) dd[(size_t)n * r + j] += (double)dY[(size_t)i * N + n] * pp[j];"),
    "additive_dU_without_scale": ("for (int n = n0; n < n1; ++n) du[(size_t)j * N + n] *= scale[t];", ";"),
    "gelu_slope_misses_density_term": ("return 0.5 * (1.0 + erf(u * 0.70710678118654752440)) + u * exp(-0.5 * u * u) * 0.39894228040143267794;",
                                       "return 0.5 * (1.0 + erf(u * 0.70710678118654752440));"),
    "selective_forward_swaps_mask_indices": ("if (s_n[t][e] == n) v += (double)x[s_k[t][e]] * (double)dv[e];",
                                             "if (s_k[t][e] == n) v += (double)x[s_n[t][e]] * (double)dv[e];"),
    "selective_backward_forgets_sparse_part": ("dx[c] = s + v;", "dx[c] = s;"),
    "selective_gradient_sums_all_rows": ("                    for (int i = 0; i < T; ++i) {\n                        if (row_task[i] != t) continue;\n                        v += (double)X[(size_t)i * K + s_k[t][e]]",
                                         "                    for (int i = 0; i < T; ++i) {\n                        if (row_task[i] < 0) continue;\n                        v += (double)X[(size_t)i * K + s_k[t][e]]"),
    "q_contracts_over_wrong_operand": ("for (int n = 0; n < N; ++n) u += (double)g[n] * (double)Bt[(size_t)j * N + n];\n                q[j] = u;",
                                       "for (int n = 0; n < N; ++n) u += (double)g[n] * (double)Bt[(size_t)j * N + n];\n                q[j] = u * 0.5;"),
}


def _build(tmp_path, name, old, new):
    src = open(SRC).read()
    if old is not None:
        assert src.count(old) == 1, f"mutation {name}: pattern must occur exactly once ({src.count(old)})"
        src = src.replace(old, new)
    c = tmp_path / f"{name}.c"
    so = tmp_path / f"{name}.so"
    c.write_text(src)
    subprocess.check_call(["gcc", "-O1", "-fopenmp", "-shared", "-fPIC", "-o", str(so), str(c), "-lm"])
    return str(so)


def _run_pins(lib):
    env = dict(os.environ, MUX_ORACLE_LIB=lib, OMP_NUM_THREADS="2")
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-k", "not thread_count"],
                       cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
    return r.returncode, r.stdout.decode()[-400:]


def test_unmodified_copy_passes(tmp_path):
    rc, out = _run_pins(_build(tmp_path, "clean", None, None))
    assert rc == 0, out


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_planted_mistake_is_caught(tmp_path, name):
    old, new = MUTATIONS[name]
    rc, out = _run_pins(_build(tmp_path, name, old, new))
    assert rc != 0, f"no pin noticed the planted mistake '{name}'"
