/*
 * TEST INFRASTRUCTURE -- fp64 CPU oracle of the multiplexed multi-task PEFT linear layer.
 *
 * Only the tests, the smoke check and the benchmark's cpu_baseline leg may call this.
 * It shares no code with the HIP library and is written for legibility, not speed:
 * every output element is the plain definition, summed in a fixed order
 * (rows ascending, inner index ascending), in double precision.
 *
 * What is computed (paper section 3.2, "Isolation and Convergence Guarantee"):
 *   - BaseOp forward (Eq. 1): the concatenated batch times the shared frozen weight,
 *     which equals each task's batch times that weight, row block by row block.
 *   - BaseOp backward (Eq. 2): the concatenated output gradients times the weight
 *     transposed.  No gradient of the backbone weight is ever formed (sections 1, 2.2).
 *   - Adapters are computed per task, independently (section 3.2, section 3.4.3).
 *     LoRA is the low-rank reparameterisation named in section 2.1 with the operator
 *     shape [tokens,K] x [K,r] given in section 2.2:  y = x W + s (x A) B.
 *   - Aggregate = add (section 3.4.3 names the Add operator); for the IA3-style task
 *     kind of the benchmark configs the aggregate is an elementwise product with a
 *     per-task vector l:  y = (x W) * l.
 *   - The additive kind (section 2.1 names Adapter-Tuning as the additive PEFT type and section 5
 *     lists it among the implemented ones, without a formula) is read as the usual bottleneck
 *     inserted after the BaseOp:  z = x W,  u = z D,  y = z + s gelu(u) U,  with D [N,r] passed
 *     in the A slot and U [r,N] in the B slot; gelu(u) = u/2 (1 + erf(u / sqrt 2)).
 *   - The selective kind (section 2.1 names Diff-Pruning: a subset of the parameters is fine-tuned through a
 *     binary mask; also among the implemented types of section 5, without a formula) is read as
 *     y = x (W + M * delta) with a fixed 0/1 mask M over the entries of W and trainable values delta on
 *     the masked entries only, given as a list of (k, n, value) sorted by (k, n); its gradient is the masked
 *     slice of the dense x^T g, the one place where entries of a weight gradient are formed.
 *   - Chunk alignment pads with zero tokens (section 3.5): a padding row's buffer
 *     content is ignored (selected away, never multiplied, so NaN there cannot leak),
 *     its outputs are zero, and it adds nothing to any gradient.
 *
 * Inputs are float arrays (every bf16 value is exactly a float; float -> double is exact).
 * row_task[i] is the task of row i, or -1 for a padding row.
 * cols/kcols optionally restrict the evaluated output columns (NULL = all), which lets
 * full-size workloads be checked on a sample of columns; everything that is contracted
 * over (h, q, dA, dB) is always evaluated in full.
 *
 * Pins: tests/test_oracle_pins.py (special cases against numpy's float64 matmul, the
 * merged-weight closed form, exact finite differences, hand-worked goldens, isolation
 * invariants).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define KIND_NONE 0
#define KIND_LORA 1
#define KIND_IA3 2
#define KIND_ADAPTER 3
#define KIND_DIFF 4
#define MAX_RANK 1024

static inline int has_rank(int kind) { return kind == KIND_LORA || kind == KIND_ADAPTER; }
static inline double gelu(double u) { return 0.5 * u * (1.0 + erf(u * 0.70710678118654752440)); }
static inline double gelu_prime(double u)
{
    return 0.5 * (1.0 + erf(u * 0.70710678118654752440)) + u * exp(-0.5 * u * u) * 0.39894228040143267794;
}

/* z[0..N) = x W, every column, summed in ascending k */
static void full_row_times_w(const float* x, const float* W, int K, int N, double* z)
{
    for (int n = 0; n < N; ++n) z[n] = 0.0;
    for (int k = 0; k < K; ++k) {
        const double xk = (double)x[k];
        const float* wrow = W + (size_t)k * N;
        for (int n = 0; n < N; ++n) z[n] += xk * (double)wrow[n];
    }
}

static inline int col_of(const int32_t* cols, int c) { return cols ? cols[c] : c; }

/* Forward.  Y[T,n_cols], H[T,r_max] (LoRA: x A_t, unscaled; additive kind: the pre-activation u = z D_t;
 * zero beyond rank and on pad rows), Z[T,n_cols] (x W before the aggregate; may be NULL). */
int mux_oracle_forward(int T, int K, int N,
                       const float* X, const float* W, const int32_t* row_task,
                       int n_tasks, const int32_t* kind, const int32_t* rank, const double* scale,
                       const float* const* A, const float* const* B, const float* const* L,
                       int n_cols, const int32_t* cols, int r_max,
                       double* Y, double* H, double* Z,
                       const int32_t* s_nnz, const int32_t* const* s_k, const int32_t* const* s_n)
{   /* selective kind: task t has s_nnz[t] masked entries (s_k[t][e], s_n[t][e]) with values A[t][e] */
    if (T < 0 || K <= 0 || N <= 0 || n_cols < 0 || r_max < 0) return 1;
    for (int i = 0; i < T; ++i) {
        int t = row_task[i];
        if (t >= n_tasks) return 2;
        if (t >= 0 && has_rank(kind[t]) && (rank[t] > r_max || rank[t] < 0 || rank[t] > MAX_RANK))
            return 3;
    }
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 4)
    for (int i = 0; i < T; ++i) {
        const int t = row_task[i];
        double* y = Y + (size_t)i * n_cols;
        double* h = H ? H + (size_t)i * r_max : NULL;
        double* zrow = Z ? Z + (size_t)i * n_cols : NULL;
        for (int c = 0; c < n_cols; ++c) y[c] = 0.0;
        if (h) for (int j = 0; j < r_max; ++j) h[j] = 0.0;
        if (zrow) for (int c = 0; c < n_cols; ++c) zrow[c] = 0.0;
        if (t < 0) continue;                       /* padding row: zero token in, zero out */
        const float* x = X + (size_t)i * K;
        /* z = x W   (Eq. 1); k outermost so that W is read row by row, each y[c] still
         * sums its products in ascending k */
        for (int k = 0; k < K; ++k) {
            const double xk = (double)x[k];
            const float* wrow = W + (size_t)k * N;
            for (int c = 0; c < n_cols; ++c) y[c] += xk * (double)wrow[col_of(cols, c)];
        }
        if (zrow) for (int c = 0; c < n_cols; ++c) zrow[c] = y[c];
        if (kind[t] == KIND_LORA) {
            const int r = rank[t];
            const float* At = A[t];
            const float* Bt = B[t];
            double hh[MAX_RANK];
            for (int j = 0; j < r; ++j) hh[j] = 0.0;
            for (int k = 0; k < K; ++k) {          /* h = x A_t */
                const double xk = (double)x[k];
                for (int j = 0; j < r; ++j) hh[j] += xk * (double)At[(size_t)k * r + j];
            }
            if (h) for (int j = 0; j < r; ++j) h[j] = hh[j];
            for (int c = 0; c < n_cols; ++c) {     /* y = z + s_t (h B_t)   (aggregate: add) */
                const int n = col_of(cols, c);
                double u = 0.0;
                for (int j = 0; j < r; ++j) u += hh[j] * (double)Bt[(size_t)j * N + n];
                y[c] += scale[t] * u;
            }
        } else if (kind[t] == KIND_IA3) {          /* y = z * l_t  (aggregate: multiply) */
            const float* l = L[t];
            for (int c = 0; c < n_cols; ++c) y[c] *= (double)l[col_of(cols, c)];
        } else if (kind[t] == KIND_DIFF) {         /* y = x (W + M_t * delta_t) = z + sum over masked (k, n) of x_k delta_kn */
            const float* dv = A[t];
            for (int c = 0; c < n_cols; ++c) {
                const int n = col_of(cols, c);
                double v = 0.0;
                for (int e = 0; e < s_nnz[t]; ++e)     /* entries are sorted by (k, n): ascending k inside a column */
                    if (s_n[t][e] == n) v += (double)x[s_k[t][e]] * (double)dv[e];
                y[c] += v;
            }
        } else if (kind[t] == KIND_ADAPTER) {      /* y = z + s_t gelu(z D_t) U_t */
            const int r = rank[t];
            const float* Dt = A[t];                /* [N, r] */
            const float* Ut = B[t];                /* [r, N] */
            double* zf = (double*)malloc(sizeof(double) * (size_t)N);
            if (!zf) { failed = 1; continue; }
            full_row_times_w(x, W, K, N, zf);      /* the bottleneck contracts over every output column */
            double uu[MAX_RANK], aa[MAX_RANK];
            for (int j = 0; j < r; ++j) uu[j] = 0.0;
            for (int n = 0; n < N; ++n)
                for (int j = 0; j < r; ++j) uu[j] += zf[n] * (double)Dt[(size_t)n * r + j];
            for (int j = 0; j < r; ++j) aa[j] = gelu(uu[j]);
            if (h) for (int j = 0; j < r; ++j) h[j] = uu[j];
            for (int c = 0; c < n_cols; ++c) {
                const int n = col_of(cols, c);
                double v = 0.0;
                for (int j = 0; j < r; ++j) v += aa[j] * (double)Ut[(size_t)j * N + n];
                y[c] += scale[t] * v;
            }
            free(zf);
        }
    }
    return failed ? 4 : 0;
}

/* Backward.
 *   dX[T,n_kcols]           (Eq. 2 plus the adapter's own input gradient)
 *   G[T,r_max]              q = g B_t^T, unscaled (may be NULL)
 *   dA[t] : [K, rank_t]     s_t * sum_i x_i^T q_i
 *   dB[t] : [rank_t, N]     s_t * sum_i h_i^T g_i
 *   dL[t] : [n_cols]        sum_i g_i * z_i   on the sampled output columns `cols`
 * Additive kind (D in the A slot, U in the B slot), per row: a = gelu(u), p = s_t (g U_t^T) * gelu'(u),
 *   dX = (g + p D_t^T) W^T,   G = p,   dA[t] : [N, rank_t] = sum_i z_i^T p_i,   dB[t] : [rank_t, N] = s_t sum_i a_i^T g_i
 * Gradient outputs are overwritten.  Entries of dA/dB/dL may be NULL to skip a task. */
int mux_oracle_backward(int T, int K, int N,
                        const float* X, const float* dY, const float* W, const int32_t* row_task,
                        int n_tasks, const int32_t* kind, const int32_t* rank, const double* scale,
                        const float* const* A, const float* const* B, const float* const* L,
                        int n_kcols, const int32_t* kcols,
                        int n_cols, const int32_t* cols, int r_max,
                        double* dX, double* G, double* const* dA, double* const* dB,
                        double* const* dL,
                        const int32_t* s_nnz, const int32_t* const* s_k, const int32_t* const* s_n)
{   /* selective kind: dX = g (W + M_t * delta_t)^T, dA[t][e] = sum_i x_i[k_e] g_i[n_e] */
    if (T < 0 || K <= 0 || N <= 0 || r_max < 0) return 1;
    for (int i = 0; i < T; ++i) {
        int t = row_task[i];
        if (t >= n_tasks) return 2;
        if (t >= 0 && has_rank(kind[t]) && (rank[t] > r_max || rank[t] < 0 || rank[t] > MAX_RANK))
            return 3;
    }
    /* per-row quantities h = x A_t and q = g B_t^T (additive kind: a and p), kept in full */
    double* Hf = (double*)calloc((size_t)(T > 0 ? T : 1) * (r_max > 0 ? r_max : 1), sizeof(double));
    double* Qf = (double*)calloc((size_t)(T > 0 ? T : 1) * (r_max > 0 ? r_max : 1), sizeof(double));
    if (!Hf || !Qf) { free(Hf); free(Qf); return 4; }
    /* z = x W of the additive kind's rows, every column (its D gradient contracts z with p) */
    int any_adapter = 0;
    for (int t = 0; t < n_tasks; ++t) any_adapter |= kind[t] == KIND_ADAPTER;
    double* Zf = any_adapter ? (double*)calloc((size_t)(T > 0 ? T : 1) * N, sizeof(double)) : NULL;
    if (any_adapter && !Zf) { free(Hf); free(Qf); return 4; }
    int failed = 0;

#pragma omp parallel for schedule(dynamic, 4)
    for (int i = 0; i < T; ++i) {
        const int t = row_task[i];
        double* dx = dX ? dX + (size_t)i * n_kcols : NULL;
        if (dx) for (int c = 0; c < n_kcols; ++c) dx[c] = 0.0;
        if (t < 0) continue;                       /* padding row: zero gradient in and out */
        const float* x = X + (size_t)i * K;
        const float* g = dY + (size_t)i * N;
        if (kind[t] == KIND_LORA) {
            const int r = rank[t];
            const float* At = A[t];
            const float* Bt = B[t];
            double* h = Hf + (size_t)i * r_max;
            double* q = Qf + (size_t)i * r_max;
            for (int k = 0; k < K; ++k) {                   /* h = x A_t */
                const double xk = (double)x[k];
                for (int j = 0; j < r; ++j) h[j] += xk * (double)At[(size_t)k * r + j];
            }
            for (int j = 0; j < r; ++j) {                   /* q = g B_t^T */
                double u = 0.0;
                for (int n = 0; n < N; ++n) u += (double)g[n] * (double)Bt[(size_t)j * N + n];
                q[j] = u;
            }
            if (dx) for (int c = 0; c < n_kcols; ++c) {     /* dx = g W^T + s_t q A_t^T */
                const int k = col_of(kcols, c);
                double s = 0.0;
                for (int n = 0; n < N; ++n) s += (double)g[n] * (double)W[(size_t)k * N + n];
                double u = 0.0;
                for (int j = 0; j < r; ++j) u += q[j] * (double)At[(size_t)k * r + j];
                dx[c] = s + scale[t] * u;
            }
        } else if (kind[t] == KIND_ADAPTER) {
            const int r = rank[t];
            const float* Dt = A[t];
            const float* Ut = B[t];
            double* zf = Zf + (size_t)i * N;
            double* a = Hf + (size_t)i * r_max;
            double* pp = Qf + (size_t)i * r_max;
            double* dz = (double*)malloc(sizeof(double) * (size_t)N);
            if (!dz) { failed = 1; continue; }
            full_row_times_w(x, W, K, N, zf);
            for (int j = 0; j < r; ++j) {
                double u = 0.0;                              /* u = z D_t */
                for (int n = 0; n < N; ++n) u += zf[n] * (double)Dt[(size_t)n * r + j];
                double da = 0.0;                             /* g U_t^T */
                for (int n = 0; n < N; ++n) da += (double)g[n] * (double)Ut[(size_t)j * N + n];
                a[j] = gelu(u);
                pp[j] = scale[t] * da * gelu_prime(u);
            }
            for (int n = 0; n < N; ++n) {                    /* dz = g + p D_t^T */
                double v = 0.0;
                for (int j = 0; j < r; ++j) v += pp[j] * (double)Dt[(size_t)n * r + j];
                dz[n] = (double)g[n] + v;
            }
            if (dx) for (int c = 0; c < n_kcols; ++c) {     /* dx = dz W^T */
                const int k = col_of(kcols, c);
                double s = 0.0;
                for (int n = 0; n < N; ++n) s += dz[n] * (double)W[(size_t)k * N + n];
                dx[c] = s;
            }
            free(dz);
        } else if (kind[t] == KIND_DIFF) {                  /* dx = g W^T + g (M_t * delta_t)^T */
            const float* dv = A[t];
            if (dx) for (int c = 0; c < n_kcols; ++c) {
                const int k = col_of(kcols, c);
                double s = 0.0;
                for (int n = 0; n < N; ++n) s += (double)g[n] * (double)W[(size_t)k * N + n];
                double v = 0.0;
                for (int e = 0; e < s_nnz[t]; ++e)
                    if (s_k[t][e] == k) v += (double)g[s_n[t][e]] * (double)dv[e];
                dx[c] = s + v;
            }
        } else if (kind[t] == KIND_IA3) {                   /* dx = (g * l_t) W^T */
            const float* l = L[t];
            if (dx) for (int c = 0; c < n_kcols; ++c) {
                const int k = col_of(kcols, c);
                double s = 0.0;
                for (int n = 0; n < N; ++n)
                    s += ((double)g[n] * (double)l[n]) * (double)W[(size_t)k * N + n];
                dx[c] = s;
            }
        } else {                                            /* dx = g W^T      (Eq. 2) */
            if (dx) for (int c = 0; c < n_kcols; ++c) {
                const int k = col_of(kcols, c);
                double s = 0.0;
                for (int n = 0; n < N; ++n) s += (double)g[n] * (double)W[(size_t)k * N + n];
                dx[c] = s;
            }
        }
    }
    if (G) memcpy(G, Qf, sizeof(double) * (size_t)T * r_max);

    /* per-task parameter gradients: rows of the task only, added in ascending row order;
     * threads split the output (never the sum), so the order is the same for any thread count */
    for (int t = 0; t < n_tasks; ++t) {
        if (kind[t] == KIND_LORA) {
            const int r = rank[t];
            if (dA && dA[t]) {                              /* dA_t = s_t sum_i x_i^T q_i */
                double* da = dA[t];
#pragma omp parallel for schedule(static)
                for (int k0 = 0; k0 < K; k0 += 64) {
                    const int k1 = k0 + 64 < K ? k0 + 64 : K;
                    for (int k = k0; k < k1; ++k)
                        for (int j = 0; j < r; ++j) da[(size_t)k * r + j] = 0.0;
                    for (int i = 0; i < T; ++i) {
                        if (row_task[i] != t) continue;
                        const float* x = X + (size_t)i * K;
                        const double* q = Qf + (size_t)i * r_max;
                        for (int k = k0; k < k1; ++k)
                            for (int j = 0; j < r; ++j) da[(size_t)k * r + j] += (double)x[k] * q[j];
                    }
                    for (int k = k0; k < k1; ++k)
                        for (int j = 0; j < r; ++j) da[(size_t)k * r + j] *= scale[t];
                }
            }
            if (dB && dB[t]) {                              /* dB_t = s_t sum_i h_i^T g_i */
                double* db = dB[t];
#pragma omp parallel for schedule(static)
                for (int n0 = 0; n0 < N; n0 += 256) {
                    const int n1 = n0 + 256 < N ? n0 + 256 : N;
                    for (int j = 0; j < r; ++j)
                        for (int n = n0; n < n1; ++n) db[(size_t)j * N + n] = 0.0;
                    for (int i = 0; i < T; ++i) {
                        if (row_task[i] != t) continue;
                        const double* h = Hf + (size_t)i * r_max;
                        const float* g = dY + (size_t)i * N;
                        for (int j = 0; j < r; ++j)
                            for (int n = n0; n < n1; ++n) db[(size_t)j * N + n] += h[j] * (double)g[n];
                    }
                    for (int j = 0; j < r; ++j)
                        for (int n = n0; n < n1; ++n) db[(size_t)j * N + n] *= scale[t];
                }
            }
        } else if (kind[t] == KIND_DIFF) {
            if (dA && dA[t]) {                              /* d delta_e = sum_i x_i[k_e] g_i[n_e]: masked entries of x^T g */
                double* dd = dA[t];
#pragma omp parallel for schedule(static)
                for (int e = 0; e < s_nnz[t]; ++e) {
                    double v = 0.0;
                    for (int i = 0; i < T; ++i) {
                        if (row_task[i] != t) continue;
                        v += (double)X[(size_t)i * K + s_k[t][e]] * (double)dY[(size_t)i * N + s_n[t][e]];
                    }
                    dd[e] = v;
                }
            }
        } else if (kind[t] == KIND_ADAPTER) {
            const int r = rank[t];
            if (dA && dA[t]) {                              /* dD_t = sum_i z_i^T p_i   [N, r] */
                double* dd = dA[t];
#pragma omp parallel for schedule(static)
                for (int n0 = 0; n0 < N; n0 += 64) {
                    const int n1 = n0 + 64 < N ? n0 + 64 : N;
                    for (int n = n0; n < n1; ++n)
                        for (int j = 0; j < r; ++j) dd[(size_t)n * r + j] = 0.0;
                    for (int i = 0; i < T; ++i) {
                        if (row_task[i] != t) continue;
                        const double* zf = Zf + (size_t)i * N;
                        const double* pp = Qf + (size_t)i * r_max;
                        for (int n = n0; n < n1; ++n)
                            for (int j = 0; j < r; ++j) dd[(size_t)n * r + j] += zf[n] * pp[j];
                    }
                }
            }
            if (dB && dB[t]) {                              /* dU_t = s_t sum_i a_i^T g_i   [r, N] */
                double* du = dB[t];
#pragma omp parallel for schedule(static)
                for (int n0 = 0; n0 < N; n0 += 256) {
                    const int n1 = n0 + 256 < N ? n0 + 256 : N;
                    for (int j = 0; j < r; ++j)
                        for (int n = n0; n < n1; ++n) du[(size_t)j * N + n] = 0.0;
                    for (int i = 0; i < T; ++i) {
                        if (row_task[i] != t) continue;
                        const double* a = Hf + (size_t)i * r_max;
                        const float* g = dY + (size_t)i * N;
                        for (int j = 0; j < r; ++j)
                            for (int n = n0; n < n1; ++n) du[(size_t)j * N + n] += a[j] * (double)g[n];
                    }
                    for (int j = 0; j < r; ++j)
                        for (int n = n0; n < n1; ++n) du[(size_t)j * N + n] *= scale[t];
                }
            }
        } else if (kind[t] == KIND_IA3) {
            if (dL && dL[t]) {                              /* dl_t = sum_i g_i * z_i,  z = x W */
                double* dl = dL[t];
#pragma omp parallel for schedule(static)
                for (int c0 = 0; c0 < n_cols; c0 += 16) {
                    const int c1 = c0 + 16 < n_cols ? c0 + 16 : n_cols;
                    double z[16];
                    for (int c = c0; c < c1; ++c) dl[c] = 0.0;
                    for (int i = 0; i < T; ++i) {
                        if (row_task[i] != t) continue;
                        const float* x = X + (size_t)i * K;
                        for (int c = c0; c < c1; ++c) z[c - c0] = 0.0;
                        for (int k = 0; k < K; ++k) {
                            const double xk = (double)x[k];
                            const float* wrow = W + (size_t)k * N;
                            for (int c = c0; c < c1; ++c) z[c - c0] += xk * (double)wrow[col_of(cols, c)];
                        }
                        for (int c = c0; c < c1; ++c)
                            dl[c] += (double)dY[(size_t)i * N + col_of(cols, c)] * z[c - c0];
                    }
                }
            }
        }
    }
    free(Hf);
    free(Qf);
    free(Zf);
    return failed ? 4 : 0;
}

int mux_oracle_max_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
