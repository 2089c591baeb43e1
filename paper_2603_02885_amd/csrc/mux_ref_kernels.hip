// Plain HIP kernels (LDS-tiled FMA, no matrix cores) for every step of the layer, in both
// storage types.  They serve the fp32 correctness mode and MUX_LAYER_REFERENCE_KERNELS.
//
// One generic 64x64 output tile per workgroup of 256 threads; the operands are given as
// accessors so that the masking rules live next to the formula they implement:
// a padding row is *selected* to zero before any product (its buffer content may be NaN).
#include "mux_device_utils.h"

namespace mux {
namespace {

constexpr int TS64 = 0;  // index of the 64-row work list

// acc[u][v] += sum_k fa(ty*4+u, k) * fb(k, tx*4+v),  k in [0, Kc)
template <class FA, class FB>
__device__ __forceinline__ void tile64(FA fa, FB fb, int Kc, float (&acc)[4][4]) {
  __shared__ float sa[16][65];
  __shared__ float sb[16][65];
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  for (int k0 = 0; k0 < Kc; k0 += 16) {
    for (int e = threadIdx.x; e < 1024; e += 256) {
      const int m = e >> 4, kk = e & 15;
      sa[kk][m] = (k0 + kk < Kc) ? fa(m, k0 + kk) : 0.f;
    }
    for (int e = threadIdx.x; e < 1024; e += 256) {
      const int kk = e >> 6, n = e & 63;
      sb[kk][n] = (k0 + kk < Kc) ? fb(k0 + kk, n) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) a[u] = sa[kk][ty * 4 + u];
#pragma unroll
      for (int v = 0; v < 4; ++v) b[v] = sb[kk][tx * 4 + v];
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[u][v] = fmaf(a[u], b[v], acc[u][v]);
    }
    __syncthreads();
  }
}

// gelu(u) = u/2 (1 + erf(u / sqrt 2)) and its slope, in fp32
__device__ __forceinline__ float gelu_f(float u) { return 0.5f * u * (1.f + erff(u * 0.70710678f)); }
__device__ __forceinline__ float gelu_slope_f(float u) {
  return 0.5f * (1.f + erff(u * 0.70710678f)) + u * __expf(-0.5f * u * u) * 0.39894228f;
}
__device__ __forceinline__ bool kind_in(int kind, unsigned mask) { return (mask >> kind) & 1u; }
constexpr unsigned KM_LORA = 1u << MUX_ADAPTER_LORA, KM_TUNING = 1u << MUX_ADAPTER_TUNING;

#define ZERO_ACC(acc)                         \
  float acc[4][4];                            \
  _Pragma("unroll") for (int u = 0; u < 4; ++u) _Pragma("unroll") for (int v = 0; v < 4; ++v) acc[u][v] = 0.f

// S1: Hs = s_t * (x A_t) for LoRA rows, 0 elsewhere.  grid.x = 64-row items.
template <class S>
__global__ __launch_bounds__(256) void k_ref_down(const int32_t* __restrict__ dtab, const DevTask* __restrict__ tasks,
                                                  const S* __restrict__ X, S* __restrict__ H, int K, int RP) {
  const ItemView it = load_item(dtab, TS64, blockIdx.x);
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  ZERO_ACC(acc);
  float scale = 0.f;
  if (it.task >= 0 && tasks[it.task].kind == MUX_ADAPTER_LORA) {
    const DevTask tk = tasks[it.task];
    const S* A = (const S*)tk.A;
    const int r = tk.rank;
    scale = tk.scale;
    auto fa = [&](int m, int k) -> float {
      const int row = it.row0 + m;
      return (m < it.nrows && row_is_valid(dtab, row)) ? Store<S>::ld(X, (size_t)row * K + k) : 0.f;
    };
    auto fb = [&](int k, int j) -> float { return j < r ? Store<S>::ld(A, (size_t)k * r + j) : 0.f; };
    tile64(fa, fb, K, acc);
  }
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int m = ty * 4 + u, row = it.row0 + m;
    if (m >= it.nrows) continue;
    const bool ok = scale != 0.f && row_is_valid(dtab, row);
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int j = tx * 4 + v;
      if (j < RP) Store<S>::st(H, (size_t)row * RP + j, ok ? scale * acc[u][v] : 0.f);
    }
  }
}

// S2: Y = mask * (x W + Hs B_t)   or   mask * ((x W) * l_t).  grid = (items, ceil(N/64)).
template <class S>
__global__ __launch_bounds__(256) void k_ref_fwd(const int32_t* __restrict__ dtab, const DevTask* __restrict__ tasks,
                                                 const S* __restrict__ X, const S* __restrict__ W, int64_t ldw,
                                                 const S* __restrict__ H, S* __restrict__ Y, S* __restrict__ Z, int K, int N,
                                                 int RP) {
  const ItemView it = load_item(dtab, TS64, blockIdx.x);
  const int n0 = blockIdx.y * 64;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  ZERO_ACC(acc);
  int kind = MUX_ADAPTER_NONE;
  DevTask tk{};
  if (it.task >= 0 && it.nvalid > 0) {
    tk = tasks[it.task];
    kind = tk.kind;
    auto fa = [&](int m, int k) -> float {
      const int row = it.row0 + m;
      return (m < it.nrows && row_is_valid(dtab, row)) ? Store<S>::ld(X, (size_t)row * K + k) : 0.f;
    };
    auto fb = [&](int k, int n) -> float { return n0 + n < N ? Store<S>::ld(W, (size_t)k * ldw + n0 + n) : 0.f; };
    tile64(fa, fb, K, acc);
    if (kind == MUX_ADAPTER_LORA) {
      const S* B = (const S*)tk.B;
      const int r = tk.rank;
      auto ha = [&](int m, int j) -> float {   // Hs is zero on padding rows by construction
        return m < it.nrows ? Store<S>::ld(H, (size_t)(it.row0 + m) * RP + j) : 0.f;
      };
      auto hb = [&](int j, int n) -> float { return n0 + n < N ? Store<S>::ld(B, (size_t)j * N + n0 + n) : 0.f; };
      tile64(ha, hb, r, acc);
    }
  }
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int m = ty * 4 + u, row = it.row0 + m;
    if (m >= it.nrows) continue;
    const bool ok = it.task >= 0 && row_is_valid(dtab, row);
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int n = n0 + tx * 4 + v;
      if (n >= N) continue;
      float y = acc[u][v];
      if (kind == MUX_ADAPTER_IA3_OUT || kind == MUX_ADAPTER_TUNING) {
        if (Z) Store<S>::st(Z, (size_t)(tk.zrow0 + row - tk.row_begin) * N + n, ok ? y : 0.f);
        if (kind == MUX_ADAPTER_IA3_OUT) y *= Store<S>::ld((const S*)tk.L, n);
      }
      Store<S>::st(Y, (size_t)row * N + n, ok ? y : 0.f);      // TUNING: z for now, the bottleneck is added after this kernel
    }
  }
}

// S4a: Gs = s_t * (g B_t^T) for LoRA rows; TUNING rows: Gs = s_t (g U_t^T) * gelu'(u) with the saved pre-activation u.
// Rows of the kinds in `kinds` are computed; the others are written as zero if `zero_others`, else left alone.
// grid.x = items.
template <class S>
__global__ __launch_bounds__(256) void k_ref_g(const int32_t* __restrict__ dtab, const DevTask* __restrict__ tasks,
                                               const S* __restrict__ dY, const S* __restrict__ U2, S* __restrict__ G, int N,
                                               int RP, unsigned kinds, int zero_others) {
  const ItemView it = load_item(dtab, TS64, blockIdx.x);
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  ZERO_ACC(acc);
  float scale = 0.f;
  const int kind = it.task >= 0 ? tasks[it.task].kind : MUX_ADAPTER_NONE;
  const bool mine = kind_in(kind, kinds & (KM_LORA | KM_TUNING));
  if (!mine && !zero_others) return;
  if (mine) {
    const DevTask tk = tasks[it.task];
    const S* B = (const S*)tk.B;
    const int r = tk.rank;
    scale = tk.scale;
    auto fa = [&](int m, int n) -> float {
      const int row = it.row0 + m;
      return (m < it.nrows && row_is_valid(dtab, row)) ? Store<S>::ld(dY, (size_t)row * N + n) : 0.f;
    };
    auto fb = [&](int n, int j) -> float { return j < r ? Store<S>::ld(B, (size_t)j * N + n) : 0.f; };
    tile64(fa, fb, N, acc);
  }
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int m = ty * 4 + u, row = it.row0 + m;
    if (m >= it.nrows) continue;
    const bool ok = scale != 0.f && row_is_valid(dtab, row);
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int j = tx * 4 + v;
      if (j >= RP) continue;
      float q = ok ? scale * acc[u][v] : 0.f;
      if (ok && kind == MUX_ADAPTER_TUNING) q *= gelu_slope_f(Store<S>::ld(U2, (size_t)row * RP + j));
      Store<S>::st(G, (size_t)row * RP + j, q);
    }
  }
}

// S5: dX = mask * (g W^T + Gs A_t^T)   or   mask * ((g * l_t) W^T).  grid = (items, ceil(K/64)).
template <class S>
__global__ __launch_bounds__(256) void k_ref_dx(const int32_t* __restrict__ dtab, const DevTask* __restrict__ tasks,
                                                const S* __restrict__ dY, const S* __restrict__ W, int64_t ldw,
                                                const S* __restrict__ G, const S* __restrict__ dYs, S* __restrict__ dX, int K,
                                                int N, int RP) {
  const ItemView it = load_item(dtab, TS64, blockIdx.x);
  const int k0 = blockIdx.y * 64;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  ZERO_ACC(acc);
  if (it.task >= 0 && it.nvalid > 0) {
    const DevTask tk = tasks[it.task];
    const S* L = tk.kind == MUX_ADAPTER_IA3_OUT ? (const S*)tk.L : nullptr;
    const bool tuning = tk.kind == MUX_ADAPTER_TUNING;      // its rows enter as dY + p D_t^T, prepared in dYs
    auto fa = [&](int m, int n) -> float {
      const int row = it.row0 + m;
      if (!(m < it.nrows && row_is_valid(dtab, row))) return 0.f;
      if (tuning) return Store<S>::ld(dYs, (size_t)(tk.zrow0 + row - tk.row_begin) * N + n);
      const float g = Store<S>::ld(dY, (size_t)row * N + n);
      return L ? g * Store<S>::ld(L, n) : g;
    };
    auto fb = [&](int n, int kk) -> float { return k0 + kk < K ? Store<S>::ld(W, (size_t)(k0 + kk) * ldw + n) : 0.f; };
    tile64(fa, fb, N, acc);
    if (tk.kind == MUX_ADAPTER_LORA) {
      const S* A = (const S*)tk.A;
      const int r = tk.rank;
      auto ga = [&](int m, int j) -> float { return m < it.nrows ? Store<S>::ld(G, (size_t)(it.row0 + m) * RP + j) : 0.f; };
      auto gb = [&](int j, int kk) -> float { return k0 + kk < K ? Store<S>::ld(A, (size_t)(k0 + kk) * r + j) : 0.f; };
      tile64(ga, gb, r, acc);
    }
  }
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int m = ty * 4 + u, row = it.row0 + m;
    if (m >= it.nrows) continue;
    const bool ok = it.task >= 0 && row_is_valid(dtab, row);
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int k = k0 + tx * 4 + v;
      if (k < K) Store<S>::st(dX, (size_t)row * K + k, ok ? acc[u][v] : 0.f);
    }
  }
}

// S4b: dB_t[j][n] = sum_{rows of t} Hs[i][j] g[i][n].  grid = (tasks, ceil(N/64)); one workgroup walks all
// rows of the task in ascending order, so the sum order is fixed.
template <class S>
__global__ __launch_bounds__(256) void k_ref_db(const int32_t* __restrict__ dtab, const DevTask* __restrict__ tasks,
                                                const S* __restrict__ dY, const S* __restrict__ H, int N, int RP,
                                                int accumulate, unsigned kinds) {
  const DevTask tk = tasks[blockIdx.x];      // TUNING: Hs = s_t gelu(u), so the same sum gives dU_t
  if (!kind_in(tk.kind, kinds & (KM_LORA | KM_TUNING)) || tk.dB == nullptr) return;
  const int n0 = blockIdx.y * 64;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int r = tk.rank;
  ZERO_ACC(acc);
  auto fa = [&](int j, int i) -> float { return j < r ? Store<S>::ld(H, (size_t)(tk.row_begin + i) * RP + j) : 0.f; };
  auto fb = [&](int i, int n) -> float {
    const int row = tk.row_begin + i;
    return (n0 + n < N && row_is_valid(dtab, row)) ? Store<S>::ld(dY, (size_t)row * N + n0 + n) : 0.f;
  };
  tile64(fa, fb, tk.row_count, acc);
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int j = ty * 4 + u;
    if (j >= r) continue;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int n = n0 + tx * 4 + v;
      if (n >= N) continue;
      float* p = tk.dB + (size_t)j * N + n;
      *p = accumulate ? *p + acc[u][v] : acc[u][v];
    }
  }
}

// S6a: dA_t[k][j] = sum_{rows of t} x[i][k] Gs[i][j]; TUNING: dD_t[n][j] = sum z[i][n] Gs[i][j] with the saved z.
// grid = (tasks, ceil(max(K, N)/64)).
template <class S>
__global__ __launch_bounds__(256) void k_ref_da(const int32_t* __restrict__ dtab, const DevTask* __restrict__ tasks,
                                                const S* __restrict__ X, const S* __restrict__ Z, const S* __restrict__ G,
                                                int Kx, int N, int RP, int accumulate, unsigned kinds) {
  const DevTask tk = tasks[blockIdx.x];
  if (!kind_in(tk.kind, kinds & (KM_LORA | KM_TUNING)) || tk.dA == nullptr) return;
  const bool tuning = tk.kind == MUX_ADAPTER_TUNING;
  const int K = tuning ? N : Kx;               // rows of the gradient
  const int k0 = blockIdx.y * 64;
  if (k0 >= K) return;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int r = tk.rank;
  ZERO_ACC(acc);
  auto fa = [&](int kk, int i) -> float {
    const int row = tk.row_begin + i;
    if (!(k0 + kk < K && row_is_valid(dtab, row))) return 0.f;
    return tuning ? Store<S>::ld(Z, (size_t)(tk.zrow0 + i) * N + k0 + kk) : Store<S>::ld(X, (size_t)row * K + k0 + kk);
  };
  auto fb = [&](int i, int j) -> float { return j < r ? Store<S>::ld(G, (size_t)(tk.row_begin + i) * RP + j) : 0.f; };
  tile64(fa, fb, tk.row_count, acc);
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int k = k0 + ty * 4 + u;
    if (k >= K) continue;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int j = tx * 4 + v;
      if (j >= r) continue;
      float* p = tk.dA + (size_t)k * r + j;
      *p = accumulate ? *p + acc[u][v] : acc[u][v];
    }
  }
}

// S6b: dl_t[n] = sum_{rows of t} g[i][n] * z[i][n].  grid = (tasks, ceil(N/256)).
template <class S>
__global__ __launch_bounds__(256) void k_ref_dl(const int32_t* __restrict__ dtab, const DevTask* __restrict__ tasks,
                                                const S* __restrict__ dY, const S* __restrict__ Z, int N, int accumulate) {
  const DevTask tk = tasks[blockIdx.x];
  if (tk.kind != MUX_ADAPTER_IA3_OUT || tk.dL == nullptr) return;
  const int n = blockIdx.y * 256 + threadIdx.x;
  if (n >= N) return;
  float s = 0.f;
  for (int i = 0; i < tk.row_count; ++i) {
    const int row = tk.row_begin + i;
    if (!row_is_valid(dtab, row)) continue;
    s = fmaf(Store<S>::ld(dY, (size_t)row * N + n), Store<S>::ld(Z, (size_t)(tk.zrow0 + i) * N + n), s);
  }
  tk.dL[n] = accumulate ? tk.dL[n] + s : s;
}

// TUNING forward, first part: u = z D_t (kept for the backward pass), Hs = s_t gelu(u).  Only the rows of TUNING
// tasks are written.  grid.x = items.
template <class S>
__global__ __launch_bounds__(256) void k_tune_down(const int32_t* __restrict__ dtab, const DevTask* __restrict__ tasks,
                                                   const S* __restrict__ Z, S* __restrict__ U2, S* __restrict__ H, int N, int RP) {
  const ItemView it = load_item(dtab, TS64, blockIdx.x);
  if (it.task < 0 || tasks[it.task].kind != MUX_ADAPTER_TUNING) return;
  const DevTask tk = tasks[it.task];
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const S* D = (const S*)tk.A;                 // [N, r]
  const int r = tk.rank;
  ZERO_ACC(acc);
  auto fa = [&](int m, int n) -> float {
    const int row = it.row0 + m;
    return (m < it.nrows && row_is_valid(dtab, row)) ? Store<S>::ld(Z, (size_t)(tk.zrow0 + row - tk.row_begin) * N + n) : 0.f;
  };
  auto fb = [&](int n, int j) -> float { return j < r ? Store<S>::ld(D, (size_t)n * r + j) : 0.f; };
  tile64(fa, fb, N, acc);
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int m = ty * 4 + u, row = it.row0 + m;
    if (m >= it.nrows) continue;
    const bool valid = row_is_valid(dtab, row);
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int j = tx * 4 + v;
      if (j >= RP) continue;
      const bool ok = valid && j < r;
      Store<S>::st(U2, (size_t)row * RP + j, ok ? acc[u][v] : 0.f);
      Store<S>::st(H, (size_t)row * RP + j, ok ? tk.scale * gelu_f(acc[u][v]) : 0.f);
    }
  }
}

// TUNING: Out = In + Small P for the rows of TUNING tasks; P = U_t [r, N] (forward: Y = z + Hs U_t, In = saved z,
// Out = Y) or P = D_t^T (backward: dYs = dY + Gs D_t^T, In = dY, Out = the compact dYs rows).
// grid = (items, ceil(N/64)).
template <class S>
__global__ __launch_bounds__(256) void k_tune_add(const int32_t* __restrict__ dtab, const DevTask* __restrict__ tasks,
                                                  const S* __restrict__ In, const S* __restrict__ Small, S* __restrict__ Out,
                                                  int N, int RP, int backward) {
  const ItemView it = load_item(dtab, TS64, blockIdx.x);
  if (it.task < 0 || tasks[it.task].kind != MUX_ADAPTER_TUNING) return;
  const DevTask tk = tasks[it.task];
  const int n0 = blockIdx.y * 64;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const S* P = (const S*)(backward ? tk.A : tk.B);
  const int r = tk.rank;
  ZERO_ACC(acc);
  auto fa = [&](int m, int j) -> float {       // Hs / Gs are zero on padding rows by construction
    return m < it.nrows ? Store<S>::ld(Small, (size_t)(it.row0 + m) * RP + j) : 0.f;
  };
  auto fb = [&](int j, int n) -> float {
    if (n0 + n >= N) return 0.f;
    return backward ? Store<S>::ld(P, (size_t)(n0 + n) * r + j) : Store<S>::ld(P, (size_t)j * N + n0 + n);
  };
  tile64(fa, fb, r, acc);
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int m = ty * 4 + u, row = it.row0 + m;
    if (m >= it.nrows) continue;
    const bool ok = row_is_valid(dtab, row);
    const size_t zrow = (size_t)(tk.zrow0 + row - tk.row_begin);
    const size_t irow = backward ? (size_t)row : zrow, orow = backward ? zrow : (size_t)row;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int n = n0 + tx * 4 + v;
      if (n >= N) continue;
      Store<S>::st(Out, orow * N + n, ok ? Store<S>::ld(In, irow * N + n) + acc[u][v] : 0.f);
    }
  }
}

template <class S>
void steps(const CallCtx& c, unsigned which, const void* X, const void* dY, void* Y, void* dX, void* H, void* Z, void* G,
           int accumulate) {
  const int n_items = (int)c.st->items[TS64].size();
  const int M = c.st->n_tasks;
  if (n_items == 0) return;
  const bool lora = c.st->n_lora > 0, ia3 = c.st->n_ia3 > 0, tuning = c.st->n_tuning > 0;
  const bool only_tuning = (which & REF_ONLY_TUNING) != 0;
  const unsigned kinds = only_tuning ? KM_TUNING : (KM_LORA | KM_TUNING);
  const bool ranked = only_tuning ? tuning : (lora || tuning);
  if ((which & REF_DOWN) && lora)
    MUX_LAUNCH("ref_down", k_ref_down<S>, dim3(n_items), dim3(256), 0, c.stream, c.dtab, c.dtasks, (const S*)X, (S*)H, c.K, c.RP);
  if (which & REF_FWD)
    MUX_LAUNCH("ref_fwd", k_ref_fwd<S>, dim3(n_items, (c.N + 63) / 64), dim3(256), 0, c.stream, c.dtab, c.dtasks, (const S*)X,
                       (const S*)c.W, c.ldw, (const S*)H, (S*)Y, (S*)Z, c.K, c.N, c.RP);
  if ((which & REF_TUNE_DOWN) && tuning)
    MUX_LAUNCH("tune_down", k_tune_down<S>, dim3(n_items), dim3(256), 0, c.stream, c.dtab, c.dtasks, (const S*)Z, (S*)c.U2,
                       (S*)H, c.N, c.RP);
  if ((which & REF_TUNE_UP) && tuning)
    MUX_LAUNCH("tune_up", k_tune_add<S>, dim3(n_items, (c.N + 63) / 64), dim3(256), 0, c.stream, c.dtab, c.dtasks,
                       (const S*)Z, (const S*)H, (S*)Y, c.N, c.RP, 0);
  if ((which & REF_G) && ranked)     // on its own the kernel also zeroes the rows of the other kinds
    MUX_LAUNCH("ref_g", k_ref_g<S>, dim3(n_items), dim3(256), 0, c.stream, c.dtab, c.dtasks, (const S*)dY, (const S*)c.U2,
                       (S*)G, c.N, c.RP, kinds, only_tuning ? 0 : 1);
  if ((which & REF_TUNE_DZ) && tuning)
    MUX_LAUNCH("tune_dz", k_tune_add<S>, dim3(n_items, (c.N + 63) / 64), dim3(256), 0, c.stream, c.dtab, c.dtasks,
                       (const S*)dY, (const S*)G, (S*)c.dYs, c.N, c.RP, 1);
  if ((which & REF_DB) && ranked)
    MUX_LAUNCH("ref_db", k_ref_db<S>, dim3(M, (c.N + 63) / 64), dim3(256), 0, c.stream, c.dtab, c.dtasks, (const S*)dY,
                       (const S*)H, c.N, c.RP, accumulate, kinds);
  if ((which & REF_DA) && ranked) {
    const int rows = (tuning && c.N > c.K) ? c.N : c.K;
    MUX_LAUNCH("ref_da", k_ref_da<S>, dim3(M, (rows + 63) / 64), dim3(256), 0, c.stream, c.dtab, c.dtasks, (const S*)X,
                       (const S*)Z, (const S*)G, c.K, c.N, c.RP, accumulate, kinds);
  }
  if ((which & REF_DL) && ia3)
    MUX_LAUNCH("ref_dl", k_ref_dl<S>, dim3(M, (c.N + 255) / 256), dim3(256), 0, c.stream, c.dtab, c.dtasks, (const S*)dY,
                       (const S*)Z, c.N, accumulate);
  if ((which & REF_DX) && dX)
    MUX_LAUNCH("ref_dx", k_ref_dx<S>, dim3(n_items, (c.K + 63) / 64), dim3(256), 0, c.stream, c.dtab, c.dtasks,
                       (const S*)dY, (const S*)c.W, c.ldw, (const S*)G, (const S*)c.dYs, (S*)dX, c.K, c.N, c.RP);
}

}  // namespace

void ref_steps(const CallCtx& c, int dtype, unsigned which, const void* X, const void* dY, void* Y, void* dX, void* H,
               void* Z, void* G, int accumulate) {
  if (dtype == MUX_DT_F32)
    steps<float>(c, which, X, dY, Y, dX, H, Z, G, accumulate);
  else
    steps<bf16_t>(c, which, X, dY, Y, dX, H, Z, G, accumulate);
}

mux_status ref_forward(const CallCtx& c, int dtype, const void* X, void* Y, void* H, void* Z) {
  ref_steps(c, dtype, REF_DOWN | REF_FWD | REF_TUNE_DOWN | REF_TUNE_UP, X, nullptr, Y, nullptr, H, Z, nullptr, 0);
  return MUX_OK;
}

mux_status ref_backward(const CallCtx& c, int dtype, const void* X, const void* dY, const void* H, const void* Z, void* G,
                        void* dX, int accumulate) {
  ref_steps(c, dtype, REF_G | REF_TUNE_DZ | REF_DB | REF_DA | REF_DL | REF_DX, X, dY, nullptr, dX, (void*)H, (void*)Z, G,
            accumulate);
  return MUX_OK;
}

}  // namespace mux
