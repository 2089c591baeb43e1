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
      if (kind == MUX_ADAPTER_IA3_OUT) {
        if (Z) Store<S>::st(Z, (size_t)(tk.zrow0 + row - tk.row_begin) * N + n, ok ? y : 0.f);
        y *= Store<S>::ld((const S*)tk.L, n);
      }
      Store<S>::st(Y, (size_t)row * N + n, ok ? y : 0.f);
    }
  }
}

// S4a: Gs = s_t * (g B_t^T) for LoRA rows, 0 elsewhere.  grid.x = items.
template <class S>
__global__ __launch_bounds__(256) void k_ref_g(const int32_t* __restrict__ dtab, const DevTask* __restrict__ tasks,
                                               const S* __restrict__ dY, S* __restrict__ G, int N, int RP) {
  const ItemView it = load_item(dtab, TS64, blockIdx.x);
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  ZERO_ACC(acc);
  float scale = 0.f;
  if (it.task >= 0 && tasks[it.task].kind == MUX_ADAPTER_LORA) {
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
      if (j < RP) Store<S>::st(G, (size_t)row * RP + j, ok ? scale * acc[u][v] : 0.f);
    }
  }
}

// S5: dX = mask * (g W^T + Gs A_t^T)   or   mask * ((g * l_t) W^T).  grid = (items, ceil(K/64)).
template <class S>
__global__ __launch_bounds__(256) void k_ref_dx(const int32_t* __restrict__ dtab, const DevTask* __restrict__ tasks,
                                                const S* __restrict__ dY, const S* __restrict__ W, int64_t ldw,
                                                const S* __restrict__ G, S* __restrict__ dX, int K, int N, int RP) {
  const ItemView it = load_item(dtab, TS64, blockIdx.x);
  const int k0 = blockIdx.y * 64;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  ZERO_ACC(acc);
  if (it.task >= 0 && it.nvalid > 0) {
    const DevTask tk = tasks[it.task];
    const S* L = tk.kind == MUX_ADAPTER_IA3_OUT ? (const S*)tk.L : nullptr;
    auto fa = [&](int m, int n) -> float {
      const int row = it.row0 + m;
      if (!(m < it.nrows && row_is_valid(dtab, row))) return 0.f;
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
                                                int accumulate) {
  const DevTask tk = tasks[blockIdx.x];
  if (tk.kind != MUX_ADAPTER_LORA || tk.dB == nullptr) return;
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

// S6a: dA_t[k][j] = sum_{rows of t} x[i][k] Gs[i][j].  grid = (tasks, ceil(K/64)).
template <class S>
__global__ __launch_bounds__(256) void k_ref_da(const int32_t* __restrict__ dtab, const DevTask* __restrict__ tasks,
                                                const S* __restrict__ X, const S* __restrict__ G, int K, int RP,
                                                int accumulate) {
  const DevTask tk = tasks[blockIdx.x];
  if (tk.kind != MUX_ADAPTER_LORA || tk.dA == nullptr) return;
  const int k0 = blockIdx.y * 64;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int r = tk.rank;
  ZERO_ACC(acc);
  auto fa = [&](int kk, int i) -> float {
    const int row = tk.row_begin + i;
    return (k0 + kk < K && row_is_valid(dtab, row)) ? Store<S>::ld(X, (size_t)row * K + k0 + kk) : 0.f;
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

template <class S>
void steps(const CallCtx& c, unsigned which, const void* X, const void* dY, void* Y, void* dX, void* H, void* Z, void* G,
           int accumulate) {
  const int n_items = (int)c.st->items[TS64].size();
  const int M = c.st->n_tasks;
  if (n_items == 0) return;
  const bool lora = c.st->n_lora > 0, ia3 = c.st->n_ia3 > 0;
  if ((which & REF_DOWN) && lora)
    MUX_LAUNCH("ref_down", k_ref_down<S>, dim3(n_items), dim3(256), 0, c.stream, c.dtab, c.dtasks, (const S*)X, (S*)H, c.K, c.RP);
  if (which & REF_FWD)
    MUX_LAUNCH("ref_fwd", k_ref_fwd<S>, dim3(n_items, (c.N + 63) / 64), dim3(256), 0, c.stream, c.dtab, c.dtasks, (const S*)X,
                       (const S*)c.W, c.ldw, (const S*)H, (S*)Y, (S*)Z, c.K, c.N, c.RP);
  if ((which & REF_G) && lora)
    MUX_LAUNCH("ref_g", k_ref_g<S>, dim3(n_items), dim3(256), 0, c.stream, c.dtab, c.dtasks, (const S*)dY, (S*)G, c.N, c.RP);
  if ((which & REF_DB) && lora)
    MUX_LAUNCH("ref_db", k_ref_db<S>, dim3(M, (c.N + 63) / 64), dim3(256), 0, c.stream, c.dtab, c.dtasks, (const S*)dY,
                       (const S*)H, c.N, c.RP, accumulate);
  if ((which & REF_DA) && lora)
    MUX_LAUNCH("ref_da", k_ref_da<S>, dim3(M, (c.K + 63) / 64), dim3(256), 0, c.stream, c.dtab, c.dtasks, (const S*)X,
                       (const S*)G, c.K, c.RP, accumulate);
  if ((which & REF_DL) && ia3)
    MUX_LAUNCH("ref_dl", k_ref_dl<S>, dim3(M, (c.N + 255) / 256), dim3(256), 0, c.stream, c.dtab, c.dtasks, (const S*)dY,
                       (const S*)Z, c.N, accumulate);
  if ((which & REF_DX) && dX)
    MUX_LAUNCH("ref_dx", k_ref_dx<S>, dim3(n_items, (c.K + 63) / 64), dim3(256), 0, c.stream, c.dtab, c.dtasks,
                       (const S*)dY, (const S*)c.W, c.ldw, (const S*)G, (S*)dX, c.K, c.N, c.RP);
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
  ref_steps(c, dtype, REF_DOWN | REF_FWD, X, nullptr, Y, nullptr, H, Z, nullptr, 0);
  return MUX_OK;
}

mux_status ref_backward(const CallCtx& c, int dtype, const void* X, const void* dY, const void* H, const void* Z, void* G,
                        void* dX, int accumulate) {
  ref_steps(c, dtype, REF_G | REF_DB | REF_DA | REF_DL | REF_DX, X, dY, nullptr, dX, (void*)H, (void*)Z, G, accumulate);
  return MUX_OK;
}

}  // namespace mux
