// Diff-Pruning kind (section 2.1, section 5: trainable values delta_t on a fixed sparse mask M_t over W):
//   forward   Y  = x (W + M_t * delta_t)      -> after the backbone GEMM wrote x W:      Y  += x (M_t * delta_t)
//   backward  dX = g (W + M_t * delta_t)^T    -> after the backbone GEMM wrote g W^T:    dX += g (M_t * delta_t)^T
//             d delta_t[e] = sum over the task's rows of x[i][k_e] * g[i][n_e]
//
// All three are sums over (entry, row) pairs with a handful of FMAs each, so what they cost is how x and g are
// fetched.  An entry needs one COLUMN of the task's rows of x (or g).  The rows of the Diff-Pruning tasks are
// therefore first copied in blocks of 64 rows with the block transposed -- T[block][column][64 rows], one aligned
// 128-byte (bf16) or 256-byte (fp32) line per (block, column) -- with the padding rows selected to zero.  After that
// every (entry, block) pair reads whole lines:
//   sparse update   a few lanes per output column and block with the 64 row sums between them, a plain loop over the
//                   entries of that column (column listing of the mask forward, row listing backward)
//   masked gradient a few lanes per entry, a plain loop over the task's blocks, two lines per block
// No barriers, no atomics; every sum has one owner and a fixed order.
#include <type_traits>

#include "mux_device_utils.h"

namespace mux {
namespace {

constexpr int TS64 = 0;  // index of the 64-row work list

// A line of a transposed block (64 rows of one column) is read by LPL neighbouring lanes, 16 bytes each, so that one
// load instruction of a wave covers 64 / LPL whole lines and no byte is fetched twice.
template <class S> struct Piece;
template <> struct Piece<float> {
  static constexpr int LPL = 16, RPL = 4;      // lanes per line, rows per lane
  static __device__ __forceinline__ void ld(const float* __restrict__ line, int sub, float (&x)[4]) {
    const float4 v = ((const float4*)line)[sub];
    x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w;
  }
};
template <> struct Piece<bf16_t> {
  static constexpr int LPL = 8, RPL = 8;
  static __device__ __forceinline__ void ld(const bf16_t* __restrict__ line, int sub, float (&x)[8]) {
    const uint4 v = ((const uint4*)line)[sub];
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int h = 0; h < 4; ++h) {
      x[2 * h] = __uint_as_float(w[h] << 16);
      x[2 * h + 1] = __uint_as_float(w[h] & 0xffff0000u);
    }
  }
};

// Block-transposed copy of the Diff-Pruning rows of In [T, C]:  Out[(block * C + c) * 64 + r] = In[row0 + r][c], zero
// for padding rows and for r beyond the item.  grid = (64-row items, ceil(C / 64), matrices): the launch copies one
// matrix or two (blockIdx.z picks; the backward copies dY and X together).  VEC: the rows of every In can be read
// 16 bytes at a time (C a multiple of 16 bytes' worth of elements, In 16-byte aligned).
template <class S>
struct TransposeSrc { const S* In; S* Out; int C; };
template <class S, bool VEC>
__global__ __launch_bounds__(256) void k_diff_transpose(const int32_t* __restrict__ dtab, const TaskRef tasks,
                                                        const TransposeSrc<S> s0, const TransposeSrc<S> s1) {
  constexpr int VE = 16 / (int)sizeof(S);          // elements per 16-byte vector
  __shared__ __align__(16) S tile[64][64 + VE];
  const S* __restrict__ In = blockIdx.z == 0 ? s0.In : s1.In;
  S* __restrict__ Out = blockIdx.z == 0 ? s0.Out : s1.Out;
  const int C = blockIdx.z == 0 ? s0.C : s1.C;
  if ((int)blockIdx.y * 64 >= C) return;
  const ItemView it = load_item(dtab, TS64, blockIdx.x);
  if (it.task < 0 || get_task_kind(tasks, it.task) != MUX_ADAPTER_DIFF) return;
  const DevTask tk = get_task(tasks, it.task);
  if (tk.at_off == 0) return;
  const int c0 = blockIdx.y * 64;
  {
    const int r = threadIdx.x >> 2, cq = (threadIdx.x & 3) * 16;
    const bool v = r < it.nrows && row_is_valid(dtab, it.row0 + r);
    __align__(16) S tmp[16];
    const S* src = In + (size_t)(it.row0 + r) * C + c0 + cq;
    if (VEC) {
#pragma unroll
      for (int i = 0; i < 16 / VE; ++i)
        ((uint4*)tmp)[i] = (v && c0 + cq + i * VE < C) ? ((const uint4*)src)[i] : uint4{0u, 0u, 0u, 0u};
    } else {
#pragma unroll
      for (int i = 0; i < 16; ++i) tmp[i] = (v && c0 + cq + i < C) ? src[i] : S(0);
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) tile[cq + i][r] = tmp[i];
  }
  __syncthreads();
  const int cc = threadIdx.x >> 2, rq = (threadIdx.x & 3) * 16;
  if (c0 + cc < C) {
    const size_t block = (size_t)(tk.zrow0 + it.row0 - tk.row_begin) >> 6;
    uint4* o = (uint4*)(Out + (block * (size_t)C + c0 + cc) * 64 + rq);
    const uint4* t = (const uint4*)&tile[cc][rq];
#pragma unroll
    for (int i = 0; i < 16 / VE; ++i) o[i] = t[i];
  }
}

// Sparse update of one 64-row item: Out[row][c] += sum over the entries (j, v) of output column c of Tin[block][j][row] * v.
// LPL lanes share one output column, each with RPL of the 64 row sums; grid = items x ceil(Cout / (256 / LPL))
// workgroups, the column blocks of one item next to each other so that they find the item's block in the L2 caches.
template <class S>
__global__ __launch_bounds__(256) void k_diff_apply(const int32_t* __restrict__ dtab, const TaskRef tasks,
                                                    const S* __restrict__ Tin, S* __restrict__ Out, int Cin, int Cout,
                                                    int backward) {
  constexpr int LPL = Piece<S>::LPL, RPL = Piece<S>::RPL, CPW = 256 / LPL;
  const int ncb = (Cout + CPW - 1) / CPW;
  const ItemView it = load_item(dtab, TS64, blockIdx.x / ncb);
  if (it.task < 0 || it.nvalid == 0 || get_task_kind(tasks, it.task) != MUX_ADAPTER_DIFF) return;
  const DevTask tk = get_task(tasks, it.task);
  const int sub = threadIdx.x % LPL;
  const int c = (blockIdx.x % ncb) * CPW + threadIdx.x / LPL;
  if (tk.at_off == 0 || c >= Cout) return;
  const S* val = (const S*)tk.A;
  const int32_t* ptr = backward ? (const int32_t*)tk.B : (const int32_t*)tk.dB;       // row_ptr / col_ptr
  const int32_t* ent = backward ? (const int32_t*)tk.L : (const int32_t*)tk.dL;       // col_idx / (k, e) pairs
  const int e0 = ptr[c], e1 = ptr[c + 1];
  if (e0 >= e1) return;
  const size_t block = (size_t)(tk.zrow0 + it.row0 - tk.row_begin) >> 6;
  const S* base = Tin + block * (size_t)Cin * 64;
  float acc[RPL];
#pragma unroll
  for (int r = 0; r < RPL; ++r) acc[r] = 0.f;
#pragma unroll 4
  for (int e = e0; e < e1; ++e) {
    const int j = backward ? ent[e] : ent[2 * e];
    const float v = Store<S>::ld(val, (size_t)(backward ? e : ent[2 * e + 1]));
    float x[RPL];
    Piece<S>::ld(base + (size_t)j * 64, sub, x);
#pragma unroll
    for (int r = 0; r < RPL; ++r) acc[r] = fmaf(x[r], v, acc[r]);
  }
#pragma unroll
  for (int r = 0; r < RPL; ++r) {
    const int m = sub * RPL + r;
    if (m < it.nrows && row_is_valid(dtab, it.row0 + m)) {
      const size_t o = (size_t)(it.row0 + m) * Cout + c;
      Store<S>::st(Out, o, Store<S>::ld(Out, o) + acc[r]);
    }
  }
}

// d delta[e] = sum over the task's 64-row blocks of <Xt[block][k_e][.], Gt[block][n_e][.]>.  A wave owns 64 consecutive
// entries; LPL lanes share one entry at a time (a wave's load covers 64 / LPL whole lines), each lane summing its RPL
// rows over the blocks in ascending order; the LPL partial sums are then added in a fixed tree.
// grid = (tasks, ceil(max nnz / 256)).
template <class S>
__global__ __launch_bounds__(256) void k_diff_grad(const TaskRef tasks, const S* __restrict__ Xt,
                                                   const S* __restrict__ Gt, int K, int N, int accumulate) {
  constexpr int LPL = Piece<S>::LPL, RPL = Piece<S>::RPL, EPI = 64 / LPL;    // EPI: entries per load instruction
  const DevTask tk = get_task(tasks, (int)blockIdx.x);
  if (tk.kind != MUX_ADAPTER_DIFF || tk.dA == nullptr) return;
  const int lane = threadIdx.x & 63;
  const int wave_e0 = blockIdx.y * 256 + (threadIdx.x & ~63);
  if (wave_e0 >= tk.at_off) return;                       // whole wave
  const int e_own = wave_e0 + lane;
  int k_own = 0, n_own = 0;                               // lanes past the last entry work on entry (0, 0), unused
  if (e_own < tk.at_off) {
    const int32_t* row_ptr = (const int32_t*)tk.B;
    int lo = 0, hi = K;                                   // the row k with row_ptr[k] <= e < row_ptr[k+1]
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (row_ptr[mid] <= e_own) lo = mid; else hi = mid;
    }
    k_own = lo;
    n_own = ((const int32_t*)tk.L)[e_own];
  }
  const int sub = lane % LPL, grp = lane / LPL;
  int ks[LPL], ns[LPL];
#pragma unroll
  for (int i = 0; i < LPL; ++i) {                         // pass i works on entry wave_e0 + i * EPI + grp
    ks[i] = __shfl(k_own, i * EPI + grp);
    ns[i] = __shfl(n_own, i * EPI + grp);
  }
  float acc[LPL];
#pragma unroll
  for (int i = 0; i < LPL; ++i) acc[i] = 0.f;
  const int nb = (tk.row_count + 63) >> 6;
  const size_t b0 = (size_t)tk.zrow0 >> 6;
  for (int b = 0; b < nb; ++b) {
    const S* xb = Xt + (b0 + b) * (size_t)K * 64;
    const S* gb = Gt + (b0 + b) * (size_t)N * 64;
#pragma unroll
    for (int i = 0; i < LPL; ++i) {
      float x[RPL], g[RPL];
      Piece<S>::ld(xb + (size_t)ks[i] * 64, sub, x);
      Piece<S>::ld(gb + (size_t)ns[i] * 64, sub, g);
#pragma unroll
      for (int r = 0; r < RPL; ++r) acc[i] = fmaf(x[r], g[r], acc[i]);
    }
  }
  float mine = 0.f;
#pragma unroll
  for (int i = 0; i < LPL; ++i) {
    float v = acc[i];
#pragma unroll
    for (int m = 1; m < LPL; m <<= 1) v += __shfl_xor(v, m);
    if (sub == i) mine = v;
  }
  const int e_w = wave_e0 + sub * EPI + grp;              // the lane with sub == i writes the entry of pass i
  if (e_w < tk.at_off) tk.dA[e_w] = accumulate ? tk.dA[e_w] + mine : mine;
}

// The masked gradient by blocks of the mask (bf16).  A workgroup owns the entries of one GBK x GBN block of one task's mask
// and walks the task's 64-row blocks: the GBK lines of Xt and the GBN lines of Gt of a row block (two contiguous
// stretches of the transposed copies) are staged in LDS once and serve all entries of the mask block, so a line is
// fetched once per mask block instead of once per entry; the loads of the next row block are in flight (in registers)
// while the entries are summed.  The entries of the block come from the row listing: thread i looks up, by two binary
// searches in row k0 + i, the stretch of its entries whose column lies in the block; a prefix sum over the rows numbers
// them, and a thread holds G_EPT of them per pass (more entries: more passes over the row blocks).  Every entry has one
// owner and a fixed order of summation (row blocks ascending, rows ascending).  grid = (mask blocks, tasks).
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
constexpr int GBK = 512, GBN = 256;     // rows and columns of a mask block
constexpr int GP = 72;                  // LDS pitch (elements) of a line of 64 rows: 144 bytes
constexpr int G_EPT = 2;                // entries per thread and pass
constexpr int G_THREADS = 1024;
constexpr int G_SMEM = (GBK + GBN) * GP * 2 + (GBK + 1) * 4 + GBK * 4;
__global__ __launch_bounds__(G_THREADS) void k_diff_grad_tiled(const TaskRef tasks, const bf16_t* __restrict__ Xt,
                                                               const bf16_t* __restrict__ Gt, int K, int N, int accumulate) {
  extern __shared__ __align__(16) unsigned char g_smem[];
  bf16_t* Xs = (bf16_t*)g_smem;
  bf16_t* Gs = Xs + GBK * GP;
  int* offs = (int*)(Gs + GBN * GP);    // GBK + 1: entries of the block before row i
  int* start = offs + GBK + 1;          // GBK: index (in the row listing) of row i's first entry inside the block
  const DevTask tk = get_task(tasks, (int)blockIdx.y);
  if (tk.kind != MUX_ADAPTER_DIFF || tk.dA == nullptr || tk.at_off == 0) return;
  // Workgroups go to the eight XCDs round-robin: XCD x takes a contiguous stretch of the blocks in row-major order, so
  // that the blocks running on it at one time share their lines of Xt in its L2.
  const int n_nb = (N + GBN - 1) / GBN, n_blocks = ((K + GBK - 1) / GBK) * n_nb;
  const int per_xcd = (n_blocks + 7) / 8;
  const int block = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
  if ((int)(blockIdx.x >> 3) >= per_xcd || block >= n_blocks) return;
  const int k0 = (block / n_nb) * GBK, n0 = (block % n_nb) * GBN;
  const int tid = threadIdx.x;
  const int32_t* row_ptr = (const int32_t*)tk.B;
  const int32_t* col_idx = (const int32_t*)tk.L;
  if (tid < GBK) {
    int my_start = 0, my_cnt = 0;
    if (k0 + tid < K) {
      int a = row_ptr[k0 + tid], b = row_ptr[k0 + tid + 1];
      const int hi = b;
      while (a < b) { const int m = (a + b) >> 1; if (col_idx[m] < n0) a = m + 1; else b = m; }
      my_start = a;
      b = hi;
      while (a < b) { const int m = (a + b) >> 1; if (col_idx[m] < n0 + GBN) a = m + 1; else b = m; }
      my_cnt = a - my_start;
    }
    start[tid] = my_start;
    offs[tid + 1] = my_cnt;             // inclusive prefix sums in offs[1 .. GBK]
    if (tid == 0) offs[0] = 0;
  }
  __syncthreads();
  for (int d = 1; d < GBK; d <<= 1) {
    const int v = (tid < GBK && tid >= d) ? offs[tid + 1 - d] : 0;
    __syncthreads();
    if (tid < GBK) offs[tid + 1] += v;
    __syncthreads();
  }
  const int total = offs[GBK];
  if (total == 0) return;               // whole workgroup
  const int lx = K - k0 < GBK ? K - k0 : GBK, lg = N - n0 < GBN ? N - n0 : GBN;   // lines of this block that exist
  const int nbk = (tk.row_count + 63) >> 6;
  const size_t b0 = (size_t)tk.zrow0 >> 6;
  constexpr int PPTX = GBK * 8 / G_THREADS, PPTG = GBN * 8 / G_THREADS;   // 16-byte pieces per thread of either operand
  // piece q of this thread: index tid + q * G_THREADS of the stretch (a line that does not exist reads line 0 instead
  // and is never staged)
  const int lx8 = lx * 8, lg8 = lg * 8;
  for (int f0 = 0; f0 < total; f0 += G_THREADS * G_EPT) {
    int kl[G_EPT], nl[G_EPT], ee[G_EPT];
    float acc[G_EPT];
#pragma unroll
    for (int i = 0; i < G_EPT; ++i) {
      const int f = f0 + i * G_THREADS + tid;
      acc[i] = 0.f;
      kl[i] = 0; nl[i] = 0; ee[i] = -1;
      if (f < total) {
        int lo = 0, hi = GBK;                       // the row r with offs[r] <= f < offs[r + 1]
        while (hi - lo > 1) { const int m = (lo + hi) >> 1; if (offs[m] <= f) lo = m; else hi = m; }
        kl[i] = lo;
        ee[i] = start[lo] + (f - offs[lo]);
        nl[i] = col_idx[ee[i]] - n0;
      }
    }
    // two sets of staging registers: the lines of row blocks b + 1 and b + 2 are in flight while block b is summed
    u32x4 rx0[PPTX], rg0[PPTG], rx1[PPTX], rg1[PPTG];
#define DIFF_FETCH(RX, RG, B)                                                                  \
    if ((B) < nbk) {                                                                             \
      const u32x4* xs_ = (const u32x4*)(Xt + ((b0 + (B)) * (size_t)K + k0) * 64);                \
      const u32x4* gs_ = (const u32x4*)(Gt + ((b0 + (B)) * (size_t)N + n0) * 64);                \
      _Pragma("unroll") for (int q = 0; q < PPTX; ++q) {                                         \
        const int p_ = tid + q * G_THREADS;                                                      \
        RX[q] = xs_[p_ < lx8 ? p_ : 0];                                                          \
      }                                                                                          \
      _Pragma("unroll") for (int q = 0; q < PPTG; ++q) {                                         \
        const int p_ = tid + q * G_THREADS;                                                      \
        RG[q] = gs_[p_ < lg8 ? p_ : 0];                                                          \
      }                                                                                          \
    }
#define DIFF_STEP(RX, RG, B)                                                                   \
    {                                                                                            \
      __syncthreads(); /* every read of the previous row block is done */                        \
      _Pragma("unroll") for (int q = 0; q < PPTX; ++q) {                                         \
        const int p_ = tid + q * G_THREADS;                                                      \
        if (p_ < lx8) *(u32x4*)(Xs + (p_ >> 3) * GP + (p_ & 7) * 8) = RX[q];                     \
      }                                                                                          \
      _Pragma("unroll") for (int q = 0; q < PPTG; ++q) {                                         \
        const int p_ = tid + q * G_THREADS;                                                      \
        if (p_ < lg8) *(u32x4*)(Gs + (p_ >> 3) * GP + (p_ & 7) * 8) = RG[q];                     \
      }                                                                                          \
      __syncthreads();                                                                           \
      DIFF_FETCH(RX, RG, (B) + 2)                                                                \
      _Pragma("unroll") for (int i = 0; i < G_EPT; ++i) {                                        \
        if (ee[i] < 0) continue;                                                                 \
        const u32x4* xl = (const u32x4*)(Xs + kl[i] * GP);                                       \
        const u32x4* gl = (const u32x4*)(Gs + nl[i] * GP);                                       \
        float a = acc[i];                                                                        \
        _Pragma("unroll 2") for (int j = 0; j < 8; ++j) {                                        \
          const u32x4 xv = xl[j], gv = gl[j];                                                    \
          _Pragma("unroll") for (int h = 0; h < 4; ++h) {                                        \
            a = fmaf(__uint_as_float(xv[h] << 16), __uint_as_float(gv[h] << 16), a);             \
            a = fmaf(__uint_as_float(xv[h] & 0xffff0000u), __uint_as_float(gv[h] & 0xffff0000u), a); \
          }                                                                                      \
        }                                                                                        \
        acc[i] = a;                                                                              \
      }                                                                                          \
    }
    DIFF_FETCH(rx0, rg0, 0)
    DIFF_FETCH(rx1, rg1, 1)
    for (int b = 0; b < nbk; b += 2) {
      DIFF_STEP(rx0, rg0, b)
      if (b + 1 < nbk) DIFF_STEP(rx1, rg1, b + 1)
    }
#undef DIFF_FETCH
#undef DIFF_STEP
#pragma unroll
    for (int i = 0; i < G_EPT; ++i)
      if (ee[i] >= 0) tk.dA[ee[i]] = accumulate ? tk.dA[ee[i]] + acc[i] : acc[i];
  }
}

// Merged weight of one Diff-Pruning task (bf16): Wm = W + M_t * delta_t, rounded once.  A workgroup copies MR rows of W
// (16-byte pieces; N a multiple of 8, W and Wm 16-byte aligned with the same row pitch) and then, behind a workgroup
// barrier, rewrites the masked entries of those rows -- the entries of consecutive rows are consecutive in the row
// listing.  grid = (ceil(K / MR), tasks).  (Reading W once for all tasks in one workgroup was slower: fewer
// workgroups, 82 against 61 us for two tasks.)
constexpr int MR = 8;
__global__ __launch_bounds__(256) void k_diff_merge(const TaskRef tasks, const bf16_t* __restrict__ W,
                                                    bf16_t* __restrict__ Wm_all, int64_t stride, int K, int N, int64_t ldw) {
  const DevTask tk = get_task(tasks, (int)blockIdx.y);
  if (tk.kind != MUX_ADAPTER_DIFF || tk.rank < 0) return;
  bf16_t* Wm = Wm_all + (size_t)tk.rank * (size_t)stride;
  const int k0 = blockIdx.x * MR;
  const int rows = K - k0 < MR ? K - k0 : MR;
  const int ppr = N / 8;                                  // 16-byte pieces per row
  const int n_pieces = rows * ppr;
  constexpr int UNR = 4;
  for (int e0 = threadIdx.x; e0 < n_pieces; e0 += 256 * UNR) {
    uint4 v[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int e = e0 + 256 * u;
      if (e < n_pieces) v[u] = *(const uint4*)(W + (size_t)(k0 + e / ppr) * ldw + (e % ppr) * 8);
    }
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int e = e0 + 256 * u;
      if (e < n_pieces) *(uint4*)(Wm + (size_t)(k0 + e / ppr) * ldw + (e % ppr) * 8) = v[u];
    }
  }
  __syncthreads();                                        // the copies of these rows are ordered before the entries' stores
  const int32_t* row_ptr = (const int32_t*)tk.B;
  const int32_t* col_idx = (const int32_t*)tk.L;
  const bf16_t* val = (const bf16_t*)tk.A;
  const int e_begin = row_ptr[k0], e_end = row_ptr[k0 + rows];
  for (int e = e_begin + threadIdx.x; e < e_end; e += 256) {
    int k = k0;
    while (k + 1 < k0 + rows && row_ptr[k + 1] <= e) ++k;
    const size_t o = (size_t)k * ldw + col_idx[e];
    Store<bf16_t>::st(Wm, o, Store<bf16_t>::ld(W, o) + Store<bf16_t>::ld(val, (size_t)e));
  }
}

constexpr int kTiledMinBlocks = 48;
// the tiled kernel's LDS is above the default limit of a launch: raised once per process
bool tiled_grad_ready() {
  static const bool ok = hipFuncSetAttribute((const void*)k_diff_grad_tiled, hipFuncAttributeMaxDynamicSharedMemorySize, G_SMEM) == hipSuccess;
  return ok;
}

// One matrix (In1 null) or two in one launch.
template <class S>
void transpose(const CallCtx& c, const char* name, const void* In0, void* Out0, int C0, const void* In1 = nullptr,
               void* Out1 = nullptr, int C1 = 0) {
  const int n_items = (int)c.st->items[TS64].size();
  constexpr int VE = 16 / (int)sizeof(S);
  const bool vec = C0 % VE == 0 && ((uintptr_t)In0 & 15) == 0 && (!In1 || (C1 % VE == 0 && ((uintptr_t)In1 & 15) == 0));
  const TransposeSrc<S> s0{(const S*)In0, (S*)Out0, C0}, s1{(const S*)In1, (S*)Out1, C1};
  const int cmax = C0 > C1 ? C0 : C1;
  const dim3 grid(n_items, (cmax + 63) / 64, In1 ? 2 : 1);
  if (vec) MUX_LAUNCH(name, (k_diff_transpose<S, true>), grid, dim3(256), 0, c.stream, c.dtab, *c.tref, s0, s1);
  else MUX_LAUNCH(name, (k_diff_transpose<S, false>), grid, dim3(256), 0, c.stream, c.dtab, *c.tref, s0, s1);
}

template <class S>
void forward(const CallCtx& c, const void* X, void* Y) {
  if (c.diffW || c.diffPack) return;         // the backbone product read W + M_t * delta_t for these rows
  const int n_items = (int)c.st->items[TS64].size();
  transpose<S>(c, "diff_xt", X, c.diffT[0], c.K);
  constexpr int CPW = 256 / Piece<S>::LPL;
  MUX_LAUNCH("diff_fwd", k_diff_apply<S>, dim3((unsigned)n_items * (unsigned)((c.N + CPW - 1) / CPW)), dim3(256), 0, c.stream, c.dtab, *c.tref,
             (const S*)c.diffT[0], (S*)Y, c.K, c.N, 0);
}

template <class S>
void backward(const CallCtx& c, const void* X, const void* dY, void* dX, int accumulate) {
  const int n_items = (int)c.st->items[TS64].size();
  transpose<S>(c, "diff_gxt", dY, c.diffT[1], c.N, X, c.diffT[0], c.K);     // both copies the gradient needs
  if (dX && !c.diffW && !c.diffPack)         // else the backbone product read W + M_t * delta_t for these rows
    MUX_LAUNCH("diff_bwd", k_diff_apply<S>, dim3((unsigned)n_items * (unsigned)((c.K + (256 / Piece<S>::LPL) - 1) / (256 / Piece<S>::LPL))), dim3(256), 0, c.stream, c.dtab, *c.tref,
               (const S*)c.diffT[1], (S*)dX, c.N, c.K, 1);
  // by blocks of the mask where there are enough of them to occupy the compute units (bf16), else by entries
  const int blocks = ((c.K + GBK - 1) / GBK) * ((c.N + GBN - 1) / GBN);
  if (std::is_same<S, bf16_t>::value && blocks * c.st->n_diff >= kTiledMinBlocks && tiled_grad_ready()) {
    MUX_LAUNCH("diff_grad", k_diff_grad_tiled, dim3((unsigned)(8 * ((blocks + 7) / 8)), (unsigned)c.st->n_tasks), dim3(G_THREADS), G_SMEM, c.stream,
               *c.tref, (const bf16_t*)c.diffT[0], (const bf16_t*)c.diffT[1], c.K, c.N, accumulate);
    return;
  }
  MUX_LAUNCH("diff_grad", k_diff_grad<S>, dim3(c.st->n_tasks, (c.diff_max_nnz + 255) / 256), dim3(256), 0, c.stream,
             *c.tref, (const S*)c.diffT[0], (const S*)c.diffT[1], c.K, c.N, accumulate);
}

}  // namespace

size_t diff_transposed_bytes(int K, int N, const mux_segtab* st, size_t esz) {
  return st->n_diff > 0 ? align256((size_t)st->d_rows * (size_t)(K > N ? K : N) * esz) : 0;
}

// The entries of every Diff-Pruning mask in the order of the listing by tiles of this call's direction (tk.dB, tk.dL),
// with their values: (position inside the bucket's tile) << 16 | bf16(delta).  A task's list starts at element tk.rank
// of `out`.  grid = (tasks, ceil(max nnz / 256)).
namespace {
__global__ __launch_bounds__(256) void k_diff_pack(const TaskRef tasks, uint32_t* __restrict__ out, int backward) {
  const DevTask tk = get_task(tasks, (int)blockIdx.x);
  if (tk.kind != MUX_ADAPTER_DIFF || tk.rank < 0) return;
  const int pos = blockIdx.y * 256 + threadIdx.x;
  if (pos >= tk.at_off) return;
  const bf16_t* val = (const bf16_t*)tk.A;
  const int2 ent = ((const int2*)tk.dL)[pos];        // (number of the entry, position inside the tile)
  out[(size_t)tk.rank + pos] = (uint32_t)ent.y << 16 | (uint32_t)val[ent.x];
}
}  // namespace

void diff_pack(const CallCtx& c, bool backward) {
  if (!c.diffPack || c.diff_max_nnz == 0) return;
  MUX_LAUNCH("diff_pack", k_diff_pack, dim3((unsigned)c.st->n_tasks, (unsigned)((c.diff_max_nnz + 255) / 256)), dim3(256), 0,
             c.stream, *c.tref, (uint32_t*)c.diffPack, backward ? 1 : 0);
}

size_t diff_merged_bytes(int K, int64_t ldw) { return align256((size_t)K * (size_t)ldw * 2); }

// The merged weights of the Diff-Pruning tasks that have entries, when the call has room for them (matrix-core path):
// W in and one copy out per such task.
void diff_merge(const CallCtx& c, int slots) {
  if (!c.diffW || slots <= 0) return;
  prof_note_bytes(4.0 * c.K * c.N * slots);
  MUX_LAUNCH("diff_merge", k_diff_merge, dim3((unsigned)((c.K + MR - 1) / MR), (unsigned)c.st->n_tasks), dim3(256), 0, c.stream,
             *c.tref, (const bf16_t*)c.W, (bf16_t*)c.diffW, c.diffW_stride, c.K, c.N, c.ldw);
}

void diff_forward(const CallCtx& c, int dtype, const void* X, void* Y) {
  if (c.st->n_diff == 0 || c.diff_max_nnz == 0 || c.st->items[TS64].empty()) return;
  if (dtype == MUX_DT_F32) forward<float>(c, X, Y); else forward<bf16_t>(c, X, Y);
}

void diff_backward(const CallCtx& c, int dtype, const void* X, const void* dY, void* dX, int accumulate) {
  if (c.st->n_diff == 0 || c.diff_max_nnz == 0 || c.st->items[TS64].empty()) return;
  if (dtype == MUX_DT_F32) backward<float>(c, X, dY, dX, accumulate); else backward<bf16_t>(c, X, dY, dX, accumulate);
}

}  // namespace mux
