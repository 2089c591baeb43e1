// Entry points of the layer: argument checks, buffer carving, kernel sequencing.
#include <cstring>
#include <mutex>
#include <string>

#include "mux_device_utils.h"

namespace mux {

// Launch-argument block for k_fill_tasks: adapter pointers of up to 16 tasks.
struct TaskPtrArgs {
  const void* A[16];
  const void* B[16];
  const void* L[16];
  float* dA[16];
  float* dB[16];
  float* dL[16];
  int64_t at_off[16];
};

// Block 0 writes the per-call task table.  With pack_at, blocks 1.. also write A_t^T [round_up(r,16)][K] (zero rows
// beyond r) for the forward's down-projection: block b handles 64 k-values of task base + (b-1)/ceil(K/64), reading
// the pointers from the launch arguments (not from the table block 0 is writing).
__global__ __launch_bounds__(256) void k_fill_tasks(const int32_t* __restrict__ dtab, DevTask* __restrict__ out, TaskPtrArgs p,
                                                     int base, int count, uint16_t* __restrict__ pack_at, int Kin, int Nout,
                                                     int only_tuning) {
  if (blockIdx.x == 0) {
    const int i = threadIdx.x;
    if (i >= count) return;
    const int32_t* te = dtab + dtab[DH_OFF_TASKS] + (base + i) * DT_WORDS;
    DevTask d;
    d.A = p.A[i]; d.B = p.B[i]; d.L = p.L[i];
    d.dA = p.dA[i]; d.dB = p.dB[i]; d.dL = p.dL[i];
    d.scale = __int_as_float(te[DT_SCALE_BITS]);
    d.kind = te[DT_KIND];
    d.rank = te[DT_RANK];
    d.row_begin = te[DT_ROW_BEGIN];
    d.row_count = te[DT_ROW_COUNT];
    d.zrow0 = te[DT_ZROW0];
    d.at_off = p.at_off[i];
    out[base + i] = d;
    return;
  }
  __shared__ uint16_t t[64][66];
  const int nkb = ((Kin > Nout ? Kin : Nout) + 63) / 64;
  const int i = (blockIdx.x - 1) / nkb, k0 = ((blockIdx.x - 1) % nkb) * 64;
  if (i >= count) return;
  const int32_t* te = dtab + dtab[DH_OFF_TASKS] + (base + i) * DT_WORDS;
  // LORA: A_t [K, r]; TUNING: D_t [N, r] (in the same slot); both go out as [round_up(r,16)][rows]
  if (te[DT_KIND] != MUX_ADAPTER_LORA && te[DT_KIND] != MUX_ADAPTER_TUNING) return;
  if (only_tuning && te[DT_KIND] != MUX_ADAPTER_TUNING) return;     // the backward pass needs D_t^T only
  const int K = te[DT_KIND] == MUX_ADAPTER_LORA ? Kin : Nout;
  if (k0 >= K) return;
  const int r = te[DT_RANK], rp = (r + 15) & ~15;
  const uint16_t* A = (const uint16_t*)p.A[i];
  for (int e = threadIdx.x; e < 64 * rp; e += 256) {
    const int kk = e / rp, j = e % rp;
    t[j][kk] = (j < r && k0 + kk < K) ? A[(size_t)(k0 + kk) * r + j] : (uint16_t)0;
  }
  __syncthreads();
  uint16_t* dst = pack_at + p.at_off[i];
  for (int e = threadIdx.x; e < 64 * rp; e += 256) {
    const int j = e >> 6, kk = e & 63;
    if (k0 + kk < K) dst[(size_t)j * K + k0 + kk] = t[j][kk];
  }
}

// A table without rows: every task's gradient is zero.  grid = (tasks, blocks over the largest gradient).
__global__ __launch_bounds__(256) void k_zero_grads(const DevTask* __restrict__ tasks, int K, int N) {
  const DevTask tk = tasks[blockIdx.x];
  const size_t e = (size_t)blockIdx.y * 256 + threadIdx.x;
  if (tk.kind == MUX_ADAPTER_LORA || tk.kind == MUX_ADAPTER_TUNING) {
    if (tk.dA && e < (size_t)(tk.kind == MUX_ADAPTER_LORA ? K : N) * tk.rank) tk.dA[e] = 0.f;
    if (tk.dB && e < (size_t)tk.rank * N) tk.dB[e] = 0.f;
  } else if (tk.kind == MUX_ADAPTER_IA3_OUT) {
    if (tk.dL && e < (size_t)N) tk.dL[e] = 0.f;
  } else if (tk.kind == MUX_ADAPTER_DIFF) {
    if (tk.dA && e < (size_t)tk.at_off) tk.dA[e] = 0.f;
  }
}

namespace {

struct Layout {
  size_t esz;          // bytes per stored element
  int RP;              // H / G row pitch in elements
  size_t h_bytes, z_bytes, u2_bytes, saved_bytes;
  size_t tasks_bytes, g_bytes, at_bytes, dys_bytes, part_bytes, dt_bytes, ws_bytes;
};

Layout make_layout(const mux_layer_desc* L, const mux_segtab* st) {
  Layout o{};
  o.esz = L->dtype == MUX_DT_F32 ? 4 : 2;
  o.RP = rank_pitch(st);
  o.h_bytes = align256((size_t)st->T * o.RP * o.esz);
  o.z_bytes = align256((size_t)st->z_rows * (size_t)L->N * o.esz);
  o.u2_bytes = st->n_tuning > 0 ? o.h_bytes : 0;
  o.saved_bytes = o.h_bytes + o.z_bytes + o.u2_bytes;
  o.tasks_bytes = align256((size_t)st->n_tasks * sizeof(DevTask));
  o.g_bytes = o.h_bytes;
  size_t at_elems = 0;
  for (const HostTask& ht : st->tasks)
    if (ht.kind == MUX_ADAPTER_LORA) at_elems += (size_t)round_up(ht.rank, 16) * L->K;
    else if (ht.kind == MUX_ADAPTER_TUNING) at_elems += (size_t)round_up(ht.rank, 16) * L->N;
  o.at_bytes = L->dtype == MUX_DT_BF16 ? align256(at_elems * 2) : 0;
  o.part_bytes = L->dtype == MUX_DT_BF16 ? fast_partial_bytes(L->K, L->N, st) : 0;
  o.dys_bytes = (L->dtype == MUX_DT_BF16 || st->n_tuning > 0) ? o.z_bytes : 0;
  o.dt_bytes = diff_transposed_bytes(L->K, L->N, st, o.esz);
  o.ws_bytes = o.tasks_bytes + o.g_bytes + o.at_bytes + o.dys_bytes + o.part_bytes + 2 * o.dt_bytes;
  return o;
}

mux_status check_layer(const char* fn, const mux_layer_desc* L, const mux_segtab* st) {
  if (!L || !st) return fail(MUX_ERR_INVALID_ARG, std::string(fn) + ": null layer or table");
  if (L->K <= 0 || L->N <= 0) return fail(MUX_ERR_INVALID_ARG, std::string(fn) + ": K and N must be positive");
  if (L->dtype != MUX_DT_BF16 && L->dtype != MUX_DT_F32) return fail(MUX_ERR_INVALID_ARG, std::string(fn) + ": unknown dtype");
  if (L->flags & ~MUX_LAYER_REFERENCE_KERNELS) return fail(MUX_ERR_INVALID_ARG, std::string(fn) + ": unknown layer flag");
  if (!L->W) return fail(MUX_ERR_INVALID_ARG, std::string(fn) + ": W is null");
  if (L->ldw < L->N) return fail(MUX_ERR_SHAPE, std::string(fn) + ": ldw < N");
  if (L->n_tasks != st->n_tasks) return fail(MUX_ERR_SHAPE, std::string(fn) + ": layer and table disagree on the number of tasks");
  if ((int64_t)st->T * (int64_t)(L->K > L->N ? L->K : L->N) >= ((int64_t)1 << 40))
    return fail(MUX_ERR_SHAPE, std::string(fn) + ": problem too large");
  for (int t = 0; t < st->n_tasks; ++t) {
    const HostTask& ht = st->tasks[t];
    if ((ht.kind == MUX_ADAPTER_LORA || ht.kind == MUX_ADAPTER_TUNING) && (!L->A || !L->B || !L->A[t] || !L->B[t]))
      return fail(MUX_ERR_INVALID_ARG, std::string(fn) + ": LoRA or Adapter-Tuning task without its two matrices");
    if (ht.kind == MUX_ADAPTER_IA3_OUT && (!L->L || !L->L[t]))
      return fail(MUX_ERR_INVALID_ARG, std::string(fn) + ": IA3 task without scale vector");
    if (ht.kind == MUX_ADAPTER_DIFF) {
      if (!L->masks || !L->masks[t]) return fail(MUX_ERR_INVALID_ARG, std::string(fn) + ": Diff-Pruning task without a mask");
      const mux_sparse_mask* m = L->masks[t];
      if (m->nnz < 0 || !m->row_ptr || !m->col_ptr) return fail(MUX_ERR_INVALID_ARG, std::string(fn) + ": bad mask");
      if (m->nnz > 0 && (!m->col_idx || !m->col_ent || !L->A || !L->A[t]))
        return fail(MUX_ERR_INVALID_ARG, std::string(fn) + ": Diff-Pruning task without entries or values");
    }
  }
  return MUX_OK;
}

int diff_max_nnz(const mux_layer_desc* L, const mux_segtab* st) {
  int m = 0;
  if (st->n_diff > 0 && L->masks)
    for (int t = 0; t < st->n_tasks; ++t)
      if (st->tasks[t].kind == MUX_ADAPTER_DIFF && L->masks[t] && L->masks[t]->nnz > m) m = L->masks[t]->nnz;
  return m;
}

mux_status check_hip(const char* fn) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(MUX_ERR_DEVICE, std::string(fn) + ": " + hipGetErrorString(e));
  return MUX_OK;
}

void fill_tasks(const mux_layer_desc* L, const mux_segtab* st, const int32_t* dtab, DevTask* dtasks, void* const* dA,
                void* const* dB, void* const* dL, hipStream_t stream, void* pack_at, int only_tuning) {
  int64_t at_off = 0;
  for (int base = 0; base < st->n_tasks; base += 16) {
    TaskPtrArgs p;
    std::memset(&p, 0, sizeof(p));
    const int count = st->n_tasks - base < 16 ? st->n_tasks - base : 16;
    for (int i = 0; i < count; ++i) {
      const int t = base + i;
      const int kind = st->tasks[t].kind;
      const bool ranked = kind == MUX_ADAPTER_LORA || kind == MUX_ADAPTER_TUNING;
      p.A[i] = ranked ? L->A[t] : nullptr;
      p.B[i] = ranked ? L->B[t] : nullptr;
      p.L[i] = (kind == MUX_ADAPTER_IA3_OUT) ? L->L[t] : nullptr;
      p.dA[i] = (ranked && dA) ? (float*)dA[t] : nullptr;
      p.dB[i] = (ranked && dB) ? (float*)dB[t] : nullptr;
      p.dL[i] = (kind == MUX_ADAPTER_IA3_OUT && dL) ? (float*)dL[t] : nullptr;
      p.at_off[i] = at_off;
      if (kind == MUX_ADAPTER_DIFF) {
        const mux_sparse_mask* m = L->masks[t];
        p.A[i] = m->nnz > 0 ? L->A[t] : nullptr;
        p.dA[i] = (m->nnz > 0 && dA) ? (float*)dA[t] : nullptr;
        p.B[i] = m->row_ptr; p.L[i] = m->col_idx;
        p.dB[i] = (float*)m->col_ptr; p.dL[i] = (float*)m->col_ent;
        p.at_off[i] = m->nnz;
      }
      if (kind == MUX_ADAPTER_LORA) at_off += (int64_t)round_up(st->tasks[t].rank, 16) * L->K;
      else if (kind == MUX_ADAPTER_TUNING) at_off += (int64_t)round_up(st->tasks[t].rank, 16) * L->N;
    }
    const int rows_max = L->K > L->N ? L->K : L->N;
    const unsigned pack_blocks = pack_at ? (unsigned)count * (unsigned)((rows_max + 63) / 64) : 0u;
    MUX_LAUNCH("fill_tasks", k_fill_tasks, dim3(1 + pack_blocks), dim3(256), 0, stream, dtab, dtasks, p, base, count,
               (uint16_t*)pack_at, L->K, L->N, only_tuning);
  }
}

}  // namespace
}  // namespace mux

using namespace mux;

extern "C" size_t mux_lora_saved_bytes(const mux_layer_desc* layer, const mux_segtab* st) {
  if (!layer || !st || layer->N <= 0) return 0;
  return make_layout(layer, st).saved_bytes;
}

extern "C" size_t mux_lora_workspace_bytes(const mux_layer_desc* layer, const mux_segtab* st) {
  if (!layer || !st || layer->N <= 0 || layer->K <= 0) return 0;
  return make_layout(layer, st).ws_bytes;
}

extern "C" mux_status mux_lora_forward(const mux_layer_desc* layer, const mux_segtab* st, const void* dev_segtab,
                                       const void* X, void* Y, void* saved, void* ws, size_t ws_bytes, void* hip_stream) {
  static const char* fn = "mux_lora_forward";
  if (mux_status s = check_layer(fn, layer, st)) return s;
  if (st->T == 0) return MUX_OK;
  if (!dev_segtab || !X || !Y || !ws) return fail(MUX_ERR_INVALID_ARG, std::string(fn) + ": null device pointer");
  const Layout lo = make_layout(layer, st);
  if (ws_bytes < lo.ws_bytes) return fail(MUX_ERR_WORKSPACE, std::string(fn) + ": workspace too small");
  if (!saved && (st->n_lora > 0 || st->n_tuning > 0))
    return fail(MUX_ERR_INVALID_ARG, std::string(fn) + ": saved is null but a task is LoRA or Adapter-Tuning");
  hipStream_t stream = (hipStream_t)hip_stream;
  DevTask* dtasks = (DevTask*)ws;
  const bool fast = layer->dtype == MUX_DT_BF16 && !(layer->flags & MUX_LAYER_REFERENCE_KERNELS);
  void* at_region = (char*)ws + lo.tasks_bytes + lo.g_bytes;
  fill_tasks(layer, st, (const int32_t*)dev_segtab, dtasks, nullptr, nullptr, nullptr, stream,
             (fast && st->n_lora + st->n_tuning > 0) ? at_region : nullptr, 0);
  CallCtx c{st, (const int32_t*)dev_segtab, dtasks, layer->K, layer->N, layer->ldw, lo.RP,
            (char*)ws + lo.tasks_bytes + lo.g_bytes, (char*)ws + lo.tasks_bytes + lo.g_bytes + lo.at_bytes, layer->W, stream,
            (saved && lo.u2_bytes) ? (char*)saved + lo.h_bytes + lo.z_bytes : nullptr, diff_max_nnz(layer, st),
            {(char*)ws + lo.ws_bytes - 2 * lo.dt_bytes, (char*)ws + lo.ws_bytes - lo.dt_bytes}};
  void* H = saved;
  void* Z = (saved && st->z_rows > 0) ? (char*)saved + lo.h_bytes : nullptr;
  mux_status s;
  if (layer->dtype == MUX_DT_F32 || (layer->flags & MUX_LAYER_REFERENCE_KERNELS))
    s = ref_forward(c, layer->dtype, X, Y, H, Z);
  else
    s = fast_forward(c, X, Y, H, Z, (char*)ws + lo.tasks_bytes + lo.g_bytes + lo.at_bytes + lo.dys_bytes);
  if (s) return s;
  // Diff-Pruning rows: the backbone wrote x W; the masked sparse update follows
  diff_forward(c, layer->dtype, X, Y);
  return check_hip(fn);
}

// The backward pass behind both entry points; `ws` is the caller's workspace or the library's static one.
static mux_status backward_impl(const char* fn, const mux_layer_desc* layer, const mux_segtab* st, const void* dev_segtab,
                                const void* X, const void* dY, const void* saved, void* dX, void* const* dA,
                                void* const* dB, void* const* dL, int accumulate, void* ws, size_t ws_bytes,
                                void* hip_stream) {
  if (mux_status s = check_layer(fn, layer, st)) return s;
  if (accumulate != 0 && accumulate != 1) return fail(MUX_ERR_INVALID_ARG, std::string(fn) + ": accumulate must be 0 or 1");
  if (st->T == 0 && st->n_tasks == 0) return MUX_OK;
  if (!dev_segtab || !ws) return fail(MUX_ERR_INVALID_ARG, std::string(fn) + ": null device pointer");
  if (st->T > 0 && (!X || !dY)) return fail(MUX_ERR_INVALID_ARG, std::string(fn) + ": null device pointer");
  if (!saved && st->T > 0 && (st->n_lora > 0 || st->n_ia3 > 0 || st->n_tuning > 0))
    return fail(MUX_ERR_INVALID_ARG, std::string(fn) + ": saved is null but a task has an adapter");
  const Layout lo = make_layout(layer, st);
  if (ws_bytes < lo.ws_bytes) return fail(MUX_ERR_WORKSPACE, std::string(fn) + ": workspace too small");
  hipStream_t stream = (hipStream_t)hip_stream;
  DevTask* dtasks = (DevTask*)ws;
  const bool fast = layer->dtype == MUX_DT_BF16 && !(layer->flags & MUX_LAYER_REFERENCE_KERNELS);
  fill_tasks(layer, st, (const int32_t*)dev_segtab, dtasks, dA, dB, dL, stream,
             (fast && st->n_tuning > 0) ? (char*)ws + lo.tasks_bytes + lo.g_bytes : nullptr, 1);
  CallCtx c{st, (const int32_t*)dev_segtab, dtasks, layer->K, layer->N, layer->ldw, lo.RP,
            (char*)ws + lo.tasks_bytes + lo.g_bytes, (char*)ws + lo.tasks_bytes + lo.g_bytes + lo.at_bytes, layer->W, stream,
            (saved && lo.u2_bytes) ? (char*)saved + lo.h_bytes + lo.z_bytes : nullptr, diff_max_nnz(layer, st),
            {(char*)ws + lo.ws_bytes - 2 * lo.dt_bytes, (char*)ws + lo.ws_bytes - lo.dt_bytes}};
  if (st->T == 0) {                 // no rows at all: zero gradients (or leave the accumulators as they are)
    if (!accumulate) {
      size_t big = (size_t)(st->r_max > 0 ? st->r_max : 1) * (size_t)(layer->K > layer->N ? layer->K : layer->N);
      if ((size_t)c.diff_max_nnz > big) big = (size_t)c.diff_max_nnz;
      MUX_LAUNCH("zero_grads", k_zero_grads, dim3(st->n_tasks, (unsigned)((big + 255) / 256)), dim3(256), 0, stream, dtasks,
                 layer->K, layer->N);
    }
    return check_hip(fn);
  }
  const void* H = saved;
  const void* Z = (saved && st->z_rows > 0) ? (const char*)saved + lo.h_bytes : nullptr;
  void* G = (char*)ws + lo.tasks_bytes;
  mux_status s;
  if (layer->dtype == MUX_DT_F32 || (layer->flags & MUX_LAYER_REFERENCE_KERNELS))
    s = ref_backward(c, layer->dtype, X, dY, H, Z, G, dX, accumulate);
  else
    s = fast_backward(c, X, dY, H, Z, G, dX, accumulate, (char*)ws + lo.tasks_bytes + lo.g_bytes + lo.at_bytes + lo.dys_bytes);
  if (s) return s;
  diff_backward(c, layer->dtype, X, dY, dX, accumulate);
  return check_hip(fn);
}

extern "C" mux_status mux_lora_backward(const mux_layer_desc* layer, const mux_segtab* st, const void* dev_segtab,
                                        const void* X, const void* dY, const void* saved, void* dX, void* const* dA,
                                        void* const* dB, void* const* dL, int accumulate, void* ws, size_t ws_bytes,
                                        void* hip_stream) {
  return backward_impl("mux_lora_backward", layer, st, dev_segtab, X, dY, saved, dX, dA, dB, dL, accumulate, ws, ws_bytes,
                       hip_stream);
}

// ---- the backward pass for callers that cannot allocate: its workspace is a file-scope device array -------------------
namespace {

constexpr size_t kStaticWsBytes = MUX_STATIC_WS_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticWsBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices];      // per device: the address of that device's copy of `scratch`

// Address of the current device's copy of the array (looked up once per device, with that device current).
mux_status static_workspace(const char* fn, void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
    return fail(MUX_ERR_DEVICE, std::string(fn) + ": no current device");
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p)
      return fail(MUX_ERR_DEVICE, std::string(fn) + ": hipGetSymbolAddress: " + hipGetErrorString(e));
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return MUX_OK;
}

}  // namespace

extern "C" mux_status mux_lora_backward_static_ws(const mux_layer_desc* layer, const mux_segtab* st, const void* dev_segtab,
                                                  const void* X, const void* dY, const void* saved, void* dX,
                                                  void* const* dA, void* const* dB, void* const* dL, int accumulate,
                                                  void* hip_stream) {
  static const char* fn = "mux_lora_backward_static_ws";
  if (mux_status s = check_layer(fn, layer, st)) return s;
  const size_t need = make_layout(layer, st).ws_bytes;
  if (need > kStaticWsBytes)
    return fail(MUX_ERR_WORKSPACE, std::string(fn) + ": this call needs " + std::to_string(need) +
                                       " bytes of workspace, the static one holds " + std::to_string(kStaticWsBytes));
  void* ws = nullptr;
  if (mux_status s = static_workspace(fn, &ws)) return s;
  return backward_impl(fn, layer, st, dev_segtab, X, dY, saved, dX, dA, dB, dL, accumulate, ws, kStaticWsBytes, hip_stream);
}
