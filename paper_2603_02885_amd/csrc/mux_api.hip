// Entry points of the layer: argument checks, buffer carving, kernel sequencing.
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

#include "mux_device_utils.h"

namespace mux {

// Writes `count` entries of the per-call task table, handed over in the launch arguments, into the workspace.
__global__ __launch_bounds__(64) void k_write_tasks(DevTask* __restrict__ out, const TaskTable tb, int base, int count) {
  const int i = threadIdx.x;
  if (i < count) out[base + i] = tb.t[i];
}

// A_t^T [round_up(r,16)][K] (zero rows beyond r) of the LoRA tasks whose rank is not a multiple of 8, and D_t^T
// [round_up(r,16)][N] of the Adapter-Tuning tasks, into the transposed region of the workspace: the down-projection
// reads these operands with the contraction index contiguous.  Block b handles 64 rows of task b / nkb.
__global__ __launch_bounds__(256) void k_pack_at(const TaskRef tasks, uint16_t* __restrict__ pack_at, int Kin, int Nout,
                                                  int only_tuning) {
  __shared__ uint16_t t[64][66];
  const int nkb = ((Kin > Nout ? Kin : Nout) + 63) / 64;
  const int i = blockIdx.x / nkb, k0 = (blockIdx.x % nkb) * 64;
  const DevTask tk = get_task(tasks, i);
  // LORA: A_t [K, r]; TUNING: D_t [N, r] (in the same slot); both go out as [round_up(r,16)][rows]
  if (tk.kind != MUX_ADAPTER_LORA && tk.kind != MUX_ADAPTER_TUNING) return;
  if (only_tuning && tk.kind != MUX_ADAPTER_TUNING) return;     // the backward pass needs D_t^T only
  if (tk.at_off < 0) return;                                     // a LoRA task whose A_t is read as it is
  const int K = tk.kind == MUX_ADAPTER_LORA ? Kin : Nout;
  if (k0 >= K) return;
  const int r = tk.rank, rp = (r + 15) & ~15;
  const uint16_t* A = (const uint16_t*)tk.A;
  for (int e = threadIdx.x; e < 64 * rp; e += 256) {
    const int kk = e / rp, j = e % rp;
    t[j][kk] = (j < r && k0 + kk < K) ? A[(size_t)(k0 + kk) * r + j] : (uint16_t)0;
  }
  __syncthreads();
  uint16_t* dst = pack_at + tk.at_off;
  for (int e = threadIdx.x; e < 64 * rp; e += 256) {
    const int j = e >> 6, kk = e & 63;
    if (k0 + kk < K) dst[(size_t)j * K + k0 + kk] = t[j][kk];
  }
}

// A table without rows: every task's gradient is zero.  grid = (tasks, blocks over the largest gradient).
__global__ __launch_bounds__(256) void k_zero_grads(const TaskRef tasks, int K, int N) {
  const DevTask tk = get_task(tasks, blockIdx.x);
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
  size_t tasks_bytes, g_bytes, at_bytes, dys_bytes, part_bytes, dt_bytes, dw_bytes, dp_bytes, ws_bytes;
  int dw_slots;        // DIFF tasks with entries: each gets room for its merged weight (matrix-core path)
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
  // Diff-Pruning on the matrix-core path.  Where the shapes allow it (see fast_gemm_patches_diff) the backbone product
  // adds the masked entries to its tiles of W in LDS and the call only packs them: 4 bytes an entry.
  bool patchable = false;
  if (L->dtype == MUX_DT_BF16 && !(L->flags & MUX_LAYER_REFERENCE_KERNELS) && st->n_diff > 0 && L->masks &&
      L->K < 65536 && L->N < 65536 && (L->K % 64 == 0 || L->N % 64 == 0)) {
    size_t nnz = 0;
    bool listed = true;                                // every mask brings its listing by tiles
    for (int t = 0; t < st->n_tasks; ++t)
      if (st->tasks[t].kind == MUX_ADAPTER_DIFF && L->masks[t] && L->masks[t]->nnz > 0) {
        const mux_sparse_mask* m = L->masks[t];
        nnz += (size_t)m->nnz;
        listed = listed && m->fwd_ptr && m->fwd_ent && m->bwd_ptr && m->bwd_ent;
      }
    o.dp_bytes = (nnz > 0 && listed) ? align256(nnz * 4) : 0;
    patchable = o.dp_bytes > 0 && L->K % 64 == 0 && L->N % 64 == 0;   // both directions: no call of this layer needs another route
  }
  // Otherwise: the sparse updates after the backbone products cost about 0.65 us per
  // million (row, entry) pairs, a merged weight W + M_t * delta_t per task about 2.3 us per million elements of W and
  // nothing per row; the call merges when that is the cheaper of the two (measured on 4096 x 4096 with masks of 0.5 %:
  // from about 700 rows a task on).
  if (!patchable && L->dtype == MUX_DT_BF16 && !(L->flags & MUX_LAYER_REFERENCE_KERNELS) && st->n_diff > 0 && L->masks) {
    int slots = 0;
    double pairs = 0.0;
    for (int t = 0; t < st->n_tasks; ++t)
      if (st->tasks[t].kind == MUX_ADAPTER_DIFF && L->masks[t] && L->masks[t]->nnz > 0) {
        ++slots;
        pairs += (double)st->tasks[t].row_count * (double)L->masks[t]->nnz;
      }
    if (0.65 * pairs > 2.3 * (double)slots * (double)L->K * (double)L->N) o.dw_slots = slots;
  }
  o.dw_bytes = (size_t)o.dw_slots * diff_merged_bytes(L->K, L->ldw);
  o.ws_bytes = o.tasks_bytes + o.g_bytes + o.at_bytes + o.dys_bytes + o.part_bytes + 2 * o.dt_bytes + o.dw_bytes + o.dp_bytes;
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

// Does the down-projection read this LoRA task's A_t [K, r] as it is (rows of 16-byte pieces), or a transposed copy?
inline bool lora_a_natural(const HostTask& ht) { return (ht.rank & 7) == 0; }

// The per-call task parameters, laid out on the host.  at_off: element offset of the task's transposed operand in the
// workspace region, -1 for a LoRA task whose A_t is read as it is.
void build_tasks(const mux_layer_desc* L, const mux_segtab* st, void* const* dA, void* const* dB, void* const* dL,
                 bool fast, int diff_route, bool backward, std::vector<DevTask>& out) {
  out.assign((size_t)st->n_tasks, DevTask{});
  int64_t at_off = 0;
  int slot = 0;         // diff_route 1: index of the next merged weight; 2: element offset of the next packed list
  for (int t = 0; t < st->n_tasks; ++t) {
    const HostTask& ht = st->tasks[t];
    const int kind = ht.kind;
    const bool ranked = kind == MUX_ADAPTER_LORA || kind == MUX_ADAPTER_TUNING;
    DevTask& d = out[t];
    d.A = ranked ? L->A[t] : nullptr;
    d.B = ranked ? L->B[t] : nullptr;
    d.L = (kind == MUX_ADAPTER_IA3_OUT) ? L->L[t] : nullptr;
    d.dA = (ranked && dA) ? (float*)dA[t] : nullptr;
    d.dB = (ranked && dB) ? (float*)dB[t] : nullptr;
    d.dL = (kind == MUX_ADAPTER_IA3_OUT && dL) ? (float*)dL[t] : nullptr;
    d.scale = ht.scale; d.kind = kind; d.rank = ht.rank;
    d.row_begin = ht.row_begin; d.row_count = ht.row_count; d.zrow0 = ht.zrow0;
    d.at_off = at_off;
    if (kind == MUX_ADAPTER_DIFF) {
      const mux_sparse_mask* m = L->masks[t];
      d.A = m->nnz > 0 ? L->A[t] : nullptr;
      d.dA = (m->nnz > 0 && dA) ? (float*)dA[t] : nullptr;
      d.B = m->row_ptr; d.L = m->col_idx;
      d.dB = (float*)m->col_ptr; d.dL = (float*)m->col_ent;
      d.at_off = m->nnz;
      d.rank = -1;
      if (m->nnz > 0 && diff_route == 1) d.rank = slot++;
      if (m->nnz > 0 && diff_route == 2) {              // the listing by tiles of this direction instead of the column listing
        d.rank = slot; slot += m->nnz;
        d.dB = (float*)(backward ? m->bwd_ptr : m->fwd_ptr);
        d.dL = (float*)(backward ? m->bwd_ent : m->fwd_ent);
      }
    }
    if (kind == MUX_ADAPTER_LORA) {
      if (fast && lora_a_natural(ht)) d.at_off = -1;
      at_off += (int64_t)round_up(ht.rank, 16) * L->K;
    } else if (kind == MUX_ADAPTER_TUNING) {
      at_off += (int64_t)round_up(ht.rank, 16) * L->N;
    }
  }
}

// Makes the tasks visible to the kernels of the call: by value in `ref` when they fit and no kernel of the call needs
// the table in memory, else written into the workspace by a small kernel; and lays out the transposed operands when
// a kernel of the call reads them (pack: 0 no, 1 all of them, 2 only those of the Adapter-Tuning tasks).
void publish_tasks(const mux_layer_desc* L, const mux_segtab* st, const std::vector<DevTask>& tasks, bool need_table,
                   DevTask* dtasks, TaskRef& ref, int pack, void* pack_at, hipStream_t stream) {
  std::memset(&ref, 0, sizeof(ref));
  if (!need_table && st->n_tasks <= kArgTasks) {
    for (int t = 0; t < st->n_tasks; ++t) ref.arg.t[t] = tasks[t];
  } else {
    for (int base = 0; base < st->n_tasks; base += kArgTasks) {
      TaskTable tb;
      std::memset(&tb, 0, sizeof(tb));
      const int count = st->n_tasks - base < kArgTasks ? st->n_tasks - base : kArgTasks;
      for (int i = 0; i < count; ++i) tb.t[i] = tasks[base + i];
      MUX_LAUNCH("fill_tasks", k_write_tasks, dim3(1), dim3(64), 0, stream, dtasks, tb, base, count);
    }
    ref.mem = dtasks;
  }
  if (pack && pack_at) {
    const int rows_max = L->K > L->N ? L->K : L->N;
    MUX_LAUNCH("pack_at", k_pack_at, dim3((unsigned)st->n_tasks * (unsigned)((rows_max + 63) / 64)), dim3(256), 0, stream,
               ref, (uint16_t*)pack_at, L->K, L->N, pack == 2 ? 1 : 0);
  }
}

bool any_packed_lora(const mux_segtab* st) {
  for (const HostTask& ht : st->tasks)
    if (ht.kind == MUX_ADAPTER_LORA && !lora_a_natural(ht)) return true;
  return false;
}
bool any_packed_tuning(const mux_segtab* st) {
  for (const HostTask& ht : st->tasks)
    if (ht.kind == MUX_ADAPTER_TUNING && (ht.rank & 7) != 0) return true;
  return false;
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

namespace {

// Everything a call's kernels share, from the layer, the table and the carved workspace.
CallCtx make_ctx(const mux_layer_desc* layer, const mux_segtab* st, const void* dev_segtab, const Layout& lo, void* ws,
                 const void* saved, hipStream_t stream) {
  CallCtx c{};
  c.st = st;
  c.dtab = (const int32_t*)dev_segtab;
  c.K = layer->K; c.N = layer->N; c.ldw = layer->ldw; c.RP = lo.RP;
  c.AT = (char*)ws + lo.tasks_bytes + lo.g_bytes;
  c.dYs = (char*)ws + lo.tasks_bytes + lo.g_bytes + lo.at_bytes;
  c.W = layer->W;
  c.stream = stream;
  c.U2 = (saved && lo.u2_bytes) ? (char*)saved + lo.h_bytes + lo.z_bytes : nullptr;
  c.diff_max_nnz = diff_max_nnz(layer, st);
  c.diffT[0] = (char*)ws + lo.ws_bytes - lo.dp_bytes - lo.dw_bytes - 2 * lo.dt_bytes;
  c.diffT[1] = (char*)ws + lo.ws_bytes - lo.dp_bytes - lo.dw_bytes - lo.dt_bytes;
  c.diffW = nullptr;
  c.diffPack = nullptr;
  c.diffW_stride = (int64_t)(diff_merged_bytes(layer->K, layer->ldw) / 2);
  c.diffW_slots = lo.dw_slots;
  return c;
}

}  // namespace

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
  CallCtx c = make_ctx(layer, st, dev_segtab, lo, ws, saved, stream);
  void* H = saved;
  void* Z = (saved && st->z_rows > 0) ? (char*)saved + lo.h_bytes : nullptr;
  // the matrix-core kernels, unless the storage type, the flag, a shape or a pointer rules them out: then the plain ones
  const bool fast = layer->dtype == MUX_DT_BF16 && !(layer->flags & MUX_LAYER_REFERENCE_KERNELS) &&
                    fast_supported(c, X, Y, H, Z, nullptr, nullptr);
  c.lora_natural = fast && !any_packed_lora(st);
  if (fast && lo.dp_bytes > 0 && fast_gemm_patches_diff(c, false)) c.diffPack = (char*)ws + lo.ws_bytes - lo.dp_bytes;
  else if (fast && lo.dw_bytes > 0) c.diffW = (char*)ws + lo.ws_bytes - lo.dp_bytes - lo.dw_bytes;
  std::vector<DevTask> tasks;
  build_tasks(layer, st, nullptr, nullptr, nullptr, c.lora_natural, c.diffPack ? 2 : (c.diffW ? 1 : 0), false, tasks);
  TaskRef tref;
  c.tune_natural = fast && !any_packed_tuning(st);
  const int pack = !fast ? 0 : ((st->n_lora > 0 && !c.lora_natural) ? 1 : ((st->n_tuning > 0 && !c.tune_natural) ? 2 : 0));
  publish_tasks(layer, st, tasks, !fast, (DevTask*)ws, tref, pack, c.AT, stream);
  c.tref = &tref;
  c.dtasks = tref.mem;
  mux_status s;
  if (!fast) s = ref_forward(c, layer->dtype, X, Y, H, Z);
  else s = fast_forward(c, X, Y, H, Z, (char*)ws + lo.tasks_bytes + lo.g_bytes + lo.at_bytes + lo.dys_bytes);
  if (s) return s;
  // Diff-Pruning rows: the backbone wrote x W (the masked sparse update follows), or x (W + M_t * delta_t) already
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
  CallCtx c = make_ctx(layer, st, dev_segtab, lo, ws, saved, stream);
  const void* H = saved;
  const void* Z = (saved && st->z_rows > 0) ? (const char*)saved + lo.h_bytes : nullptr;
  void* G = (char*)ws + lo.tasks_bytes;
  const bool fast = layer->dtype == MUX_DT_BF16 && !(layer->flags & MUX_LAYER_REFERENCE_KERNELS) &&
                    fast_supported(c, X, dY, dX, G, H, Z);
  c.lora_natural = fast && !any_packed_lora(st);
  if (fast && lo.dp_bytes > 0 && dX && fast_gemm_patches_diff(c, true)) c.diffPack = (char*)ws + lo.ws_bytes - lo.dp_bytes;
  else if (fast && lo.dw_bytes > 0 && dX) c.diffW = (char*)ws + lo.ws_bytes - lo.dp_bytes - lo.dw_bytes;
  std::vector<DevTask> tasks;
  build_tasks(layer, st, dA, dB, dL, c.lora_natural, c.diffPack ? 2 : (c.diffW ? 1 : 0), true, tasks);
  TaskRef tref;
  c.tune_natural = fast && !any_packed_tuning(st);
  publish_tasks(layer, st, tasks, !fast, (DevTask*)ws, tref, (fast && st->n_tuning > 0 && !c.tune_natural) ? 2 : 0, c.AT, stream);
  c.tref = &tref;
  c.dtasks = tref.mem;
  if (st->T == 0) {                 // no rows at all: zero gradients (or leave the accumulators as they are)
    if (!accumulate) {
      size_t big = (size_t)(st->r_max > 0 ? st->r_max : 1) * (size_t)(layer->K > layer->N ? layer->K : layer->N);
      if ((size_t)c.diff_max_nnz > big) big = (size_t)c.diff_max_nnz;
      MUX_LAUNCH("zero_grads", k_zero_grads, dim3(st->n_tasks, (unsigned)((big + 255) / 256)), dim3(256), 0, stream, tref,
                 layer->K, layer->N);
    }
    return check_hip(fn);
  }
  mux_status s;
  if (!fast) s = ref_backward(c, layer->dtype, X, dY, H, Z, G, dX, accumulate);
  else s = fast_backward(c, X, dY, H, Z, G, dX, accumulate, (char*)ws + lo.tasks_bytes + lo.g_bytes + lo.at_bytes + lo.dys_bytes);
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
