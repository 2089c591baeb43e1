// Dispatch (section 3.2, section 3.5): placement of the tasks' packed tokens on the rows of the chunk-aligned batch and
// back.  One workgroup per 64-row work item of the table; the packed position of a row's token is the item's first
// token (from the table's device image) plus the number of valid rows before it inside the item.  Rows move as
// 16-byte vectors when every address allows it, else element by element.
#include "mux_device_utils.h"
#include "mux_dispatch.h"

namespace mux {
namespace {

constexpr int kBatch = 32;      // task pointers per launch (kernel arguments)

struct DispatchParams {
  const int32_t* dtab;
  char* task[kBatch];
  int task_base, task_count;
  char* aligned;
  int64_t row_bytes_task, row_bytes_aligned;     // bytes between rows
  int width_bytes;
  int to_aligned;                                // 1: gather (packed -> aligned, padding zeroed), 0: scatter
};

// grid = (64-row items, slabs of 256 vectors across the width), four waves: wave w moves the rows w, w + 4, ...
// `first` launch of a gather also zeroes the rows of no task and the padding rows of every task.
template <class V>
__global__ __launch_bounds__(256) void k_dispatch(DispatchParams p, int first) {
  const ItemView it = load_item(p.dtab, 0, blockIdx.x);
  const bool mine = it.task >= p.task_base && it.task < p.task_base + p.task_count;
  if (!mine && !(p.to_aligned && first)) return;
  const int tok0 = p.dtab[p.dtab[DH_OFF_ITEM_TOK0] + blockIdx.x];
  uint64_t valid = 0;                              // bit r: row row0 + r carries a token
  if (it.task >= 0) {
    valid = row_valid_bits32(p.dtab, it.row0);
    if (it.nrows > 32) valid |= (uint64_t)row_valid_bits32(p.dtab, it.row0 + 32) << 32;
    if (it.nrows < 64) valid &= ((uint64_t)1 << it.nrows) - 1;
  }
  char* packed = mine ? p.task[it.task - p.task_base] : nullptr;
  // a workgroup moves a slab of 4 x 64 vectors of every row of its item; a wave has four of its rows in flight at
  // a time, four vectors per lane each (one row at a time cost a memory latency per row)
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int slab = (int)blockIdx.y * 256 * (int)sizeof(V) + lane * (int)sizeof(V);
  constexpr int RU = 4;
  for (int r0 = wave; r0 < it.nrows; r0 += 4 * RU) {
    V v[RU][4];
    char* dst[RU];
    int what[RU];                                  // 0: nothing, 1: copy, 2: zero
#pragma unroll
    for (int u = 0; u < RU; ++u) {
      const int r = r0 + 4 * u;
      what[u] = 0;
      dst[u] = nullptr;
      if (r >= it.nrows) continue;
      char* arow = p.aligned + (size_t)(it.row0 + r) * p.row_bytes_aligned;
      if ((valid >> r) & 1) {
        if (!mine) continue;
        const int tok = tok0 + __popcll(valid & (((uint64_t)1 << r) - 1));
        char* prow = packed + (size_t)tok * p.row_bytes_task;
        const char* src = p.to_aligned ? prow : arow;
        dst[u] = p.to_aligned ? arow : prow;
        what[u] = 1;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const int o = slab + k * 64 * (int)sizeof(V);
          if (o < p.width_bytes) v[u][k] = *(const V*)(src + o);
        }
      } else if (p.to_aligned && first) {
        dst[u] = arow;
        what[u] = 2;
      }
    }
#pragma unroll
    for (int u = 0; u < RU; ++u) {
      if (what[u] == 0) continue;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int o = slab + k * 64 * (int)sizeof(V);
        if (o < p.width_bytes) *(V*)(dst[u] + o) = what[u] == 1 ? v[u][k] : V{};
      }
    }
  }
}

mux_status run(const char* fn, const mux_segtab* st, const void* dev_segtab, void* const* task_ptrs, int64_t ld_task,
               void* aligned, int64_t ld_aligned, int32_t width, int32_t elem_bytes, void* hip_stream, int to_aligned) {
  if (!st) return fail(MUX_ERR_INVALID_ARG, std::string(fn) + ": null table");
  if (elem_bytes != 2 && elem_bytes != 4) return fail(MUX_ERR_INVALID_ARG, std::string(fn) + ": elem_bytes must be 2 or 4");
  if (width < 1 || ld_task < width || ld_aligned < width) return fail(MUX_ERR_SHAPE, std::string(fn) + ": bad width or leading dimension");
  if ((int64_t)st->T * ld_aligned * elem_bytes >= ((int64_t)1 << 42)) return fail(MUX_ERR_SHAPE, std::string(fn) + ": problem too large");
  if (st->T == 0) return MUX_OK;
  if (!dev_segtab || !aligned || (st->n_tasks > 0 && !task_ptrs)) return fail(MUX_ERR_INVALID_ARG, std::string(fn) + ": null pointer");
  bool vec = ((uintptr_t)aligned & 15) == 0 && (ld_aligned * elem_bytes) % 16 == 0 && (ld_task * elem_bytes) % 16 == 0 &&
             ((int64_t)width * elem_bytes) % 16 == 0;
  for (int t = 0; t < st->n_tasks; ++t) {
    if (st->tasks[t].valid > 0 && !task_ptrs[t]) return fail(MUX_ERR_INVALID_ARG, std::string(fn) + ": a task with tokens has no buffer");
    if (((uintptr_t)task_ptrs[t] & 15) != 0) vec = false;
  }
  hipStream_t stream = (hipStream_t)hip_stream;
  const unsigned n_items = (unsigned)st->items[0].size();
  bool first = true;
  for (int base = 0; base < st->n_tasks || first; base += kBatch) {
    DispatchParams p{};
    p.dtab = (const int32_t*)dev_segtab;
    p.task_base = base;
    p.task_count = std::min(kBatch, std::max(0, st->n_tasks - base));
    for (int i = 0; i < p.task_count; ++i) p.task[i] = (char*)task_ptrs[base + i];
    p.aligned = (char*)aligned;
    p.row_bytes_task = ld_task * elem_bytes;
    p.row_bytes_aligned = ld_aligned * elem_bytes;
    p.width_bytes = width * elem_bytes;
    p.to_aligned = to_aligned;
    const char* name = to_aligned ? "dispatch_gather" : "dispatch_scatter";
    const unsigned wb = (unsigned)p.width_bytes;
    if (vec) MUX_LAUNCH(name, k_dispatch<uint4>, dim3(n_items, (wb + 4095) / 4096), dim3(256), 0, stream, p, first ? 1 : 0);
    else if (elem_bytes == 4) MUX_LAUNCH(name, k_dispatch<uint32_t>, dim3(n_items, (wb + 1023) / 1024), dim3(256), 0, stream, p, first ? 1 : 0);
    else MUX_LAUNCH(name, k_dispatch<uint16_t>, dim3(n_items, (wb + 511) / 512), dim3(256), 0, stream, p, first ? 1 : 0);
    first = false;
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(MUX_ERR_DEVICE, std::string(fn) + ": " + hipGetErrorString(e));
  return MUX_OK;
}

}  // namespace
}  // namespace mux

extern "C" mux_status mux_dispatch_gather(const mux_segtab* st, const void* dev_segtab, const void* const* task_ptrs,
                                          int64_t ld_task, void* aligned, int64_t ld_aligned, int32_t width,
                                          int32_t elem_bytes, void* hip_stream) {
  return mux::run("mux_dispatch_gather", st, dev_segtab, (void* const*)task_ptrs, ld_task, aligned, ld_aligned, width,
                  elem_bytes, hip_stream, 1);
}

extern "C" mux_status mux_dispatch_scatter(const mux_segtab* st, const void* dev_segtab, const void* aligned,
                                           int64_t ld_aligned, void* const* task_ptrs, int64_t ld_task, int32_t width,
                                           int32_t elem_bytes, void* hip_stream) {
  return mux::run("mux_dispatch_scatter", st, dev_segtab, task_ptrs, ld_task, (void*)aligned, ld_aligned, width,
                  elem_bytes, hip_stream, 0);
}
