// Small device helpers shared by the kernels: bf16 conversion, table access.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mux_internal.h"

namespace mux {

typedef uint16_t bf16_t;

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float((uint32_t)v << 16); }

// float -> bfloat16, round to nearest even (v_cvt_pk_bf16_f32 on gfx950; NaN stays NaN)
typedef __attribute__((ext_vector_type(2))) float mux_f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 mux_bf16x2;

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const mux_f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, mux_bf16x2));
}

__device__ __forceinline__ bf16_t f32_to_bf16(float f) { return __builtin_bit_cast(bf16_t, (__bf16)f); }

template <class S> struct Store;
template <> struct Store<float> {
  static __device__ __forceinline__ float ld(const float* p, size_t i) { return p[i]; }
  static __device__ __forceinline__ void st(float* p, size_t i, float v) { p[i] = v; }
};
template <> struct Store<bf16_t> {
  static __device__ __forceinline__ float ld(const bf16_t* p, size_t i) { return bf16_to_f32(p[i]); }
  static __device__ __forceinline__ void st(bf16_t* p, size_t i, float v) { p[i] = f32_to_bf16(v); }
};

// Row i is a real token iff (i mod chunk) < valid_rows[i div chunk]  (chunk is a power of two).
__device__ __forceinline__ bool row_is_valid(const int32_t* __restrict__ dtab, int row) {
  const int lg = dtab[DH_LOG2C];
  const int ch = row >> lg;
  return (row & ((1 << lg) - 1)) < dtab[dtab[DH_OFF_CHUNK_VALID] + ch];
}

// Validity bits of rows row_base .. row_base+31 (bit r = row row_base + r is a real token).
__device__ __forceinline__ uint32_t row_valid_bits32(const int32_t* __restrict__ dtab, int row_base) {
  const uint32_t* bm = (const uint32_t*)(dtab + dtab[DH_OFF_ROWBITS]);
  const int w = row_base >> 5, sh = row_base & 31;
  const uint64_t two = (uint64_t)bm[w] | ((uint64_t)bm[w + 1] << 32);
  return (uint32_t)(two >> sh);
}

// Task t of the call.  t is the same for every lane of the wave (an item, a tile or a block belongs to one task), and
// so is every word of the result: saying so word by word keeps what is derived from it (buffer descriptors, loop
// bounds) in scalar registers whichever of the two sources the words came from.
__device__ __forceinline__ DevTask get_task(const TaskRef& r, int t) {
  t = __builtin_amdgcn_readfirstlane(t);
  const DevTask d = r.mem ? r.mem[t] : r.arg.t[t];
  constexpr int W = sizeof(DevTask) / 4;
  uint32_t w[W];
  __builtin_memcpy(w, &d, sizeof(DevTask));
#pragma unroll
  for (int i = 0; i < W; ++i) w[i] = (uint32_t)__builtin_amdgcn_readfirstlane((int)w[i]);
  DevTask o;
  __builtin_memcpy(&o, w, sizeof(DevTask));
  return o;
}
__device__ __forceinline__ int get_task_kind(const TaskRef& r, int t) {
  t = __builtin_amdgcn_readfirstlane(t);
  return __builtin_amdgcn_readfirstlane(r.mem ? r.mem[t].kind : r.arg.t[t].kind);
}

// The weight the rows of a task meet in the backbone product: W, or for a Diff-Pruning task whose merged weight the call
// has built, W + M_t * delta_t in the workspace.
template <class T>
__device__ __forceinline__ const T* task_weight(const DevTask& tk, const T* W, const T* Wdiff, int64_t stride) {
  return (tk.kind == MUX_ADAPTER_DIFF && Wdiff != nullptr && tk.rank >= 0) ? Wdiff + (size_t)tk.rank * (size_t)stride : W;
}

struct ItemView { int task, row0, nrows, nvalid; };
__device__ __forceinline__ ItemView load_item(const int32_t* __restrict__ dtab, int tile_size_index, int item) {
  const int32_t* p = dtab + dtab[DH_NITEMS0 + 3 * tile_size_index + 1] + item * DI_WORDS;
  return {p[DI_TASK], p[DI_ROW0], p[DI_NROWS], p[DI_NVALID]};
}

}  // namespace mux
