// bf16 matrix-core path: sequences the MFMA kernels of one layer call.
#include <cstdlib>

#include "mux_device_utils.h"

namespace mux {

size_t fast_partial_bytes(int K, int N, const mux_segtab* st) { return adapter_partial_bytes(K, N, st); }

static bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

// Measurement switch, read once per process: the register-staged backbone kernel on every shape.
static bool regstaged() {
  static const bool on = getenv("MUX_GEMM_REGSTAGED") != nullptr;
  return on;
}

// The 16-byte loads of the matrix-core kernels need 16-byte aligned rows everywhere.
bool fast_supported(const CallCtx& c, const void* p0, const void* p1, const void* p2, const void* p3, const void* p4,
                    const void* p5) {
  return gemm_mfma_supported(c) && aligned16(p0) && aligned16(p1) && aligned16(p2) && aligned16(p3) && aligned16(p4) &&
         aligned16(p5);
}

// Diff-Pruning rows through the pipelined kernel's 64-deep tile loop, which adds the masked entries to the tiles of W
// in LDS: 16-bit indices and a contraction length that is a multiple of 64.
bool fast_gemm_patches_diff(const CallCtx& c, bool backward) {
  if (regstaged() || !gemm_dma_supported(c, backward)) return false;
  static const bool narrow = getenv("MUX_GEMM_BK32") != nullptr;      // measurement switch, read once: 32-deep stages everywhere
  return !narrow && c.K < 65536 && c.N < 65536 && (backward ? c.N : c.K) % 64 == 0;
}

// The caller has checked fast_supported for the shapes and pointers of this call.
mux_status fast_forward(const CallCtx& c, const void* X, void* Y, void* H, void* Z, void*) {
  // small launches form Hs = s_t X A_t inside the backbone tile loop; the others stream X once more for it
  const bool pipelined = gemm_dma_supported(c, false) && !regstaged();
  const bool fuse_down = pipelined && gemm_dma_fuses_down(c);
  if (!fuse_down)
    if (mux_status s = adapter_down_x(c, X, H)) return s;
  // Diff-Pruning tasks: their rows meet W + M_t * delta_t in the backbone product (entries added in LDS, or a copy)
  if (c.diffPack) diff_pack(c, false); else diff_merge(c, c.diffW_slots);
  mux_status s;
  if (pipelined) s = gemm_dma_forward(c, X, H, Y, Z, fuse_down);
  else s = gemm_mfma_forward(c, X, H, Y, Z);
  if (s != MUX_OK) return s;
  // Adapter-Tuning rows: the GEMM saved x W; the bottleneck follows (u = z D_t, Y = z + s_t gelu(u) U_t)
  if (c.st->n_tuning > 0) {
    if (mux_status st = adapter_down_tune(c, Z, H)) return st;
    if (mux_status st = adapter_tune_add(c, Z, H, Y, 0)) return st;
  }
  return MUX_OK;
}

mux_status fast_backward(const CallCtx& c, const void* X, const void* dY, const void* H, const void* Z, void* G, void* dX,
                         int accumulate, void* part) {
  // one pass over dY: Gs and the partial sums of dB_t
  if (mux_status s = adapter_dy_pass(c, dY, H, G, part)) return s;
  // Adapter-Tuning rows enter the backbone backward as dY + Gs D_t^T
  if (mux_status s = adapter_tune_add(c, dY, G, c.dYs, 1)) return s;
  if (mux_status s = adapter_grads(c, X, dY, H, G, Z, part, accumulate)) return s;
  if (!dX) return MUX_OK;
  if (c.diffPack) diff_pack(c, true); else diff_merge(c, c.diffW_slots);
  if (gemm_dma_supported(c, true) && !regstaged()) {
    // IA3_OUT rows read dY * l_t, written by the dl kernel above
    return gemm_dma_backward(c, dY, G, dX);
  }
  return gemm_mfma_backward(c, dY, G, dX, 0);
}

}  // namespace mux
