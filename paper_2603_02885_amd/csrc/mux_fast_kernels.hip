// bf16 matrix-core path: sequences the MFMA kernels of one layer call.
#include "mux_device_utils.h"

namespace mux {

size_t fast_partial_bytes(int, int, const mux_segtab*) { return 0; }

static bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

mux_status fast_forward(const CallCtx& c, const void* X, void* Y, void* H, void* Z, void*) {
  if (!gemm_mfma_supported(c) || !aligned16(X) || !aligned16(Y) || !aligned16(H) || !aligned16(Z))
    return ref_forward(c, MUX_DT_BF16, X, Y, H, Z);    // shapes the 16-byte loads cannot take
  ref_steps(c, MUX_DT_BF16, REF_DOWN, X, nullptr, nullptr, nullptr, H, nullptr, nullptr, 0);
  return gemm_mfma_forward(c, X, H, Y, Z);
}

mux_status fast_backward(const CallCtx& c, const void* X, const void* dY, const void* H, const void* Z, void* G, void* dX,
                         int accumulate, void*) {
  if (!gemm_mfma_supported(c) || !aligned16(dY) || !aligned16(dX) || !aligned16(G))
    return ref_backward(c, MUX_DT_BF16, X, dY, H, Z, G, dX, accumulate);
  ref_steps(c, MUX_DT_BF16, REF_G | REF_DB | REF_DA | REF_DL, X, dY, nullptr, nullptr, (void*)H, (void*)Z, G, accumulate);
  if (dX) return gemm_mfma_backward(c, dY, G, dX);
  return MUX_OK;
}

}  // namespace mux
