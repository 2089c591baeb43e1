// bf16 matrix-core path (placeholder wiring: routes to the plain kernels until the MFMA kernels land).
#include "mux_device_utils.h"

namespace mux {

size_t fast_partial_bytes(int, int, const mux_segtab*) { return 0; }

mux_status fast_forward(const CallCtx& c, const void* X, void* Y, void* H, void* Z, void*) {
  return ref_forward(c, MUX_DT_BF16, X, Y, H, Z);
}

mux_status fast_backward(const CallCtx& c, const void* X, const void* dY, const void* H, const void* Z, void* G, void* dX,
                         int accumulate, void*) {
  return ref_backward(c, MUX_DT_BF16, X, dY, H, Z, G, dX, accumulate);
}

}  // namespace mux
