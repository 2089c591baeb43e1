// Diagnostic kernel: what the matrix cores of this part sustain on bf16 operands that never leave the registers.
// Two waves per SIMD (as in the backbone GEMM), 64 independent v_mfma_f32_32x32x16_bf16 per loop turn over eight
// accumulators, the A operands rotating over eight registers so that consecutive products see different data.
// The clock under dense MFMA load is set by power and therefore by the operand values: zeros, small integers and
// N(0,1) values give different rates, and the GEMM's fraction of the nominal peak reads differently against them.
#include "mux_device_utils.h"

namespace mux {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kProbeBlocks = 512, kProbeThreads = 256;    // 2048 waves: two per SIMD of 256 compute units

__global__ __launch_bounds__(256, 2) void k_probe_mfma(const uint4* __restrict__ operands, float* __restrict__ sink,
                                                       int iters) {
  const int lane = threadIdx.x & 63;
  bf16x8 a[8], b[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = __builtin_bit_cast(bf16x8, operands[i * 64 + lane]);
    b[i] = __builtin_bit_cast(bf16x8, operands[(8 + i) * 64 + lane]);
  }
  f32x16 acc[8];
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int r = 0; r < 8; ++r)
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(j + r) & 7], b[j], acc[j], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) s += acc[j][v];
  sink[(size_t)blockIdx.x * kProbeThreads + threadIdx.x] = s;
}

}  // namespace
}  // namespace mux

using namespace mux;

extern "C" size_t mux_probe_mfma_operand_bytes(void) { return 16 * 64 * sizeof(uint4); }
extern "C" size_t mux_probe_mfma_sink_bytes(void) { return (size_t)kProbeBlocks * kProbeThreads * sizeof(float); }

extern "C" mux_status mux_probe_mfma(const void* dev_operands, void* dev_sink, int32_t iters, void* hip_stream,
                                     double* flop) {
  static const char* fn = "mux_probe_mfma";
  if (!dev_operands || !dev_sink || iters < 1) return fail(MUX_ERR_INVALID_ARG, std::string(fn) + ": null buffer or iters < 1");
  if (((uintptr_t)dev_operands & 15) != 0) return fail(MUX_ERR_UNSUPPORTED, std::string(fn) + ": operands must be 16-byte aligned");
  hipLaunchKernelGGL(k_probe_mfma, dim3(kProbeBlocks), dim3(kProbeThreads), 0, (hipStream_t)hip_stream,
                     (const uint4*)dev_operands, (float*)dev_sink, (int)iters);
  if (flop) *flop = (double)kProbeBlocks * (kProbeThreads / 64) * (double)iters * 64.0 * (2.0 * 32 * 32 * 16);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(MUX_ERR_DEVICE, std::string(fn) + ": " + hipGetErrorString(e));
  return MUX_OK;
}
