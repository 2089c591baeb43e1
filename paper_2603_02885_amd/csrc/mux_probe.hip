// Diagnostic kernels.  First: what the matrix cores of this part sustain on bf16 operands that never leave the registers.
// Two waves per SIMD (as in the backbone GEMM), 64 independent v_mfma_f32_32x32x16_bf16 per loop turn over eight
// accumulators, the A operands rotating over eight registers so that consecutive products see different data.
// The clock under dense MFMA load is set by power and therefore by the operand values: zeros, small integers and
// N(0,1) values give different rates, and the GEMM's fraction of the nominal peak reads differently against them.
// Second: what a plain read stream over a large buffer draws from HBM, the yardstick of the adapter kernels.
#include "mux_device_utils.h"

namespace mux {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kProbeBlocks = 512, kProbeThreads = 256;    // 2048 waves: two per SIMD of 256 compute units

__global__ __launch_bounds__(256, 2) void k_probe_mfma(const uint4* __restrict__ operands, float* __restrict__ sink,
                                                       int iters, unsigned long long* __restrict__ clk) {
  const int lane = threadIdx.x & 63;
  const bool stamp = clk != nullptr && blockIdx.x == 0 && threadIdx.x == 0;
  if (stamp) { clk[2] = clock64(); clk[3] = wall_clock64(); }
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
  if (stamp) {
    atomicAdd(clk, (unsigned long long)clock64() - clk[2]);
    atomicAdd(clk + 1, (unsigned long long)wall_clock64() - clk[3]);
  }
}

// Read stream: a workgroup sums the 16-byte pieces of its own contiguous share of the buffer, 4 KB per wave
// instruction group and eight such groups in flight (of the variants tried -- shares against grid-wide strides, 4 to
// 16 loads in flight, 1024 to 65536 workgroups, non-temporal loads -- the fastest on this part by 5 to 25 %).
constexpr int kReadBlocks = 2048, kReadThreads = 256;
__global__ __launch_bounds__(256) void k_probe_read(const uint4* __restrict__ src, size_t n_vec, uint32_t* __restrict__ sink) {
  const size_t per = (n_vec + gridDim.x - 1) / gridDim.x;
  const size_t b0 = (size_t)blockIdx.x * per, b1 = b0 + per < n_vec ? b0 + per : n_vec;
  uint32_t s = 0;
  size_t i = b0 + threadIdx.x;
  for (; i + 7 * kReadThreads < b1; i += 8 * kReadThreads) {
    uint4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = src[i + u * kReadThreads];
#pragma unroll
    for (int u = 0; u < 8; ++u) s += v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  for (; i < b1; i += kReadThreads) {
    const uint4 v = src[i];
    s += v.x ^ v.y ^ v.z ^ v.w;
  }
  sink[(size_t)blockIdx.x * kReadThreads + threadIdx.x] = s;
}

}  // namespace
}  // namespace mux

using namespace mux;

extern "C" size_t mux_probe_read_sink_bytes(void) { return (size_t)kReadBlocks * kReadThreads * sizeof(uint32_t); }

extern "C" mux_status mux_probe_read(const void* dev_buf, size_t bytes, void* dev_sink, void* hip_stream) {
  static const char* fn = "mux_probe_read";
  if (!dev_buf || !dev_sink || bytes < 16) return fail(MUX_ERR_INVALID_ARG, std::string(fn) + ": null buffer or fewer than 16 bytes");
  if (((uintptr_t)dev_buf & 15) != 0) return fail(MUX_ERR_UNSUPPORTED, std::string(fn) + ": the buffer must be 16-byte aligned");
  hipLaunchKernelGGL(k_probe_read, dim3(kReadBlocks), dim3(kReadThreads), 0, (hipStream_t)hip_stream,
                     (const uint4*)dev_buf, bytes / 16, (uint32_t*)dev_sink);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(MUX_ERR_DEVICE, std::string(fn) + ": " + hipGetErrorString(e));
  return MUX_OK;
}

extern "C" size_t mux_probe_mfma_operand_bytes(void) { return 16 * 64 * sizeof(uint4); }
extern "C" size_t mux_probe_mfma_sink_bytes(void) { return (size_t)kProbeBlocks * kProbeThreads * sizeof(float); }

extern "C" mux_status mux_probe_mfma(const void* dev_operands, void* dev_sink, int32_t iters, void* hip_stream,
                                     double* flop) {
  static const char* fn = "mux_probe_mfma";
  if (!dev_operands || !dev_sink || iters < 1) return fail(MUX_ERR_INVALID_ARG, std::string(fn) + ": null buffer or iters < 1");
  if (((uintptr_t)dev_operands & 15) != 0) return fail(MUX_ERR_UNSUPPORTED, std::string(fn) + ": operands must be 16-byte aligned");
  hipLaunchKernelGGL(k_probe_mfma, dim3(kProbeBlocks), dim3(kProbeThreads), 0, (hipStream_t)hip_stream,
                     (const uint4*)dev_operands, (float*)dev_sink, (int)iters, diag_clock_buffer());
  if (flop) *flop = (double)kProbeBlocks * (kProbeThreads / 64) * (double)iters * 64.0 * (2.0 * 32 * 32 * 16);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(MUX_ERR_DEVICE, std::string(fn) + ": " + hipGetErrorString(e));
  return MUX_OK;
}
