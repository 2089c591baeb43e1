/*
 * mux_diag.h -- diagnostics of the multiplexed PEFT linear layer library: per-kernel timing, probes of what the box
 * sustains, and the switches that turn parts of the backbone GEMM off for measurement.  Nothing here is needed to
 * use the layer (mux.h); benchmarks and tests use it.
 *
 * Environment variables, all read once per process, for measurement and testing only:
 *   MUX_GEMM_REGSTAGED         run the backbone product (Eq. 1, Eq. 2) through the register-staged kernel also on
 *                              the shapes the pipelined kernel takes;
 *   MUX_GEMM_BK32              the pipelined kernel uses 32-deep stages everywhere;
 *   MUX_GEMM_NO_HALF_TILES     it keeps the tiles of the last round whole;
 *   MUX_GEMM_NO_QUARTER_TILES  it splits them into halves where it would take quarters;
 *   MUX_GEMM_FUSE_DOWN=0       the forward never forms Hs = s_t X A_t inside the backbone tile loop (by default it
 *                              does in launches of quarter tiles, LoRA ranks up to 32 that are multiples of 8, no
 *                              Adapter-Tuning task); =2: in launches of half tiles as well.
 */
#ifndef MUX_DIAG_H_
#define MUX_DIAG_H_

#include "mux.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Per-kernel timing for benchmarks.  While enabled (on = 1: every kernel, on = 2: only the
 * backbone GEMM kernels, on = 0: off), each such launch is bracketed by two HIP events
 * recorded on the launch stream (no synchronisation is added; an event pair costs a few
 * microseconds of stream time, which is why mode 2 exists).
 * mux_profile_collect waits for the recorded events, fills up to `cap` entries with one line
 * per kernel (name, number of launches, summed duration in milliseconds; for the kernels that only bring partial
 * sums together or write the task table -- the method itself asks for none of their bytes -- the bytes they moved
 * as the library counts them at the launch, else 0), returns the number
 * of distinct kernels in *n, and clears the record.  Process-wide, not thread-safe; leave it
 * disabled under HIP graph capture. */
typedef struct {
  const char* name;   /* static string owned by the library */
  int32_t launches;
  double total_ms;
  double bytes;       /* summed over the launches; 0 where the caller counts the algorithmic bytes itself */
} mux_profile_entry;
mux_status mux_profile_enable(int on);
mux_status mux_profile_collect(mux_profile_entry* host_out, int32_t cap, int32_t* n);

/* Diagnostic for the roofline of the backbone GEMM: what the matrix cores sustain on bf16 operands that stay in
 * registers (two waves per SIMD on every compute unit, independent v_mfma_f32_32x32x16_bf16 back to back).  The
 * clock under such load is set by power, hence by the operand values, so the caller supplies them: `dev_operands`
 * holds mux_probe_mfma_operand_bytes() bytes of bf16 values (device, 16-byte aligned; every wave reads the same),
 * `dev_sink` receives mux_probe_mfma_sink_bytes() bytes of results nobody needs (device).  One launch of `iters`
 * loop turns on `hip_stream`, no synchronisation; *flop (host, may be null) is set to the floating-point
 * operations of the launch, so that the caller's timing gives FLOP/s. */
size_t mux_probe_mfma_operand_bytes(void);
size_t mux_probe_mfma_sink_bytes(void);
mux_status mux_probe_mfma(const void* dev_operands, void* dev_sink, int32_t iters, void* hip_stream, double* flop);

/* Diagnostic for the roofline of the adapter kernels: one plain read stream over `bytes` bytes at `dev_buf` (device,
 * 16-byte aligned; the last bytes % 16 bytes are not read), every 16-byte piece read once, each workgroup walking a
 * contiguous share with eight loads a thread in flight.  `dev_sink` receives mux_probe_read_sink_bytes() bytes nobody needs (device).  One launch on `hip_stream`,
 * no synchronisation; the caller's timing over `bytes` gives the GB/s a read stream reaches on the box. */
size_t mux_probe_read_sink_bytes(void);
mux_status mux_probe_read(const void* dev_buf, size_t bytes, void* dev_sink, void* hip_stream);

/* Clock of the matrix-core kernels as they run.  While a buffer is set (device, four 64-bit words, 8-byte aligned,
 * zeroed by the caller; null switches it off; words 2 and 3 are scratch of the kernels), the first workgroup of every backbone GEMM launch and of
 * mux_probe_mfma adds, when it ends, the shader-clock cycles it ran to word 0 and the ticks of the constant 100 MHz
 * counter over the same span to word 1 (one atomic add each by one thread).  100 MHz * word 0 / word 1 is then the
 * clock the compute unit ran at, averaged over those launches: under dense matrix-core load it is set by the power
 * limit, not by the nominal 2.4 GHz.  Process-wide, not thread-safe. */
mux_status mux_diag_set_clock_buffer(void* dev_four_u64);

#ifdef __cplusplus
}
#endif
#endif /* MUX_DIAG_H_ */
