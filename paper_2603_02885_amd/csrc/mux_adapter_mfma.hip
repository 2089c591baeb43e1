// Adapter kernels on the matrix cores (bf16 in, fp32 accumulate).  All of them stream a big
// activation matrix once from HBM and are bound by that stream; the MFMA only keeps the
// arithmetic (r FLOP per byte) off the vector ALUs.
//
//   down:  Out[T,RP] = s_t * In[T,C] P_t^T      S1: In = X,  P_t^T = A_t as it is ([K][r], ranks that are multiples
//                                               of 8) or P_t = A_t^T from the transposed region ([r][K])
//   s4:    one pass over dY for both of its products (the adapter's backward is computed "in a fused manner",
//          section 3.2): per (row group, 512-column slab) the slab's share of dY B_t^T (summed over the slabs and scaled
//          by gs_reduce -> Gs[T,RP]) and the row group's share of Hs^T dY (summed over the row groups by reduce -> dB_t)
//   grad:  part[item][r][C] = sum_{rows of item} Small[i][:]^T Big[i][:]
//                                               S6: Small = Gs, Big = X   -> dA_t[K][r] (transposed on reduce)
//   dl:    part[item][N] = sum_{rows of item} dY[i][:] * Z[i][:]          (IA3_OUT)
//   reduce: per task, partials summed in ascending item order (deterministic), optional accumulate.
//
// Padding rows are masked with out-of-range buffer offsets (the load returns zeros), never multiplied.
#include <type_traits>

#include "mux_device_utils.h"

namespace mux {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __amdgpu_buffer_rsrc_t rsrc_t;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
constexpr uint32_t OOB = 0x80000000u;
constexpr int TS64 = 0, TS256 = 2, TS1024 = 3;

__device__ __forceinline__ rsrc_t make_rsrc(const void* p, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc((void*)p, 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ u32x4 buf_load16(rsrc_t r, uint32_t byte_off) {
  return __builtin_amdgcn_raw_buffer_load_b128(r, (int)byte_off, 0, 0);
}
__device__ __forceinline__ bf16x4 lds_read_tr(const bf16_t* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4bf16((__attribute__((address_space(3))) bf16x4*)p);
}
__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// Validity bits of the rows of a row group of up to 1024 rows, fetched once: lane l keeps the 32-bit word that holds
// row row0 + 32 l (and the one after it); step s of the group then takes its 32 bits from lanes with two lane reads
// instead of a memory access of its own, on which the step's loads would have to wait.
struct GroupBits { uint32_t lo, hi; int sh; };
__device__ __forceinline__ GroupBits load_group_bits(const int32_t* __restrict__ dtab, int rowbits_off, int row0, int nrows, int T, int lane) {
  const uint32_t* bm = (const uint32_t*)(dtab + rowbits_off);
  const int w0 = row0 >> 5;
  const int last = (T + 31) >> 5;                        // the spare word after the last one exists
  const int nw = ((nrows + 31) >> 5) + 1;
  GroupBits g;
  g.lo = (lane < nw && w0 + lane <= last) ? bm[w0 + lane] : 0u;
  g.hi = (lane < nw && w0 + lane + 1 <= last) ? bm[w0 + lane + 1] : 0u;
  g.sh = row0 & 31;
  return g;
}
__device__ __forceinline__ uint32_t step_bits(const GroupBits& g, int s) {
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)g.lo, s), hi = (uint32_t)__builtin_amdgcn_readlane((int)g.hi, s);
  return (uint32_t)((((uint64_t)hi << 32) | lo) >> g.sh);
}

// ------------------------------------------------------------------------------------------------
// down-projection.  One workgroup = 32 rows of one 64-row item; its waves split the contraction.
// A wave walks its share 64 columns at a time: the 32x64 slab of In and the rank x 64 slab of P_t are fetched with
// loads that cover whole 128-byte lines (8 rows x 128 B per wave instruction: rows of 64 B move at half the rate
// on this memory system), two slabs ahead in registers, pass through a wave-private LDS region in their natural
// layout and come back in the 16x16x32 MFMA operand layout.  No workgroup barrier in the loop.  The partial sums
// of the waves are combined through LDS in a fixed order.
//   DOWN_X     LoRA items: Out = s_t X A_t; rows of other kinds: zero.  NAT: A_t is read as it is, [K][r] with r a
//              multiple of 8 -- the 64 rows of a slab are one contiguous run of 128 r bytes, laid into LDS row by row
//              and read back with the contraction index contiguous through ds_read_b64_tr_b16; else P_t = A_t^T from
//              the transposed region.
//   DOWN_TUNE  TUNING items only (other rows are left alone): u = z D_t with z from the saved compact rows and
//              P_t = D_t^T from the transposed region; U2 = u, Out = s_t gelu(u)
// The work item and the validity bits of its rows come from two lists whose offsets are launch arguments, so the
// first loads of X wait for one memory latency, not for a chain of them.
enum : int { DOWN_X = 0, DOWN_TUNE = 2 };
struct DownParams {
  const int32_t* dtab;
  const bf16_t* In;    // [T, C]  (DOWN_TUNE: [z_rows, C], rows numbered like the saved x W)
  bf16_t* Out;         // [T, RP]
  const bf16_t* AT;    // base of the transposed region (null with NAT)
  bf16_t* U2;          // [T, RP] pre-activations of the TUNING rows: written by DOWN_TUNE
  int C, RP, mode;
  int items_off, bits_off;   // word offsets in dtab: 64-row items, and two words of row-validity bits per item
  TaskRef tasks;
};

__device__ __forceinline__ float gelu_f(float u) { return 0.5f * u * (1.f + erff(u * 0.70710678f)); }
__device__ __forceinline__ float gelu_slope_f(float u) {
  return 0.5f * (1.f + erff(u * 0.70710678f)) + u * __expf(-0.5f * u * u) * 0.39894228f;
}

constexpr int GP = 72;   // LDS row pitch in elements (144 B): 16 consecutive rows of one 16-byte piece hit 64 different banks

template <int NJM, int NWV, int DEPTH, bool NAT>
__global__ __launch_bounds__(64 * NWV) void k_down(const DownParams p) {
  constexpr int ROWS = 32, NTHR = 64 * NWV;
  constexpr int PP = NJM * 16 + 8;                              // NAT: LDS pitch of the [64][r] slab of A_t (elements)
  constexpr int PSLAB = NAT ? 64 * PP : NJM * 16 * GP;
  constexpr int SLAB = ROWS * GP + PSLAB;                      // elements per wave: In slab, then P slab
  constexpr int REDW = NJM * 16 * (ROWS + 4) * 2;              // the same region later holds the partial sums (floats)
  constexpr int REGION = SLAB > REDW ? SLAB : REDW;
  __shared__ __attribute__((aligned(16))) bf16_t lds[NWV][REGION];
  const int item = blockIdx.x >> 1, sub = blockIdx.x & 1;
  const int4 iw = *(const int4*)(p.dtab + p.items_off + item * DI_WORDS);
  const uint32_t vbits = ((const uint32_t*)(p.dtab + p.bits_off))[2 * item + sub];
  const ItemView it = {iw.x, iw.y, iw.z, iw.w};
  const int r0 = sub * ROWS;
  if (r0 >= it.nrows) return;
  const int nr = it.nrows - r0 < ROWS ? it.nrows - r0 : ROWS;
  const int row0 = it.row0 + r0;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int kind = it.task >= 0 ? get_task_kind(p.tasks, it.task) : MUX_ADAPTER_NONE;
  const bool mine = p.mode == DOWN_TUNE ? kind == MUX_ADAPTER_TUNING : kind == MUX_ADAPTER_LORA;
  if (!mine && p.mode == DOWN_TUNE) return;
  if (!mine || vbits == 0u) {
    for (int e = tid; e < nr * p.RP; e += NTHR) {
      const size_t o = (size_t)(row0 + e / p.RP) * p.RP + e % p.RP;
      p.Out[o] = 0;
      if (p.mode == DOWN_TUNE) p.U2[o] = 0;
    }
    return;
  }
  const DevTask tk = get_task(p.tasks, it.task);
  const int rank = tk.rank, NJ = (rank + 15) >> 4;
  const bf16_t* P = NAT ? (const bf16_t*)tk.A : p.AT + tk.at_off;
  const int prow = NJ * 16;                          // rows that exist in a transposed P

  const int per = ((p.C + NWV - 1) / NWV + 63) & ~63;
  const int cbeg = wave * per, cend = cbeg + per < p.C ? cbeg + per : p.C;
  bf16_t* sX = lds[wave];
  bf16_t* sP = lds[wave] + ROWS * GP;

  const size_t in_row0 = p.mode == DOWN_TUNE ? (size_t)(tk.zrow0 + row0 - tk.row_begin) : (size_t)row0;
  const rsrc_t rIn = make_rsrc(p.In + in_row0 * p.C, (uint32_t)nr * (uint32_t)p.C * 2u);
  const rsrc_t rP = make_rsrc(P, (NAT ? (uint32_t)p.C * (uint32_t)rank : (uint32_t)prow * (uint32_t)p.C) * 2u);
  // one wave instruction: 8 rows x 128 B; lane -> row lane/8 (+ 8 q), 16-byte piece lane%8
  const int b_row = lane >> 3, b_pc = (lane & 7) * 8;
  uint32_t x_off[4], p_off[2 * NJM];
  int p_lds[2 * NJM];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int m = b_row + 8 * q;
    x_off[q] = (m < nr && ((vbits >> m) & 1u)) ? ((uint32_t)m * (uint32_t)p.C + (uint32_t)b_pc) * 2u : OOB;
  }
  if (NAT) {
    // the [64][rank] slab is 8 rank 16-byte pieces in a row; piece -> (row, piece of the row)
    const int ppr = rank >> 3;
#pragma unroll
    for (int q = 0; q < 2 * NJM; ++q) {
      const int piece = q * 64 + lane;
      p_off[q] = q < ppr ? (uint32_t)piece * 16u : OOB;
      p_lds[q] = (piece / ppr) * PP + (piece % ppr) * 8;
    }
    // columns of the LDS slab beyond the rank are never written: they read as zero
    for (int e = lane; e < 64 * (PP / 8); e += 64) *(u32x4*)(sP + (e / (PP / 8)) * PP + (e % (PP / 8)) * 8) = (u32x4){0u, 0u, 0u, 0u};
  } else {
#pragma unroll
    for (int q = 0; q < 2 * NJM; ++q) {
      const int j = b_row + 8 * q;
      p_off[q] = (q < 2 * NJ && j < prow) ? ((uint32_t)j * (uint32_t)p.C + (uint32_t)b_pc) * 2u : OOB;
      p_lds[q] = j * GP + b_pc;
    }
  }

  f32x4 acc[2][NJM];
#pragma unroll
  for (int rt = 0; rt < 2; ++rt)
#pragma unroll
    for (int jt = 0; jt < NJM; ++jt) acc[rt][jt] = (f32x4){0.f, 0.f, 0.f, 0.f};

  u32x4 gx[DEPTH][4], gp[DEPTH][2 * NJM];
  // Every slab issues the same number of loads, whatever the rank and wherever the share ends (a piece that does not
  // exist gets an out-of-range offset, costs no memory access and reads as zeros): the compiler can then count the
  // loads still in flight when it waits for a slab, instead of waiting for all of them.
  auto load = [&](int c, int buf) {          // a slab that starts past the end of this wave's share reads as zeros
    const bool in = c < cend;                 // the share ends on a multiple of 64 or at C, where the buffer ends
    const uint32_t kx = (c + b_pc < cend) ? (uint32_t)c * 2u : OOB;     // OOB + OOB wraps into range: mask on k only
    const uint32_t kp = in ? (NAT ? (uint32_t)c * (uint32_t)rank * 2u : (uint32_t)c * 2u) : OOB;
#pragma unroll
    for (int q = 0; q < 4; ++q) gx[buf][q] = buf_load16(rIn, (x_off[q] == OOB || kx == OOB) ? OOB : x_off[q] + kx);
#pragma unroll
    for (int q = 0; q < 2 * NJM; ++q) {
      const bool ok = p_off[q] != OOB && kp != OOB && (NAT || c + b_pc < cend);
      gp[buf][q] = buf_load16(rP, ok ? p_off[q] + kp : OOB);
    }
  };
  const int i = lane & 15, g = lane >> 4;
  const int tr_off = (8 * g + (i >> 2)) * PP + 4 * (i & 3);     // NAT: transposed reads of the [k][j] slab
  // DEPTH slabs in flight while one is multiplied
#pragma unroll
  for (int d = 0; d < DEPTH; ++d) {
    load(cbeg + 64 * d, d);
    __builtin_amdgcn_sched_barrier(0);       // in the order in which the loop uses them
  }
  for (int c = cbeg; c < cend; c += 64 * DEPTH) {
#pragma unroll
    for (int buf = 0; buf < DEPTH; ++buf) {
      {                                      // also for a slab past the end (zeros): no branch around the loads
#pragma unroll
        for (int q = 0; q < 4; ++q) *(u32x4*)(sX + (b_row + 8 * q) * GP + b_pc) = gx[buf][q];
#pragma unroll
        for (int q = 0; q < 2 * NJM; ++q)
          if (NAT ? (q * 8 < rank) : (q < 2 * NJ)) *(u32x4*)(sP + p_lds[q]) = gp[buf][q];
        load(c + 64 * buf + 64 * DEPTH, buf);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        bf16x8 a[2][2], b[NJM][2];
#pragma unroll
        for (int s = 0; s < 2; ++s) {
#pragma unroll
          for (int rt = 0; rt < 2; ++rt) a[rt][s] = *(const bf16x8*)(sX + (rt * 16 + i) * GP + s * 32 + 8 * g);
#pragma unroll
          for (int jt = 0; jt < NJM; ++jt)
            if (jt < NJ) {
              if (NAT) {
                const bf16x4 lo = lds_read_tr(sP + s * 32 * PP + tr_off + jt * 16);
                const bf16x4 hi = lds_read_tr(sP + s * 32 * PP + tr_off + 4 * PP + jt * 16);
                b[jt][s] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
              } else {
                b[jt][s] = *(const bf16x8*)(sP + (jt * 16 + i) * GP + s * 32 + 8 * g);
              }
            }
        }
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
          for (int rt = 0; rt < 2; ++rt)
#pragma unroll
            for (int jt = 0; jt < NJM; ++jt)
              if (jt < NJ) acc[rt][jt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[rt][s], b[jt][s], acc[rt][jt], 0, 0, 0);
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        __builtin_amdgcn_wave_barrier();
      }
    }
  }

  // acc[rt][jt][v] = partial of Out[row0 + rt*16 + 4g + v][jt*16 + i]; staged column-major, one 16-byte store each
  float* red = (float*)lds[wave];
#pragma unroll
  for (int rt = 0; rt < 2; ++rt)
#pragma unroll
    for (int jt = 0; jt < NJM; ++jt)
      if (jt < NJ) *(f32x4*)&red[(jt * 16 + i) * (ROWS + 4) + rt * 16 + 4 * g] = acc[rt][jt];
  __syncthreads();
  for (int e = tid; e < ROWS * p.RP; e += NTHR) {
    const int orow = e / p.RP, j = e % p.RP;
    if (orow >= nr) continue;
    float s = 0.f;
    if (j < NJ * 16) {
#pragma unroll
      for (int w = 0; w < NWV; ++w) s += ((const float*)lds[w])[j * (ROWS + 4) + orow];
    }
    const bool ok = ((vbits >> orow) & 1u) && j < rank;
    const size_t o = (size_t)(row0 + orow) * p.RP + j;
    float v = ok ? tk.scale * s : 0.f;
    if (p.mode == DOWN_TUNE) {
      p.U2[o] = f32_to_bf16(ok ? s : 0.f);
      v = ok ? tk.scale * gelu_f(s) : 0.f;
    }
    p.Out[o] = f32_to_bf16(v);
  }
}

template <bool NAT>
void launch_down_t(const CallCtx& c, const char* name, const DownParams& p) {
  const unsigned items = (unsigned)c.st->items[TS64].size();
  // eight waves split the contraction (four for ranks above 32, whose LDS regions are larger); two slabs in flight
  if (c.st->r_max <= 16) MUX_LAUNCH(name, (k_down<1, 8, 2, NAT>), dim3(items * 2), dim3(512), 0, c.stream, p);
  else if (c.st->r_max <= 32) MUX_LAUNCH(name, (k_down<2, 8, 2, NAT>), dim3(items * 2), dim3(512), 0, c.stream, p);
  else MUX_LAUNCH(name, (k_down<4, 4, 2, NAT>), dim3(items * 2), dim3(256), 0, c.stream, p);
}
void launch_down(const CallCtx& c, const char* name, DownParams p, bool natural) {
  p.items_off = c.st->dev_image[DH_NITEMS0 + 3 * TS64 + 1];
  p.bits_off = c.st->dev_image[DH_OFF_ITEM_BITS];
  p.tasks = *c.tref;
  if (natural) launch_down_t<true>(c, name, p);
  else launch_down_t<false>(c, name, p);
}

// ------------------------------------------------------------------------------------------------
// The pass over dY of the backward (LoRA: Gs = s_t dY B_t^T and dB_t = Hs^T dY; Adapter-Tuning: the same two products
// with U_t in the place of B_t).  grid = (row groups of the chosen size, ceil(N / 512)); each of the eight waves owns
// 64 columns and walks the group's rows 32 at a time: the 32x64 slab of dY and the 32xRP slab of Hs go through a
// wave-private LDS region; dY is read from it twice, row-major as the A operand of the slab's share of dY B_t^T
// (B_t's [r][64] piece stays in registers for the whole group), and with the rows contiguous, through
// ds_read_b64_tr_b16, as the B operand of Hs^T dY, whose sums stay in the accumulators until the group ends.
// The shares of dY B_t^T of the eight waves are added up through LDS (two barriers a step) and go out as one fp32
// partial per (column slab, row); k_gs_reduce adds the slabs.
struct S4Params {
  const int32_t* dtab;
  const bf16_t* dY;     // [T, N]
  const bf16_t* Hs;     // [T, RP]
  float* gpart;         // [n_slabs][T][RP]: dY B_t^T over the columns of one slab, unscaled
  float* bpart;         // [n_items][RP][N]: Hs^T dY over the rows of one group
  int N, RP, ts, T;
  int items_off, rowbits_off;   // word offsets in dtab of the row-group list and of the row-validity bits
  TaskRef tasks;
};

// BATCH: steps whose shares of dY B_t^T wait in registers before the waves meet to add them up; DEPTH: steps of loads
// in flight.  The loop body has no branch and a fixed number of loads and stores per step (what does not exist gets an
// out-of-range offset), so that the waits for one step's data leave the younger loads in flight.
__device__ __forceinline__ void buf_store4(rsrc_t r, uint32_t byte_off, float v) {
  __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned int, v), r, (int)byte_off, 0, 0);
}
__device__ __forceinline__ void lds_barrier() {     // LDS traffic of every wave done; loads from memory stay in flight
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(0xC07F);               // lgkmcnt(0)
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

template <int NJM, int BATCH, int DEPTH>
__global__ __launch_bounds__(512) void k_s4(const S4Params p) {
  constexpr int NWV = 8, NTHR = 512, BROWS = BATCH * 32, RPITCH = BROWS + 4;   // RPITCH: floats between two columns of a staged share
  constexpr int UNR = BATCH > DEPTH ? BATCH : DEPTH;
  constexpr int RPJ = NJM * 16;                                   // columns of a staged share
  constexpr int NRED = BROWS * RPJ / NTHR;                        // sums a thread forms when the waves meet
  static_assert(RPJ * RPITCH * 4 <= 2 * 32 * GP * 2, "a wave's share of dY B_t^T fits its own LDS region");
  static_assert(UNR % BATCH == 0 && UNR % DEPTH == 0 && BROWS * RPJ % NTHR == 0, "powers of two");
  __shared__ __attribute__((aligned(16))) bf16_t lds[NWV][2][32 * GP];
  const int4 iw = *(const int4*)(p.dtab + p.items_off + blockIdx.x * DI_WORDS);   // the lists' offsets are launch arguments:
  const ItemView it = {iw.x, iw.y, iw.z, iw.w};                                    // one memory latency before the first load
  if (it.task < 0 || it.nvalid == 0) return;
  const DevTask tk = get_task(p.tasks, it.task);
  if (tk.kind != MUX_ADAPTER_LORA && tk.kind != MUX_ADAPTER_TUNING) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int cw0 = blockIdx.y * (64 * NWV) + wave * 64;           // may lie beyond N: such a wave adds zeros
  const int rank = tk.rank, NJ = (rank + 15) >> 4;
  bf16_t* sBig = lds[wave][0];
  bf16_t* sSm = lds[wave][1];

  const rsrc_t rB = make_rsrc(p.dY + (size_t)it.row0 * p.N, (uint32_t)it.nrows * (uint32_t)p.N * 2u);
  const rsrc_t rS = make_rsrc(p.Hs + (size_t)it.row0 * p.RP, (uint32_t)it.nrows * (uint32_t)p.RP * 2u);
  const rsrc_t rP = make_rsrc(tk.B, (uint32_t)rank * (uint32_t)p.N * 2u);
  // the partial sums of this slab for the rows of this group
  const rsrc_t rG = make_rsrc(p.gpart + ((size_t)blockIdx.y * p.T + it.row0) * p.RP, (uint32_t)it.nrows * (uint32_t)p.RP * 4u);
  const int b_row = lane >> 3, b_pc = (lane & 7) * 8;
  const bool b_col_ok = cw0 + b_pc < p.N;
  const int ppr = p.RP >> 3;                   // 16-byte pieces in a row of Hs; RP <= 16 NJM, so a lane loads at most NJM of them
  const int l16 = lane & 15, g = lane >> 4;

  // B_t[j][columns of this wave], as the B operand of dY B_t^T: lane (j = l16, g) holds 8 consecutive columns
  bf16x8 bt[NJM][2];
#pragma unroll
  for (int jt = 0; jt < NJM; ++jt)
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      const int j = jt * 16 + l16, col = cw0 + s * 32 + 8 * g;
      bt[jt][s] = as_bf16x8(buf_load16(rP, (j < rank && col < p.N) ? (uint32_t)(((size_t)j * p.N + col) * 2) : OOB));
    }

  u32x4 gb[DEPTH][4], gs[DEPTH][NJM];
  const int steps = (it.nrows + 31) >> 5;
  const GroupBits gbits = load_group_bits(p.dtab, p.rowbits_off, it.row0, it.nrows, p.T, lane);
  // per-lane pieces of the Hs slab: idx = lane + 64 q -> row idx / ppr, piece idx % ppr
  int s_row[NJM], s_pc[NJM];
#pragma unroll
  for (int q = 0; q < NJM; ++q) { const int idx = lane + 64 * q; s_row[q] = idx / ppr; s_pc[q] = (idx % ppr) * 8; }
  auto load_step = [&](int s, int buf) {       // a step past the end loads nothing (every offset out of range)
    const int base = s * 32;
    const uint32_t vbits = s < steps ? step_bits(gbits, s) : 0u;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int m = base + b_row + 8 * q;
      const bool ok = b_col_ok && m < it.nrows && ((vbits >> (b_row + 8 * q)) & 1u);
      gb[buf][q] = buf_load16(rB, ok ? (uint32_t)(((size_t)m * p.N + cw0 + b_pc) * 2) : OOB);
    }
#pragma unroll
    for (int q = 0; q < NJM; ++q) {
      const int m = base + s_row[q];
      const bool ok = s < steps && s_row[q] < 32 && m < it.nrows;
      gs[buf][q] = buf_load16(rS, ok ? (uint32_t)((m * p.RP + s_pc[q]) * 2) : OOB);
    }
  };
  auto store_step = [&](int buf) {
#pragma unroll
    for (int q = 0; q < 4; ++q) *(u32x4*)(sBig + (b_row + 8 * q) * GP + b_pc) = gb[buf][q];
#pragma unroll
    for (int q = 0; q < NJM; ++q)
      if (s_row[q] < 32) *(u32x4*)(sSm + s_row[q] * GP + s_pc[q]) = gs[buf][q];
  };

  f32x4 accb[NJM][4];
#pragma unroll
  for (int jt = 0; jt < NJM; ++jt)
#pragma unroll
    for (int ct = 0; ct < 4; ++ct) accb[jt][ct] = (f32x4){0.f, 0.f, 0.f, 0.f};
  f32x4 accg[BATCH][2][NJM];

  const int tr_off = (8 * g + (l16 >> 2)) * GP + 4 * (l16 & 3);
  float* red = (float*)lds[wave];
#pragma unroll
  for (int d = 0; d < DEPTH; ++d) load_step(d, d);
  for (int s0 = 0; s0 < steps; s0 += UNR) {
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int s = s0 + u;                       // may run past the last step: zeros in, nothing out
      store_step(u % DEPTH);
      load_step(s + DEPTH, u % DEPTH);
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      {
        // the slab's share of dY B_t^T first, one 16-row half at a time (its operands are dead before the next are read)
#pragma unroll
        for (int rt = 0; rt < 2; ++rt) {
          bf16x8 ay[2];
#pragma unroll
          for (int ks = 0; ks < 2; ++ks) ay[ks] = *(const bf16x8*)(sBig + (rt * 16 + l16) * GP + ks * 32 + 8 * g);
#pragma unroll
          for (int jt = 0; jt < NJM; ++jt) {
            f32x4 v = (f32x4){0.f, 0.f, 0.f, 0.f};
            if (jt < NJ)
#pragma unroll
              for (int ks = 0; ks < 2; ++ks) v = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ay[ks], bt[jt][ks], v, 0, 0, 0);
            accg[u % BATCH][rt][jt] = v;
          }
        }
        bf16x8 a[NJM];
#pragma unroll
        for (int jt = 0; jt < NJM; ++jt) {
          const bf16x4 lo = lds_read_tr(sSm + tr_off + jt * 16), hi = lds_read_tr(sSm + tr_off + 4 * GP + jt * 16);
          a[jt] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        }
#pragma unroll
        for (int ct = 0; ct < 4; ++ct) {
          const bf16x4 lo = lds_read_tr(sBig + tr_off + ct * 16), hi = lds_read_tr(sBig + tr_off + 4 * GP + ct * 16);
          const bf16x8 b = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
          for (int jt = 0; jt < NJM; ++jt)
            if (jt < NJ) accb[jt][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[jt], b, accb[jt][ct], 0, 0, 0);
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      if ((u % BATCH) == BATCH - 1) {
        // The waves meet: accg[bi][rt][jt][v] = this wave's share of (dY B_t^T)[row of the batch 32 bi + 16 rt + 4 g + v]
        // [16 jt + l16], staged over the slabs just read, added up in wave order, one fp32 partial per row and column out.
#pragma unroll
        for (int bi = 0; bi < BATCH; ++bi)
#pragma unroll
          for (int rt = 0; rt < 2; ++rt)
#pragma unroll
            for (int jt = 0; jt < NJM; ++jt) *(f32x4*)&red[(jt * 16 + l16) * RPITCH + bi * 32 + rt * 16 + 4 * g] = accg[bi][rt][jt];
        lds_barrier();
        const int base = (s - (BATCH - 1)) * 32;                // first row of the batch inside the group
#pragma unroll
        for (int i = 0; i < NRED; ++i) {
          const int e = tid + NTHR * i, m = e / RPJ, j = e % RPJ;
          float v = 0.f;
#pragma unroll
          for (int w = 0; w < NWV; ++w) v += ((const float*)lds[w])[j * RPITCH + m];
          const bool ok = base + m < it.nrows && j < 16 * NJ;     // (the reduction reads the task's rank pieces only)
          buf_store4(rG, ok ? (uint32_t)(((base + m) * p.RP + j) * 4) : OOB, v);
        }
        lds_barrier();
      }
    }
  }
  if (cw0 >= p.N) return;
  // accb[jt][ct][v] = bpart[j = jt*16 + 4g + v][c = cw0 + ct*16 + l16]
  float* dst = p.bpart + (size_t)blockIdx.x * ((size_t)p.RP * p.N);
#pragma unroll
  for (int jt = 0; jt < NJM; ++jt)
    if (jt < NJ)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int j = jt * 16 + 4 * g + v;
        if (j < rank)
#pragma unroll
          for (int ct = 0; ct < 4; ++ct) {
            const int c = cw0 + ct * 16 + l16;
            if (c < p.N) dst[(size_t)j * p.N + c] = accb[jt][ct][v];
          }
      }
}

// Gs[T,RP] = s_t * (sum over the column slabs of the shares k_s4 left, ascending), times gelu'(u) for the TUNING rows;
// zero on padding rows, beyond the rank and on the rows of the other kinds.  One workgroup per 64-row item.
__global__ __launch_bounds__(256) void k_gs_reduce(const int32_t* __restrict__ dtab, const TaskRef tasks,
                                                  const float* __restrict__ gpart, int n_slabs, int T, int RP,
                                                  const bf16_t* __restrict__ U2, bf16_t* __restrict__ Gs, int items_off,
                                                  int bits_off) {
  const int item = blockIdx.x;
  const int4 iw = *(const int4*)(dtab + items_off + item * DI_WORDS);
  const uint32_t* bw = (const uint32_t*)(dtab + bits_off) + 2 * item;
  const uint32_t bits0 = bw[0], bits1 = bw[1];
  const int task = iw.x, row0 = iw.y, nrows = iw.z;
  const int kind = task >= 0 ? get_task_kind(tasks, task) : MUX_ADAPTER_NONE;
  const bool mine = (kind == MUX_ADAPTER_LORA || kind == MUX_ADAPTER_TUNING) && (bits0 | bits1) != 0u;
  float scale = 0.f;
  int rank = 0;
  if (mine) { const DevTask tk = get_task(tasks, task); scale = tk.scale; rank = tk.rank; }
  const int q4 = RP >> 2;                        // groups of four columns a row
  for (int e = threadIdx.x; e < nrows * q4; e += 256) {
    const int m = e / q4, j = (e % q4) * 4;
    const size_t o = (size_t)(row0 + m) * RP + j;
    const bool valid = mine && (((m < 32 ? bits0 >> m : bits1 >> (m - 32)) & 1u) != 0u) && j < rank;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    if (valid) {
      for (int q = 0; q < n_slabs; q += 4) {     // four slabs in flight; the sum runs in ascending slab order
        float4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
          v[u] = q + u < n_slabs ? *(const float4*)(gpart + ((size_t)(q + u) * T + row0 + m) * RP + j) : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int u = 0; u < 4; ++u) { s.x += v[u].x; s.y += v[u].y; s.z += v[u].z; s.w += v[u].w; }
      }
      s.x *= scale; s.y *= scale; s.z *= scale; s.w *= scale;
      if (kind == MUX_ADAPTER_TUNING) {
        s.x *= gelu_slope_f(bf16_to_f32(U2[o])); s.y *= gelu_slope_f(bf16_to_f32(U2[o + 1]));
        s.z *= gelu_slope_f(bf16_to_f32(U2[o + 2])); s.w *= gelu_slope_f(bf16_to_f32(U2[o + 3]));
      }
      if (j + 1 >= rank) s.y = 0.f;
      if (j + 2 >= rank) s.z = 0.f;
      if (j + 3 >= rank) s.w = 0.f;
    }
    uint2 out;
    out.x = pack_bf16x2(s.x, s.y);
    out.y = pack_bf16x2(s.z, s.w);
    *(uint2*)(Gs + o) = out;
  }
}

// ------------------------------------------------------------------------------------------------
// per-item gradient partial.  grid = (items of the chosen row-group size, ceil(C/256)); each wave owns
// 64 columns and walks the item's rows 32 at a time: the 32x64 slab of Big and the 32xRP slab of Small
// go through a wave-private LDS region in their natural layout and come back k-major per lane through
// ds_read_b64_tr_b16.  No workgroup barrier: the four waves are independent streams.
struct GradParams {     // z0 + blockIdx.z picks the problem: 0 = dB (Small = Hs, Big = dY), 1 = dA (Small = Gs, Big = X)
  const int32_t* dtab;   // TUNING items: 0 = dU_t (the same sum), 1 = dD_t (Small = Gs, Big = the saved z rows, C = N)
  const bf16_t* Small[2];  // [T, RP]
  const bf16_t* Big[2];    // [T, C]
  float* part[2];          // [n_items][slot], a slot holds [RP][C] of the item's kind
  int C[2];
  int RP, ts;
  const bf16_t* Zc;        // saved x W, [z_rows, N]
  size_t slot[2];          // elements per item in part[z]
  int z0;                  // 1: the launch computes the second problem only (the pass over dY has done the first)
  int items_off, rowbits_off, T;   // word offsets in dtab of the row-group list and of the row-validity bits; rows of the batch
  TaskRef tasks;
};

// DEPTH steps of loads in flight; the loop body has no branch and a fixed number of loads per step (what does not
// exist gets an out-of-range offset), so that the wait for one step's data leaves the younger loads in flight.
template <int NJM, int DEPTH>
__global__ __launch_bounds__(256) void k_grad(const GradParams p) {
  __shared__ __attribute__((aligned(16))) bf16_t lds[4][2][32 * GP];
  const int4 iw = *(const int4*)(p.dtab + p.items_off + blockIdx.x * DI_WORDS);
  const ItemView it = {iw.x, iw.y, iw.z, iw.w};
  if (it.task < 0 || it.nvalid == 0) return;
  const DevTask tk = get_task(p.tasks, it.task);
  if (tk.kind != MUX_ADAPTER_LORA && tk.kind != MUX_ADAPTER_TUNING) return;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int z = blockIdx.z + p.z0;
  const bool from_z = z == 1 && tk.kind == MUX_ADAPTER_TUNING;
  const int C = from_z ? p.C[0] : p.C[z];
  const int cw0 = blockIdx.y * 256 + wave * 64;
  if (cw0 >= C) return;
  const int rank = tk.rank, NJ = (rank + 15) >> 4;
  bf16_t* sBig = lds[wave][0];
  bf16_t* sSm = lds[wave][1];

  const bf16_t* big = from_z ? p.Zc + (size_t)(tk.zrow0 + it.row0 - tk.row_begin) * C : p.Big[z] + (size_t)it.row0 * C;
  const rsrc_t rB = make_rsrc(big, (uint32_t)it.nrows * (uint32_t)C * 2u);
  const rsrc_t rS = make_rsrc(p.Small[z] + (size_t)it.row0 * p.RP, (uint32_t)it.nrows * (uint32_t)p.RP * 2u);
  // Big slab: 4 loads per lane, row = 8q + lane/8, 16-byte piece = lane%8
  const int b_row = lane >> 3, b_pc = (lane & 7) * 8;
  const bool b_col_ok = cw0 + b_pc < C;
  // Small slab: pieces per row = RP/8 (RP <= 16 NJM); idx = lane + 64 q -> row = idx / ppr, piece = idx % ppr
  const int ppr = p.RP >> 3;
  int s_row[NJM], s_pc[NJM];
#pragma unroll
  for (int q = 0; q < NJM; ++q) { const int idx = lane + 64 * q; s_row[q] = idx / ppr; s_pc[q] = (idx % ppr) * 8; }

  u32x4 gb[DEPTH][4], gs[DEPTH][NJM];
  const int steps = (it.nrows + 31) >> 5;
  const GroupBits gbits = load_group_bits(p.dtab, p.rowbits_off, it.row0, it.nrows, p.T, lane);
  auto load_step = [&](int s, int buf) {       // a step past the end loads nothing (every offset out of range)
    const int base = s * 32;
    // validity of the 32 rows of this step, wave-uniform, from the words fetched once for the whole group
    const uint32_t vbits = s < steps ? step_bits(gbits, s) : 0u;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int m = base + b_row + 8 * q;
      const bool ok = b_col_ok && m < it.nrows && ((vbits >> (b_row + 8 * q)) & 1u);
      gb[buf][q] = buf_load16(rB, ok ? (uint32_t)(((size_t)m * C + cw0 + b_pc) * 2) : OOB);
    }
#pragma unroll
    for (int q = 0; q < NJM; ++q) {
      const int m = base + s_row[q];
      const bool ok = s < steps && s_row[q] < 32 && m < it.nrows;
      gs[buf][q] = buf_load16(rS, ok ? (uint32_t)((m * p.RP + s_pc[q]) * 2) : OOB);
    }
  };
  auto store_step = [&](int buf) {
#pragma unroll
    for (int q = 0; q < 4; ++q) *(u32x4*)(sBig + (b_row + 8 * q) * GP + b_pc) = gb[buf][q];
#pragma unroll
    for (int q = 0; q < NJM; ++q)
      if (s_row[q] < 32) *(u32x4*)(sSm + s_row[q] * GP + s_pc[q]) = gs[buf][q];
  };

  f32x4 acc[NJM][4];
#pragma unroll
  for (int jt = 0; jt < NJM; ++jt)
#pragma unroll
    for (int ct = 0; ct < 4; ++ct) acc[jt][ct] = (f32x4){0.f, 0.f, 0.f, 0.f};

  const int l16 = lane & 15, g = lane >> 4;
  const int tr_off = (8 * g + (l16 >> 2)) * GP + 4 * (l16 & 3);
#pragma unroll
  for (int d = 0; d < DEPTH; ++d) load_step(d, d);
  for (int s0 = 0; s0 < steps; s0 += DEPTH) {
#pragma unroll
    for (int u = 0; u < DEPTH; ++u) {          // may run past the last step: zeros in
      store_step(u);
      load_step(s0 + u + DEPTH, u);
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      bf16x8 a[NJM], b[4];
#pragma unroll
      for (int jt = 0; jt < NJM; ++jt) {
        const bf16x4 lo = lds_read_tr(sSm + tr_off + jt * 16), hi = lds_read_tr(sSm + tr_off + 4 * GP + jt * 16);
        a[jt] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      }
#pragma unroll
      for (int ct = 0; ct < 4; ++ct) {
        const bf16x4 lo = lds_read_tr(sBig + tr_off + ct * 16), hi = lds_read_tr(sBig + tr_off + 4 * GP + ct * 16);
        b[ct] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      }
#pragma unroll
      for (int jt = 0; jt < NJM; ++jt)
        if (jt < NJ)
#pragma unroll
          for (int ct = 0; ct < 4; ++ct) acc[jt][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[jt], b[ct], acc[jt][ct], 0, 0, 0);
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      __builtin_amdgcn_wave_barrier();
    }
  }
  // acc[jt][ct][v] = part[j = jt*16 + 4g + v][c = cw0 + ct*16 + l16]
  float* dst = p.part[z] + (size_t)blockIdx.x * p.slot[z];
#pragma unroll
  for (int jt = 0; jt < NJM; ++jt)
    if (jt < NJ)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int j = jt * 16 + 4 * g + v;
        if (j < rank)
#pragma unroll
          for (int ct = 0; ct < 4; ++ct) {
            const int c = cw0 + ct * 16 + l16;
            if (c < C) dst[(size_t)j * C + c] = acc[jt][ct][v];
          }
      }
}

// ------------------------------------------------------------------------------------------------
// Adapter-Tuning: Out = In + Small P for the rows of TUNING items, P = [r][N] as stored (forward: U_t, Y = z + Hs U_t,
// In = the saved compact z rows, Out = Y; backward: D_t^T from the transposed region, dYs = dY + Gs D_t^T, In = dY,
// Out = the compact dYs rows).  grid = (64-row items, ceil(N/256)); each wave owns 64 columns: its [r][64] slab of P
// goes through a wave-private LDS region in natural layout and comes back k-major with ds_read_b64_tr_b16; the
// products are staged 16 rows at a time in fp32 so that In is read and Out is written in whole 128-byte lines.
struct TuneAddParams {
  const int32_t* dtab;
  const bf16_t* In;
  const bf16_t* Small;   // [T, RP]
  bf16_t* Out;
  const bf16_t* AT;      // backward: base of the transposed region (D_t^T); forward: null (U_t = tk.B)
  int N, RP, backward;
  int natural;           // backward: D_t [N][r] is read as it is (every rank a multiple of 8), nothing was transposed
  TaskRef tasks;
};

template <int NKS>      // k-steps of 32 over the rank pitch (1 or 2)
__global__ __launch_bounds__(256) void k_tune_add(const TuneAddParams p) {
  constexpr int SP = 68;                                       // fp32 staging pitch
  __shared__ __attribute__((aligned(16))) bf16_t sP[4][NKS * 32 * GP];
  __shared__ __attribute__((aligned(16))) float sC[4][16 * SP];
  const ItemView it = load_item(p.dtab, TS64, blockIdx.x);
  if (it.task < 0 || get_task_kind(p.tasks, it.task) != MUX_ADAPTER_TUNING) return;
  const DevTask tk = get_task(p.tasks, it.task);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int cw0 = blockIdx.y * 256 + wave * 64;
  if (cw0 >= p.N) return;
  const int rank = tk.rank;
  const bf16_t* P = p.backward ? p.AT + tk.at_off : (const bf16_t*)tk.B;
  const int prow = p.backward ? ((rank + 15) & ~15) : rank;
  bf16_t* sp = sP[wave];
  float* sc = sC[wave];

  // P slab [NKS*32][64] -> LDS, natural layout; rows beyond the rank read as zero
  const bool direct = p.backward && p.natural;      // D_t [N][r]: a lane's eight k of one column lie together in memory
  const rsrc_t rP = make_rsrc(P, (uint32_t)prow * (uint32_t)p.N * 2u);
  const int b_row = lane >> 3, b_pc = (lane & 7) * 8;
  if (!direct) {
#pragma unroll
    for (int q = 0; q < NKS * 4; ++q) {
      const int j = b_row + 8 * q;
      const bool ok = j < prow && cw0 + b_pc < p.N;
      const u32x4 v = buf_load16(rP, ok ? (uint32_t)(((size_t)j * p.N + cw0 + b_pc) * 2) : OOB);
      *(u32x4*)(sp + j * GP + b_pc) = v;
    }
  }
  // Small rows in the A-operand layout straight from global memory: row = 16 rt + lane%16, k = 32 ks + 8 (lane/16)
  const int i = lane & 15, g = lane >> 4;
  const rsrc_t rS = make_rsrc(p.Small + (size_t)it.row0 * p.RP, (uint32_t)it.nrows * (uint32_t)p.RP * 2u);
  bf16x8 a[4][NKS];
#pragma unroll
  for (int rt = 0; rt < 4; ++rt)
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
      const int m = rt * 16 + i, k = ks * 32 + 8 * g;
      a[rt][ks] = as_bf16x8(buf_load16(rS, (m < it.nrows && k < p.RP) ? (uint32_t)((m * p.RP + k) * 2) : OOB));
    }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  const int tr_off = (8 * g + (i >> 2)) * GP + 4 * (i & 3);
  bf16x8 b[4][NKS];
  if (direct) {
    const rsrc_t rD = make_rsrc(tk.A, (uint32_t)p.N * (uint32_t)rank * 2u);
#pragma unroll
    for (int ct = 0; ct < 4; ++ct)
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks) {
        const int col = cw0 + ct * 16 + i, k = ks * 32 + 8 * g;
        b[ct][ks] = as_bf16x8(buf_load16(rD, (col < p.N && k < rank) ? (uint32_t)(((size_t)col * rank + k) * 2) : OOB));
      }
  } else {
#pragma unroll
    for (int ct = 0; ct < 4; ++ct)
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks) {
        const bf16x4 lo = lds_read_tr(sp + ks * 32 * GP + tr_off + ct * 16), hi = lds_read_tr(sp + ks * 32 * GP + tr_off + 4 * GP + ct * 16);
        b[ct][ks] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      }
  }

  const uint32_t vbits_lo = row_valid_bits32(p.dtab, it.row0);
  const uint32_t vbits_hi = it.nrows > 32 ? row_valid_bits32(p.dtab, it.row0 + 32) : 0u;
  const size_t zrow0 = (size_t)(tk.zrow0 + it.row0 - tk.row_begin);
  const bf16_t* in = p.In + (p.backward ? (size_t)it.row0 : zrow0) * p.N;
  bf16_t* out = p.Out + (p.backward ? zrow0 : (size_t)it.row0) * p.N;
  // the eight pieces of `In` this lane adds to are fetched up front (fetched where they are used, each cost the wave
  // a memory latency)
  uint4 xin[4][2];
  bool xok[4][2];
#pragma unroll
  for (int rt = 0; rt < 4; ++rt)
#pragma unroll
    for (int ps = 0; ps < 2; ++ps) {
      const int m = rt * 16 + b_row + 8 * ps, c = cw0 + b_pc;
      xok[rt][ps] = m < it.nrows && c < p.N && ((m < 32 ? vbits_lo >> m : vbits_hi >> (m - 32)) & 1u) != 0;
      xin[rt][ps] = xok[rt][ps] ? *(const uint4*)(in + (size_t)m * p.N + c) : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
  for (int rt = 0; rt < 4; ++rt) {
    if (rt * 16 >= it.nrows) break;
    // operands exchanged: acc[ct][v] = product[row 16 rt + i][column 16 ct + 4 g + v]
#pragma unroll
    for (int ct = 0; ct < 4; ++ct) {
      f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b[ct][ks], a[rt][ks], acc, 0, 0, 0);
      *(f32x4*)(sc + i * SP + ct * 16 + 4 * g) = acc;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int ps = 0; ps < 2; ++ps) {
      const int ml = b_row + 8 * ps, m = rt * 16 + ml, c = cw0 + b_pc;
      if (m < it.nrows && c < p.N) {
        uint4 o = make_uint4(0, 0, 0, 0);
        if (xok[rt][ps]) {
          const uint4 x = xin[rt][ps];
          const f32x4 p0 = *(const f32x4*)(sc + ml * SP + b_pc), p1 = *(const f32x4*)(sc + ml * SP + b_pc + 4);
          const uint32_t* px = (const uint32_t*)&x;
          o.x = pack_bf16x2(__uint_as_float(px[0] << 16) + p0[0], __uint_as_float(px[0] & 0xffff0000u) + p0[1]);
          o.y = pack_bf16x2(__uint_as_float(px[1] << 16) + p0[2], __uint_as_float(px[1] & 0xffff0000u) + p0[3]);
          o.z = pack_bf16x2(__uint_as_float(px[2] << 16) + p1[0], __uint_as_float(px[2] & 0xffff0000u) + p1[1]);
          o.w = pack_bf16x2(__uint_as_float(px[3] << 16) + p1[2], __uint_as_float(px[3] & 0xffff0000u) + p1[3]);
        }
        *(uint4*)(out + (size_t)m * p.N + c) = o;
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }
}

// ------------------------------------------------------------------------------------------------
// IA3_OUT: part[item][n] = sum_{rows} g[i][n] * z[i][n], and dYs[i][n] = g[i][n] * l_t[n] (the operand of the
// backbone backward for these rows).  grid = (64-row items, ceil(N/1024)), 512 threads: 128 column threads of 8
// columns, times four quarters of the item's rows (16 rows each, all 32 loads of a thread issued before the first
// sum), the quarters' sums added through LDS in the order of the rows.
__global__ __launch_bounds__(512) void k_dl(const int32_t* __restrict__ dtab, const TaskRef tasks,
                                           const bf16_t* __restrict__ dY, const bf16_t* __restrict__ Z, float* __restrict__ part,
                                           bf16_t* __restrict__ dYs, int N, int items_off, int bits_off) {
  __shared__ float sq[3][128][9];
  const int item = blockIdx.x;
  const int4 iw = *(const int4*)(dtab + items_off + item * DI_WORDS);
  const int task = iw.x, row0 = iw.y, nrows = iw.z;
  if (task < 0 || iw.w == 0) return;
  if (get_task_kind(tasks, task) != MUX_ADAPTER_IA3_OUT) return;
  const DevTask tk = get_task(tasks, task);
  const uint32_t* bw = (const uint32_t*)(dtab + bits_off) + 2 * item;
  const int ct = threadIdx.x & 127, rq = threadIdx.x >> 7;
  const uint32_t bits = (rq < 2 ? bw[0] : bw[1]) >> (16 * (rq & 1)) & 0xffffu;    // validity of this quarter's 16 rows
  const int n0 = (blockIdx.y * 128 + ct) * 8;
  const bool cols = n0 < N;
  constexpr int RQ = 16;
  float s[8], lv[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) { s[e] = 0.f; lv[e] = 0.f; }
  if (cols) {
    const uint4 l4 = *(const uint4*)((const bf16_t*)tk.L + n0);
    const uint32_t* pl = (const uint32_t*)&l4;
#pragma unroll
    for (int e = 0; e < 4; ++e) { lv[2 * e] = __uint_as_float(pl[e] << 16); lv[2 * e + 1] = __uint_as_float(pl[e] & 0xffff0000u); }
    // every thread issues the same 2 RQ loads (a row that does not count reads the item's first row instead and is
    // dropped afterwards)
    uint4 gv[RQ], zv[RQ];
#pragma unroll
    for (int u = 0; u < RQ; ++u) {
      const int m = rq * RQ + u;
      const int row = row0 + (m < nrows ? m : 0);
      gv[u] = *(const uint4*)(dY + (size_t)row * N + n0);
      zv[u] = *(const uint4*)(Z + (size_t)(tk.zrow0 + row - tk.row_begin) * N + n0);
    }
#pragma unroll
    for (int u = 0; u < RQ; ++u) {
      const int m = rq * RQ + u;
      if (!(m < nrows && ((bits >> u) & 1u))) continue;
      const uint32_t* pg = (const uint32_t*)&gv[u];
      const uint32_t* pz = (const uint32_t*)&zv[u];
      uint4 sv;
      uint32_t* ps = (uint32_t*)&sv;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float g0 = __uint_as_float(pg[e] << 16), g1 = __uint_as_float(pg[e] & 0xffff0000u);
        s[2 * e] = fmaf(g0, __uint_as_float(pz[e] << 16), s[2 * e]);
        s[2 * e + 1] = fmaf(g1, __uint_as_float(pz[e] & 0xffff0000u), s[2 * e + 1]);
        ps[e] = pack_bf16x2(g0 * lv[2 * e], g1 * lv[2 * e + 1]);
      }
      *(uint4*)(dYs + (size_t)(tk.zrow0 + row0 + m - tk.row_begin) * N + n0) = sv;
    }
  }
  if (rq > 0) {
#pragma unroll
    for (int e = 0; e < 8; ++e) sq[rq - 1][ct][e] = s[e];
  }
  __syncthreads();
  if (rq == 0 && cols) {
    float* dst = part + (size_t)item * N + n0;
#pragma unroll
    for (int e = 0; e < 8; ++e) dst[e] = ((s[e] + sq[0][ct][e]) + sq[1][ct][e]) + sq[2][ct][e];
  }
}

// ------------------------------------------------------------------------------------------------
// out_t = (accumulate ? out_t : 0) + sum over the task's items, ascending.  grid = (tasks, blocks over the elements).
// LoRA and Adapter-Tuning tasks: elements [0, r*N) are dB_t [r][N] from part0, elements [r*N, r*(N+K)) are dA_t from
// part1, stored transposed as [K][r].  IA3_OUT tasks: dl_t [N] from part_ia3 (one row per 64-row item).
__global__ __launch_bounds__(256) void k_reduce(const int32_t* __restrict__ dtab, const TaskRef tasks,
                                               const float* __restrict__ part0, const float* __restrict__ part1,
                                               const float* __restrict__ part_ia3, int N, int K,
                                               int RP, int ts0, int ts1, int accumulate, size_t slot0, size_t slot1) {
  const int t = blockIdx.x;
  const DevTask tk = get_task(tasks, t);
  const bool ranked = tk.kind == MUX_ADAPTER_LORA || tk.kind == MUX_ADAPTER_TUNING;
  if (!ranked && tk.kind != MUX_ADAPTER_IA3_OUT) return;
  const int mode = ranked ? 0 : 1;
  if (mode == 1) { part0 = part_ia3; slot0 = (size_t)N; ts0 = TS64; }
  if (tk.kind == MUX_ADAPTER_TUNING) K = N;    // its first gradient is dD_t [N][r]
  const int rows = mode == 1 ? 1 : tk.rank;
  size_t e = ((size_t)blockIdx.y * 256 + threadIdx.x) * 4;     // four consecutive elements of one row (N, K multiples of 4)
  const float* part = part0;
  int C = N;
  float* out = mode == 1 ? tk.dL : tk.dB;
  bool transposed = false;
  size_t slot = slot0;
  int ts = ts0;                                // row-group size of the partials: the two passes choose their own
  if (mode == 0 && e >= (size_t)rows * N) {
    e -= (size_t)rows * N;
    part = part1; C = K; out = tk.dA; transposed = true; slot = slot1; ts = ts1;
  }
  if (!out || e >= (size_t)rows * C) return;
  const int j = (int)(e / C), c = (int)(e % C);
  const int32_t* ti = dtab + dtab[DH_NITEMS0 + 3 * ts + 2] + 2 * t;
  const int ib = ti[0], ic = ti[1];
  const int32_t* items = dtab + dtab[DH_NITEMS0 + 3 * ts + 1];
  // four items in flight (a thread that fetched them one by one would wait a memory latency per item); an item
  // without valid rows holds no partial and adds an exact zero; the sum runs in ascending item order
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int q = 0; q < ic; q += 4) {
    float4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const bool has = q + u < ic && items[(ib + q + u) * DI_WORDS + DI_NVALID] != 0;
      v[u] = has ? *(const float4*)(part + (size_t)(ib + q + u) * slot + (size_t)j * C + c) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) { s.x += v[u].x; s.y += v[u].y; s.z += v[u].z; s.w += v[u].w; }
  }
  if (transposed) {
    float* dst = out + (size_t)c * rows + j;
    dst[0] = accumulate ? dst[0] + s.x : s.x;
    dst[rows] = accumulate ? dst[rows] + s.y : s.y;
    dst[2 * (size_t)rows] = accumulate ? dst[2 * (size_t)rows] + s.z : s.z;
    dst[3 * (size_t)rows] = accumulate ? dst[3 * (size_t)rows] + s.w : s.w;
  } else if (((uintptr_t)out & 15) == 0) {
    float4* dst = (float4*)(out + e);
    float4 o = s;
    if (accumulate) { const float4 d = *dst; o.x += d.x; o.y += d.y; o.z += d.z; o.w += d.w; }
    *dst = o;
  } else {                                     // a gradient buffer of the caller that is only 4-byte aligned
    float* dst = out + e;
    dst[0] = accumulate ? dst[0] + s.x : s.x;
    dst[1] = accumulate ? dst[1] + s.y : s.y;
    dst[2] = accumulate ? dst[2] + s.z : s.z;
    dst[3] = accumulate ? dst[3] + s.w : s.w;
  }
}

void launch_grad(const CallCtx& c, const char* name, const GradParams& p, dim3 grid) {
  // two steps of loads in flight where the registers still allow four waves a SIMD
  if (c.st->r_max <= 16) MUX_LAUNCH(name, (k_grad<1, 2>), grid, dim3(256), 0, c.stream, p);
  else if (c.st->r_max <= 32) MUX_LAUNCH(name, (k_grad<2, 2>), grid, dim3(256), 0, c.stream, p);
  else MUX_LAUNCH(name, (k_grad<4, 1>), grid, dim3(256), 0, c.stream, p);
}

// Row groups of 1024 mean 1/4 of the partial bytes of groups of 256; they are taken when the launch still has
// `enough` workgroups to occupy the chip.
int choose_group(const mux_segtab* st, int col_blocks, int enough) {
  return st->items[TS1024].size() * (size_t)col_blocks >= (size_t)enough ? TS1024 : TS256;
}
constexpr int kS4Cols = 512;                          // columns of one workgroup of the dY pass
int s4_slabs(int N) { return (N + kS4Cols - 1) / kS4Cols; }
int s4_group(const mux_segtab* st, int N) { return choose_group(st, s4_slabs(N), 192); }
int da_group(const mux_segtab* st, int C) { return choose_group(st, (C + 255) / 256, 384); }

struct PartLayout { size_t gpart, part0, part1, ia3, total; };
PartLayout part_layout(int K, int N, const mux_segtab* st) {
  PartLayout o{};
  const int RP = rank_pitch(st);
  const int K1 = (st->n_tuning > 0 && N > K) ? N : K;       // a TUNING item's second partial is [RP][N]
  if (RP > 0) {
    o.gpart = align256((size_t)s4_slabs(N) * st->T * RP * 4);
    o.part0 = align256((size_t)st->items[TS256].size() * RP * N * 4);      // sized for the smaller row groups
    o.part1 = align256((size_t)st->items[TS256].size() * RP * K1 * 4);
  }
  o.ia3 = st->n_ia3 > 0 ? align256((size_t)st->items[TS64].size() * N * 4) : 0;
  o.total = o.gpart + o.part0 + o.part1 + o.ia3;     // the IA3 partials lie behind the others: one reduction takes both
  return o;
}

}  // namespace

size_t adapter_partial_bytes(int K, int N, const mux_segtab* st) { return part_layout(K, N, st).total; }

mux_status adapter_down_x(const CallCtx& c, const void* X, void* Hs) {
  if (c.st->n_lora == 0) return MUX_OK;
  // A_t is read as it is when every LoRA rank allows it; else A_t^T was laid into c.AT by the packing kernel of this call
  DownParams p{c.dtab, (const bf16_t*)X, (bf16_t*)Hs, c.lora_natural ? nullptr : (const bf16_t*)c.AT, nullptr, c.K, c.RP, DOWN_X};
  launch_down(c, "down_x", p, c.lora_natural);
  return MUX_OK;
}

// The pass over dY: Gs (LoRA: s_t dY B_t^T; Adapter-Tuning: s_t (dY U_t^T) * gelu'(u)) and the partial sums of
// dB_t = Hs^T dY (dU_t), which adapter_grads brings together.
mux_status adapter_dy_pass(const CallCtx& c, const void* dY, const void* Hs, void* Gs, void* part) {
  if (c.st->n_lora + c.st->n_tuning == 0) return MUX_OK;
  const PartLayout pl = part_layout(c.K, c.N, c.st);
  float* gpart = (float*)part;
  float* part0 = (float*)((char*)part + pl.gpart);
  const int ts = s4_group(c.st, c.N), slabs = s4_slabs(c.N);
  S4Params p{c.dtab, (const bf16_t*)dY, (const bf16_t*)Hs, gpart, part0, c.N, c.RP, ts, c.st->T,
             c.st->dev_image[DH_NITEMS0 + 3 * ts + 1], c.st->dev_image[DH_OFF_ROWBITS]};
  p.tasks = *c.tref;
  const dim3 grid((unsigned)c.st->items[ts].size(), (unsigned)slabs);
  // (rank pieces, steps between two meetings of the waves, steps of loads in flight)
  if (c.st->r_max <= 16) MUX_LAUNCH("s4_dy_pass", (k_s4<1, 2, 2>), grid, dim3(512), 0, c.stream, p);
  else if (c.st->r_max <= 32) MUX_LAUNCH("s4_dy_pass", (k_s4<2, 2, 1>), grid, dim3(512), 0, c.stream, p);
  else MUX_LAUNCH("s4_dy_pass", (k_s4<4, 1, 1>), grid, dim3(512), 0, c.stream, p);
  // moved: the partials of every slab once in (a task's real tokens, its rank rounded up to four columns), Gs once out
  double moved = (double)c.st->T * c.RP * 2;
  for (const HostTask& ht : c.st->tasks)
    if (ht.kind == MUX_ADAPTER_LORA || ht.kind == MUX_ADAPTER_TUNING) moved += (double)slabs * ht.valid * round_up(ht.rank, 4) * 4;
  prof_note_bytes(moved);
  MUX_LAUNCH("gs_reduce", k_gs_reduce, dim3((unsigned)c.st->items[TS64].size()), dim3(256), 0, c.stream, c.dtab, *c.tref,
             (const float*)gpart, slabs, c.st->T, c.RP, (const bf16_t*)c.U2, (bf16_t*)Gs,
             c.st->dev_image[DH_NITEMS0 + 3 * TS64 + 1], c.st->dev_image[DH_OFF_ITEM_BITS]);
  return MUX_OK;
}

// Adapter-Tuning: Y = z + Hs U_t (forward) or dYs = dY + Gs D_t^T (backward, D_t^T from the transposed region)
mux_status adapter_tune_add(const CallCtx& c, const void* In, const void* Small, void* Out, int backward) {
  if (c.st->n_tuning == 0) return MUX_OK;
  TuneAddParams p{c.dtab, (const bf16_t*)In, (const bf16_t*)Small, (bf16_t*)Out, (const bf16_t*)c.AT, c.N, c.RP, backward,
                  c.tune_natural ? 1 : 0};
  p.tasks = *c.tref;
  const dim3 grid((unsigned)c.st->items[TS64].size(), (c.N + 255) / 256);
  if (c.RP <= 32) MUX_LAUNCH(backward ? "tune_dz" : "tune_up", (k_tune_add<1>), grid, dim3(256), 0, c.stream, p);
  else MUX_LAUNCH(backward ? "tune_dz" : "tune_up", (k_tune_add<2>), grid, dim3(256), 0, c.stream, p);
  return MUX_OK;
}

// Adapter-Tuning forward, after the backbone GEMM saved z = x W: u = z D_t, Hs = s_t gelu(u).  D_t [N, r] is read as it
// is when every such rank is a multiple of 8; else D_t^T was laid into c.AT by the packing kernel of this call.
mux_status adapter_down_tune(const CallCtx& c, const void* Z, void* Hs) {
  if (c.st->n_tuning == 0) return MUX_OK;
  DownParams p{c.dtab, (const bf16_t*)Z, (bf16_t*)Hs, c.tune_natural ? nullptr : (const bf16_t*)c.AT, (bf16_t*)c.U2, c.N, c.RP, DOWN_TUNE};
  launch_down(c, "tune_down", p, c.tune_natural);
  return MUX_OK;
}

// After adapter_dy_pass: dA_t = X^T Gs (Adapter-Tuning: dD_t = z^T Gs) in partial sums per row group, then both
// gradients of every task brought together; IA3_OUT: dl_t and the scaled rows the backbone backward reads.
mux_status adapter_grads(const CallCtx& c, const void* X, const void* dY, const void* Hs, const void* Gs, const void* Z,
                         void* part, int accumulate) {
  const int M = c.st->n_tasks;
  const PartLayout pl = part_layout(c.K, c.N, c.st);
  const bool ranked = c.st->n_lora + c.st->n_tuning > 0;
  const int K1 = (c.st->n_tuning > 0 && c.N > c.K) ? c.N : c.K;
  const int ts_b = s4_group(c.st, c.N), ts_a = da_group(c.st, K1);
  float* part0 = (float*)((char*)part + pl.gpart);
  float* part1 = (float*)((char*)part + pl.gpart + pl.part0);
  float* part_ia3 = (float*)((char*)part + pl.gpart + pl.part0 + pl.part1);
  const size_t slot0 = (size_t)c.RP * c.N, slot1 = (size_t)c.RP * K1;
  double moved = 0.0;       // what the reduction moves: every row group's partials once in, the gradients once out
  size_t elems = 0;
  if (ranked) {
    GradParams p{c.dtab, {(const bf16_t*)Hs, (const bf16_t*)Gs}, {(const bf16_t*)dY, (const bf16_t*)X}, {part0, part1},
                 {c.N, c.K}, c.RP, ts_a, (const bf16_t*)Z, {slot0, slot1}, 1,
                 c.st->dev_image[DH_NITEMS0 + 3 * ts_a + 1], c.st->dev_image[DH_OFF_ROWBITS], c.st->T};
    p.tasks = *c.tref;
    launch_grad(c, "grad_da", p, dim3((unsigned)c.st->items[ts_a].size(), (K1 + 255) / 256, 1));
    elems = (size_t)c.st->r_max * ((size_t)c.N + K1);
    for (const HostTask& ht : c.st->tasks)
      if (ht.kind == MUX_ADAPTER_LORA || ht.kind == MUX_ADAPTER_TUNING) {
        const double kk = ht.kind == MUX_ADAPTER_TUNING ? c.N : c.K;
        const double gb = (ht.row_count + kTileRows[ts_b] - 1) / kTileRows[ts_b], ga = (ht.row_count + kTileRows[ts_a] - 1) / kTileRows[ts_a];
        moved += 4.0 * ht.rank * (gb * c.N + ga * kk) + 4.0 * ht.rank * (c.N + kk) * (accumulate ? 2 : 1);
      }
  }
  if (c.st->n_ia3 > 0) {
    MUX_LAUNCH("grad_dl", k_dl, dim3((unsigned)c.st->items[TS64].size(), (c.N + 1023) / 1024), dim3(512), 0, c.stream,
               c.dtab, *c.tref, (const bf16_t*)dY, (const bf16_t*)Z, part_ia3, (bf16_t*)c.dYs, c.N,
               c.st->dev_image[DH_NITEMS0 + 3 * TS64 + 1], c.st->dev_image[DH_OFF_ITEM_BITS]);
    if ((size_t)c.N > elems) elems = (size_t)c.N;
    for (const HostTask& ht : c.st->tasks)
      if (ht.kind == MUX_ADAPTER_IA3_OUT) moved += 4.0 * c.N * ((ht.row_count + 63) / 64) + 4.0 * c.N * (accumulate ? 2 : 1);
  }
  if (elems > 0) {
    // one reduction for every kind: a task's workgroups take the sums its kind has
    prof_note_bytes(moved);
    MUX_LAUNCH("reduce_grads", k_reduce, dim3(M, (unsigned)((elems + 1023) / 1024)), dim3(256), 0, c.stream, c.dtab, *c.tref,
               (const float*)part0, (const float*)part1, (const float*)part_ia3, c.N, c.K, c.RP, ts_b, ts_a, accumulate,
               slot0, slot1);
  }
  return MUX_OK;
}

}  // namespace mux
