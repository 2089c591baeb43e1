// Backbone GEMM, pipelined version: global -> LDS by direct buffer loads (no register staging),
// operand reads software-pipelined one MFMA step ahead.
//
//   forward  (NN):  Y[T,N]  = mask * ( X[T,K] W[K,N]      + Hs[T,r] B_t[r,N] )      Eq. 1 + LoRA + Add
//   backward (NT):  dX[T,K] = mask * ( dY[T,N] W[K,N]^T   + Gs[T,r] A_t[K,r]^T )    Eq. 2 + LoRA
//
// 256x256 output tile per workgroup of eight waves (two per SIMD), 128x64 per wave as 4x2
// v_mfma_f32_32x32x16_bf16.
//   * `buffer_load_dwordx4 ... lds` writes each lane's 16 bytes at LDS base + 16*lane, so a wave
//     instruction fills 1 KB of a stage.  A masked piece gets an out-of-range offset and lands as zeros.
//   * K-tiles are 64 deep whenever the contraction length allows: a row of a [rows][64] tile is one whole
//     128-byte line of X, dY or W.  Measured on this part, the L2 -> LDS path moves half-lines (the 64-byte rows
//     of a 32-deep tile) at half the rate of whole lines, at every level of the hierarchy, and that rate, not the
//     matrix cores, was the limit of the 32-deep version.  Two stages of 64 KB; the loads of tile kt+2 go out
//     right after the barrier that frees the stage of tile kt.  The 32-deep version (four stages, three tiles
//     in flight) remains for contraction lengths that are multiples of 32 only.
//   * LDS rows cannot be padded under the DMA rule, so 16-byte pieces are XOR-swizzled instead:
//     [rows][BK] tiles by row bits, the forward's [BK][256] tile of W by k bits.
//   * one workgroup barrier per K-tile, placed before the last MFMA step: by then every read of
//     the current stage is done (it may be refilled) and the next tile has landed (it may be read).
//   * one workgroup per compute unit at a time; the tiles left over after the last full round of workgroups are
//     cut into two 256x128 halves or four 128x128 quarters (four waves, four 32 KB stages) at the end of the
//     same launch, so that they occupy the compute units once more instead of a fraction of them for a whole
//     tile time.
// Every stage is its own __shared__ array so that the compiler's wait-count insertion can tell
// the stage being filled from the stage being read.
#include <cstdlib>
#include <type_traits>

#include "mux_device_utils.h"

namespace mux {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((address_space(3))) void* lds_void_ptr;

constexpr int BM = 256;
constexpr int TILE_N = 256;                     // width of a tile in the launch's tile index space
constexpr int TS256 = 2;
constexpr uint32_t OOB = 0x80000000u;

struct GemmParams {
  const int32_t* dtab;
  const bf16_t* Ain;   // [T, Kc]  activations (X or dY)
  const bf16_t* W;     // [K, ldw]
  int64_t ldw;
  const bf16_t* Ext;   // [T, RP]  Hs or Gs
  bf16_t* Out;         // [T, Nc]
  bf16_t* Zsave;       // forward: x W of IA3_OUT rows (may be null)
  bf16_t* HsOut;       // forward with the down-projection in the tile loop: Hs [T, RP] is written here (else null)
  int Kc, Nc, RP;
  int n_m, n_n, per_xcd;   // tile grid in units of 256 x TILE_N tiles; workgroups per XCD over the whole grid
  int n_full;              // workgroups that compute full tiles (a multiple of 8); the rest compute pieces of tiles
  int tail_split;          // pieces per tile after the full ones: 2 (halves) or 4 (quarters)
  unsigned long long* clk;  // diagnostic: counters workgroup 0 adds its elapsed cycles and 100 MHz ticks to (null: off)
  const uint32_t* DiffPack; // entries of the Diff-Pruning masks packed for this launch (index << 16 | bf16 value), or null
  const bf16_t* Wdiff;      // merged weights W + M_t * delta_t of the Diff-Pruning tasks, `wdiff_stride` elements apart (or null)
  int64_t wdiff_stride;
  const bf16_t* AinScaled;  // backward: prepared input rows (IA3_OUT: dY * l_t; TUNING: dY + p D_t^T), [z_rows, Kc], indexed like the saved x W
  TaskRef tasks;
};

// Raw buffer descriptor (stride 0) over `bytes` bytes starting at p, as four dwords.
typedef __attribute__((ext_vector_type(4))) int rsrc_t;
__device__ __forceinline__ rsrc_t make_rsrc(const void* p, uint32_t bytes) {
  const uint64_t a = (uint64_t)p;
  // wave-uniform by construction; said explicitly so that the descriptor always lives in scalar registers
  return (rsrc_t){__builtin_amdgcn_readfirstlane((int)(uint32_t)a), __builtin_amdgcn_readfirstlane((int)(uint32_t)(a >> 32)),
                  __builtin_amdgcn_readfirstlane((int)bytes), 0x00020000};
}
// One direct-to-LDS load: lane l's 16 bytes from buffer offset byte_off land at lds_dst_uniform + 16*l.
// Written as inline assembly on purpose: the wait counts of these loads are managed by hand (vmcnt) around
// the workgroup barrier, and the compiler must not pair them with the LDS reads of other stages.
__device__ __forceinline__ void dma16(rsrc_t r, bf16_t* lds_dst_uniform, uint32_t byte_off) {
  const uint32_t lds_addr = (uint32_t)(uintptr_t)(lds_void_ptr)lds_dst_uniform;
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
               :
               : "s"(lds_addr), "v"(byte_off), "s"(r)
               : "m0");
}
// The same with 4 bytes a lane: lane l's dword lands at LDS byte address lds_addr + 4*l.
__device__ __forceinline__ void dma4(rsrc_t r, uint32_t lds_addr, uint32_t byte_off) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, 0 offen lds"
               :
               : "s"(lds_addr), "v"(byte_off), "s"(r)
               : "m0");
}
__device__ __forceinline__ bf16x4 lds_read_tr(const bf16_t* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4bf16((__attribute__((address_space(3))) bf16x4*)p);
}
// s_waitcnt vmcnt(n) only (gfx9 encoding: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt_hi[15:14])
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 15) | 0x70 | 0xF00 | ((N >> 4) << 14));
}
__device__ __forceinline__ void wait_lgkm0() { __builtin_amdgcn_s_waitcnt(0xC07F); }

// Swizzle of the 16-byte piece index inside a row of a [rows][BK] tile: sixteen consecutive rows read the same
// logical piece with one ds_read_b128 and must land in sixteen different 16-byte bank groups.
template <int BK>
__device__ __forceinline__ int swz_row(int r) {
  if (BK == 32) return (((r >> 1) ^ (r >> 3)) & 1) | (((r >> 2) & 1) << 1);   // 64-byte rows: 4 pieces
  return (r >> 1) & 7;                                                          // 128-byte rows: 8 pieces
}

// Up to four A stages, four B stages and the per-row validity flags of one workgroup.
struct Smem {
  bf16_t *a0, *a1, *a2, *a3, *b0, *b1, *b2, *b3;
  int* row;
  bf16_t *e0, *e1, *e2, *e3;     // FUSE: stages of the [64][rank] slabs of A_t
  uint32_t pk_lds;               // DIFFP: LDS byte address of the stages' slots for 256 packed entries of the masks each
  int* off;                      //        per K-tile, where the entries of this tile's buckets begin, split and end
};

// One output tile.  WNW = waves along N, MI x NI = 32x32 MFMA tiles per wave; 2*WNW waves on a
// BMT x BN tile with BMT = 2*MI*32 and BN = WNW*NI*32:
//   <4,4,2> eight waves (two per SIMD), 128x64 per wave, the full 256x256 tile;
//   <4,4,1> eight waves, 128x32 per wave, a 256x128 half of a tile,
//   <2,2,2> four waves (one per SIMD), 64x64 per wave, a 128x128 quarter: for what is left after the last full
//           round of workgroups.
// BK = 64 with two stages, or BK = 32 with four.
// `xcd_slot` = (per-XCD tile slot) * 8 + XCD; `half` selects the 128 columns of a half-width tile, `mhalf` the
// 128 rows of a quarter.
// FUSE (forward, 64-deep stages, half and quarter tiles): the down-projection Hs = s_t X A_t of the tile's rows is
// computed in the same K loop -- the [64][rank] slab of A_t of every K-tile is staged beside the tile of W, wave
// (wm, wn) multiplies it with the X fragment of its row block wn (one more MFMA per step) -- and goes, scaled and
// rounded to bf16, straight into the A side of the adapter K-tile (and, from the tiles of the first column, to
// memory for the backward): no separate pass over X, no launch for it.  Every column tile redoes the product for
// its rows, which is why this is for launches that do not fill the compute units anyway.
// DIFFP (64-deep stages): the rows of a Diff-Pruning task meet W + M_t * delta_t without a copy of W: once a tile of W
// has landed in LDS, the masked entries that fall into it are added in place (one bf16 read-modify-write each) and a
// second barrier follows before the tile is read.  The mask lists its entries by tiles -- buckets of 64 of the
// contraction index by 128 lines of the W side, numbered so that the one or two buckets of a tile are neighbours --
// and the launch brings them packed, (contraction index % 64) << 23 | (line % 128) << 16 | bf16 value.  The entries
// of a K-tile travel with it: every loading wave fetches 64 of them straight into LDS with the tile's other loads
// (256 a tile; a bucket pair with more reads the rest from memory when the tile is patched).
template <bool NT, int WNW, int MI, int NI, int BK, bool FUSE = false, bool DIFFP = false>
__device__ __forceinline__ void gemm_tile(const GemmParams& p, const int xcd_slot, const int half, const int mhalf,
                                          const Smem sm) {
  static_assert(!FUSE || (!NT && BK == 64 && WNW == MI && !(MI == 4 && NI == 2)), "FUSE: forward, 64-deep, half or quarter tiles");
  static_assert(!DIFFP || (BK == 64 && !FUSE), "DIFFP: 64-deep stages");
  constexpr int BN = WNW * NI * 32;
  constexpr int BMT = 2 * MI * 32;
  static_assert(BN == 256 || BN == 128, "tile width");
  static_assert(BMT == 256 || BMT == 128, "tile height");
  static_assert(BK == 32 || BK == 64, "K-tile depth");
  // LDS stages.  A 64-deep stage of a full or half tile takes 64 or 48 KB: two fit.  A quarter's takes 32 KB and
  // half the MFMA time, which is less than the latency of the loads: four stages, three tiles in flight.
  constexpr int NST = (BK == 64 && MI == 4) ? 2 : 4;
  constexpr bool SPLIT = BK == 64 && NST == 4;    // four stages in the two arrays per operand that 64-deep stages have
  constexpr int NW = 2 * WNW, NTHR = 64 * NW;
  constexpr int A_ELEMS = BMT * BK;               // elements of one A stage
  // The loads are issued by the first half of the waves only.  Each SIMD hosts waves w and w + NW/2 and serves the
  // older one first, so wave w runs ahead and then idles at the barrier; a wave that cannot issue a load (the
  // vector memory pipeline takes 16 cycles per instruction, 1 KB) cannot issue the MFMA behind it either.
  // Giving wave w all the loads uses its slack and leaves wave w + NW/2 a pure MFMA / LDS-read stream.
  constexpr int LW = NW == 8 ? NW / 2 : NW;       // four waves: one per SIMD, all of them load
  constexpr int ACH = (A_ELEMS / 512) / LW, BCH = (BN * BK / 512) / LW;   // 1 KB chunks a loading wave fetches per K-tile
  constexpr int ECH = FUSE ? 1 : 0;               // FUSE: and one of the (up to) 4 KB of the slab of A_t
  constexpr int DCH = DIFFP ? 1 : 0;              // DIFFP: and 64 packed entries of the mask
  constexpr int NLD = ACH + BCH + ECH + DCH;      // loads a loading wave issues per K-tile
  static_assert(ACH >= 1 && BCH >= 1, "every loading wave fetches at least one chunk of each tile");
  static_assert(!FUSE || LW == 4, "FUSE: four loading waves bring the four chunks of a slab");
  constexpr int LPR = BK / 8;                     // [rows][BK] tiles: lanes (16-byte pieces) per row
  constexpr int RPC = 64 / LPR;                   //                   rows per 1 KB chunk
  constexpr int PPRB = BN / 8;                    // forward: 16-byte pieces per k-row of the [BK][BN] tile
  constexpr int RPCB = 64 / PPRB;                 // forward: k-rows per 1 KB chunk
  constexpr int WCOLS = NI * 32;                  // columns of the wave tile
  constexpr int EPW = WCOLS + 8;                  // epilogue staging pitch (elements)
  bf16_t* const sA0 = sm.a0; bf16_t* const sA1 = sm.a1; bf16_t* const sA2 = sm.a2; bf16_t* const sA3 = sm.a3;
  bf16_t* const sB0 = sm.b0; bf16_t* const sB1 = sm.b1; bf16_t* const sB2 = sm.b2; bf16_t* const sB3 = sm.b3;
  bf16_t* const sE0 = sm.e0; bf16_t* const sE1 = sm.e1; bf16_t* const sE2 = sm.e2; bf16_t* const sE3 = sm.e3;
  int* const sRow = sm.row;

  const int total = p.n_m * p.n_n;
  const int jslot = xcd_slot >> 3;
  if (jslot >= p.per_xcd) return;
  const int L = (xcd_slot & 7) * p.per_xcd + jslot;
  if (L >= total) return;
  constexpr int GROUP = 4;
  const int width = GROUP * p.n_n;
  const int first_m = (L / width) * GROUP;
  const int gsize = p.n_m - first_m < GROUP ? p.n_m - first_m : GROUP;
  const int tm = first_m + (L % width) % gsize;
  const int tn = (L % width) / gsize;

  const ItemView it = load_item(p.dtab, TS256, tm);
  const int mrow0 = mhalf * BMT;                  // first row of the item this tile covers
  const int nrows = it.nrows - mrow0 < BMT ? it.nrows - mrow0 : BMT;   // rows of the item inside this tile
  if (nrows <= 0) return;
  const int row0 = it.row0 + mrow0;
  const int c0 = tn * TILE_N + half * BN;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  if (wave >= NW) return;                         // a tile of four waves: the others end here, before any barrier
  const int wm = wave / WNW, wn = wave % WNW;
  const bool loader = wave < LW;
  const int lw = wave % LW;                       // chunk owner index (meaningful for loading waves)

  if (tid < BMT) sRow[tid] = (it.task >= 0 && tid < nrows && row_is_valid(p.dtab, row0 + tid)) ? 1 : 0;

  // FUSE: the tiles of the first column also write Hs of their rows; zeros where no LoRA product is formed
  auto zero_hs_rows = [&]() {
    if (FUSE && c0 == 0 && p.HsOut != nullptr)
      for (int e = tid; e < nrows * (p.RP / 8); e += NTHR)
        *(uint4*)(p.HsOut + (size_t)(row0 + e / (p.RP / 8)) * p.RP + (e % (p.RP / 8)) * 8) = make_uint4(0, 0, 0, 0);
  };
  if (it.task < 0 || it.nvalid == 0) {             // rows of no task, or padding only: zeros out
    for (int e = tid; e < nrows * (BN / 8); e += NTHR) {
      const int m = e / (BN / 8), c = c0 + (e % (BN / 8)) * 8;
      if (c < p.Nc) *(uint4*)(p.Out + (size_t)(row0 + m) * p.Nc + c) = make_uint4(0, 0, 0, 0);
    }
    zero_hs_rows();
    return;
  }

  const DevTask tk = get_task(p.tasks, it.task);
  const bool lora = tk.kind == MUX_ADAPTER_LORA;
  const bool ia3 = tk.kind == MUX_ADAPTER_IA3_OUT;
  const bool tuning = tk.kind == MUX_ADAPTER_TUNING;   // forward: only x W is produced here (saved); backward: prepared rows
  const int rank = tk.rank;
  const bf16_t* adapterB = NT ? (const bf16_t*)tk.A : (const bf16_t*)tk.B;
  const bf16_t* Lvec = (const bf16_t*)tk.L;

  const int KT = p.Kc / BK;                         // the contraction length is a multiple of BK
  const int KT_ext = lora ? (rank + BK - 1) / BK : 0;
  const int KT_total = KT + KT_ext;
  const bool fuse_h = FUSE && lora;                 // this tile forms Hs of its rows in the K loop
  // DIFFP: the bucket offsets of this task's listing for this direction, the buckets of this tile in a K-tile's row
  // of buckets, and per stage the entries of the tile it holds: first, first of the second bucket, end
  const bool patch = DIFFP && tk.kind == MUX_ADAPTER_DIFF && tk.rank >= 0 && p.DiffPack != nullptr && c0 < p.Nc;
  constexpr int SPAN = BN / 128;
  const int32_t* bptr = (const int32_t*)tk.dB;
  const int nbk = (p.Nc + 127) >> 7, bcol = c0 >> 7;
  const int bspan = bcol + SPAN <= nbk ? SPAN : nbk - bcol;      // a ragged last tile may hold one bucket only
  const uint32_t* dlist = p.DiffPack + (patch ? tk.rank : 0);
  const rsrc_t rPk = make_rsrc(patch ? (const void*)dlist : (const void*)p.Ain, patch ? (uint32_t)tk.at_off * 4u : 0u);
  int ps0[NST], ps1[NST], ps2[NST];
#pragma unroll
  for (int q = 0; q < NST; ++q) { ps0[q] = 0; ps1[q] = 0; ps2[q] = 0; }
  int nx0 = 0, nx1 = 0, nx2 = 0;                   // the same for the tile after the ones in flight
  // The offsets of every K-tile's entries go to LDS once (a load from the listing inside the loop would have the loop
  // wait for it, and for the tiles in flight with it, at every K-tile).
  if (DIFFP && patch) {
    for (int t = tid; t < KT; t += NTHR) {
      const int32_t* q = bptr + (size_t)t * nbk + bcol;
      sm.off[3 * t] = q[0];
      sm.off[3 * t + 1] = q[1];
      sm.off[3 * t + 2] = q[bspan];
    }
    __syncthreads();
  }
  // offsets of the entries of K-tile t (none past the backbone tiles, none without a mask)
  auto bucket_offsets = [&](int t, int& o0, int& o1, int& o2) {
    o0 = 0; o1 = 0; o2 = 0;
    if (DIFFP && patch && t < KT) {
      o0 = __builtin_amdgcn_readfirstlane(sm.off[3 * t]);
      o1 = __builtin_amdgcn_readfirstlane(sm.off[3 * t + 1]);
      o2 = __builtin_amdgcn_readfirstlane(sm.off[3 * t + 2]);
    }
  };

  // ---- DMA geometry.  A wave instruction fills 1 KB: RPC rows x 2 BK bytes of a [rows][BK] tile
  // (lane -> row lane/LPR, physical piece lane%LPR), or RPCB k-rows of the forward's [BK][BN] tile of W
  // (lane -> k-row lane/PPRB, physical piece lane%PPRB).  Loading wave w owns chunks w*ACH .. of A and w*BCH .. of B.
  const int r_in = lane / LPR;                                  // row inside the chunk
  const uint32_t a_rows_bytes = (uint32_t)nrows * (uint32_t)p.Kc * 2u;
  const bf16_t* a_base = (NT && (ia3 || tuning)) ? p.AinScaled + (size_t)(tk.zrow0 + row0 - tk.row_begin) * p.Kc
                                     : p.Ain + (size_t)row0 * p.Kc;
  const rsrc_t rA = make_rsrc(a_base, a_rows_bytes);
  const rsrc_t rW = make_rsrc(task_weight(tk, p.W, p.Wdiff, p.wdiff_stride), (uint32_t)((size_t)(NT ? p.Nc : p.Kc) * p.ldw * 2));
  const rsrc_t rE = make_rsrc(lora ? p.Ext + (size_t)row0 * p.RP : p.Ain, lora ? (uint32_t)nrows * (uint32_t)p.RP * 2u : 0u);
  const rsrc_t rP = make_rsrc(lora ? adapterB : p.Ain, lora ? (uint32_t)(NT ? (size_t)p.Nc * rank : (size_t)rank * p.Nc) * 2u : 0u);

  // FUSE: A_t [K][rank] as it is; the slab of K-tile kt is the 128 rank bytes from byte kt * 128 rank on, loading wave
  // w brings its w-th KB (lane l the 16 bytes at 1024 w + 16 l), so the slab lies in LDS as in memory, [64][rank]
  const rsrc_t rAt = make_rsrc(fuse_h ? tk.A : (const void*)p.Ain, fuse_h ? (uint32_t)p.Kc * (uint32_t)rank * 2u : 0u);
  const uint32_t offE = (fuse_h && (uint32_t)(lw * 1024 + lane * 16) < 128u * (uint32_t)rank) ? (uint32_t)(lw * 1024 + lane * 16) : OOB;
  uint32_t kE = 0;
  const uint32_t stepE = 128u * (uint32_t)rank;

  // row of the [rows][BK] tile chunk q of this wave puts this lane on, and the logical k-piece it fetches there
  auto a_row_of = [&](int q) { return lw * (RPC * ACH) + RPC * q + r_in; };
  auto b_row_of = [&](int q) { return lw * (RPC * BCH) + RPC * q + r_in; };   // backward: row of W inside the tile
  auto piece_of = [&](int row) { return (lane % LPR) ^ swz_row<BK>(row); };
  // forward W tile: k-row = (lw*BCH + q)*RPCB + lane/PPRB, physical piece lane%PPRB -> logical n
  const int nk_in = lane / PPRB;
  const int n_pp = lane % PPRB;

  // Per-thread byte offsets of the pieces this lane fetches per tile, without the K-tile term.
  // A piece that must read as zero is parked out of range.
  uint32_t offA[ACH], offB[BCH];
#pragma unroll
  for (int q = 0; q < ACH; ++q)
    offA[q] = ((uint32_t)a_row_of(q) * (uint32_t)p.Kc + (uint32_t)(piece_of(a_row_of(q)) * 8)) * 2u;
#pragma unroll
  for (int q = 0; q < BCH; ++q) {
    if (NT) {
      offB[q] = (uint32_t)(((size_t)(c0 + b_row_of(q)) * p.ldw + piece_of(b_row_of(q)) * 8) * 2);
    } else {
      const int kk = (lw * BCH + q) * RPCB + nk_in;          // k-row inside the tile
      const int seg = (n_pp >> 1) ^ ((kk & 3) << 1);         // logical 32-byte segment
      const int n = seg * 16 + (n_pp & 1) * 8;
      offB[q] = (c0 + n < p.Nc) ? (uint32_t)(((size_t)kk * p.ldw + c0 + n) * 2) : OOB;
    }
  }
  // K-tile term: advances by one tile per issue (scalar).  After the last backbone tile the sources switch
  // to the adapter operands (Ext rows and B_t / A_t), whose offsets restart from zero; past the last tile
  // everything is parked out of range (zeros land in a stage nobody reads).
  rsrc_t curA = rA, curB = rW;
  uint32_t kA = 0, kB = 0, stepA = BK * 2u, stepB = NT ? BK * 2u : (uint32_t)((size_t)BK * p.ldw * 2);
  int next_tile = 0;                                          // index of the tile the next issue() fetches

  // uniform, rarely taken: everything that changes at a tile-kind boundary
  auto prepare = [&]() {
    if (next_tile >= KT) {
      if (FUSE) kE = OOB;                                     // no slab of A_t past the backbone tiles
      if (next_tile >= KT_total) {
        kA = OOB; kB = OOB;
      } else {
        const int j0 = (next_tile - KT) * BK;                 // first contraction index of this adapter tile
        curB = rP; kB = 0; stepA = 0; stepB = 0;
        if (FUSE) {
          kA = OOB;                                           // the A side of the adapter tile comes from the accumulators
        } else {
          curA = rE; kA = 0;
#pragma unroll
          for (int q = 0; q < ACH; ++q) {
            const int j = j0 + piece_of(a_row_of(q)) * 8;
            offA[q] = (j < p.RP) ? ((uint32_t)a_row_of(q) * (uint32_t)p.RP + (uint32_t)j) * 2u : OOB;
          }
        }
#pragma unroll
        for (int q = 0; q < BCH; ++q) {
          if (NT) {
            const int c = c0 + b_row_of(q);
            const int j = j0 + piece_of(b_row_of(q)) * 8;
            offB[q] = (c < p.Nc && j < rank) ? (uint32_t)(((size_t)c * rank + j) * 2) : OOB;
          } else {
            const int kk = (lw * BCH + q) * RPCB + nk_in;
            const int seg = (n_pp >> 1) ^ ((kk & 3) << 1);
            const int n = seg * 16 + (n_pp & 1) * 8;
            offB[q] = (c0 + n < p.Nc && j0 + kk < rank) ? (uint32_t)(((size_t)(j0 + kk) * p.Nc + c0 + n) * 2) : OOB;
          }
        }
      }
    }
  };
  // one load of the tile being fetched: i = 0 .. NLD-1, the A pieces first, then W, then (FUSE) the slab of A_t
  // (DIFFP: the last load brings entries o0 + 64 lw .. of the tile's buckets, below o2, into the stage's entry slots)
  auto issue_one = [&](bf16_t* dA, bf16_t* dB, bf16_t* dE, int i, uint32_t dP = 0, int o0 = 0, int o2 = 0) {
    if (!loader) return;
    if (i < ACH) dma16(curA, dA + (lw * ACH + i) * 512, offA[i] + kA);
    else if (i < ACH + BCH) dma16(curB, dB + (lw * BCH + (i - ACH)) * 512, offB[i - ACH] + kB);
    else if (DIFFP) dma4(rPk, dP + lw * 256, (o0 + lw * 64 + lane < o2) ? (uint32_t)(o0 + lw * 64 + lane) * 4u : OOB);
    else dma16(rAt, dE + lw * 512, (offE == OOB || kE == OOB) ? OOB : offE + kE);
  };
  auto issue_done = [&]() { kA += stepA; kB += stepB; if (FUSE && kE != OOB) kE += stepE; ++next_tile; };
  auto issue = [&](bf16_t* dA, bf16_t* dB, bf16_t* dE, uint32_t dP = 0, int o0 = 0, int o2 = 0) {
#pragma unroll
    for (int i = 0; i < NLD; ++i) issue_one(dA, dB, dE, i, dP, o0, o2);
    issue_done();
  };

  // ---- operand read geometry
  const int li = lane & 31, lg = lane >> 5;
  const int l16 = lane & 15, lhalf = (lane >> 4) & 1;
  // [rows][BK] tiles: row = (wm|wn)*128 + t*32 + li; logical piece 2*ks + lg (the swizzle depends on li only)
  const int swz = swz_row<BK>(li);
  const int a_rd = (wm * (32 * MI) + li) * BK;  // elements; + t*32*BK + ((2ks+lg)^swz)*8
  const int bt_rd = (wn * WCOLS + li) * BK;
  // forward W tile: k = ks*16 + 8 lg + 4 h + l16/4 ; logical seg = wn*8 + 2 t + lhalf ; + 4*(l16%4) elements
  const int kq = l16 >> 2;                      // k & 3 of the rows this lane addresses
  const int bn_col = 4 * (l16 & 3);

  auto read_ops = [&](const bf16_t* cA, const bf16_t* cB, int ks, bf16x8 (&a)[MI], bf16x8 (&b)[NI]) {
    const int pa = ((2 * ks + lg) ^ swz) * 8;
#pragma unroll
    for (int t = 0; t < MI; ++t) a[t] = *(const bf16x8*)(cA + a_rd + t * 32 * BK + pa);
    if (NT) {
#pragma unroll
      for (int t = 0; t < NI; ++t) b[t] = *(const bf16x8*)(cB + bt_rd + t * 32 * BK + pa);
    } else {
      const int krow = ks * 16 + 8 * lg + kq;
#pragma unroll
      for (int t = 0; t < NI; ++t) {
        const int seg = (wn * (2 * NI) + 2 * t + lhalf) ^ (kq << 1);
        const bf16x4 lo = lds_read_tr(cB + krow * BN + seg * 16 + bn_col);
        const bf16x4 hi = lds_read_tr(cB + (krow + 4) * BN + seg * 16 + bn_col);
        b[t] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      }
    }
  };

  // Accumulators.  The MFMAs are issued with the operands exchanged, so acc[mi][ni] holds the transposed 32x32
  // block: this lane has row 32 mi + li and the four consecutive columns 32 ni + 8 j + 4 lg .. + 3 in registers
  // 4j .. 4j+3, which the epilogue packs into one 8-byte LDS store.
  f32x16 acc[MI][NI];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;

  auto mma = [&](const bf16x8 (&a)[MI], const bf16x8 (&b)[NI]) {
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[ni], a[mi], acc[mi][ni], 0, 0, 0);
  };

  auto mma_one = [&](const bf16x8 (&a)[MI], const bf16x8 (&b)[NI], int m) {
    const int mi = m / NI, ni = m % NI;
    acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[ni], a[mi], acc[mi][ni], 0, 0, 0);
  };
  // one MFMA step with the loads of one tile (all ACH+BCH of them) spread between its MFMA pairs
  auto mma_with_loads = [&](const bf16x8 (&a)[MI], const bf16x8 (&b)[NI], bf16_t* dA, bf16_t* dB) {
    constexpr int PAIRS = MI * NI / 2;
#pragma unroll
    for (int i = 0; i < PAIRS; ++i) {
      mma_one(a, b, 2 * i);
      mma_one(a, b, 2 * i + 1);
#pragma unroll
      for (int d = (i * (ACH + BCH)) / PAIRS; d < ((i + 1) * (ACH + BCH)) / PAIRS; ++d) issue_one(dA, dB, nullptr, d);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // One operand fragment of step ks: r = 0, 1 .. in the order the next step's MFMAs first need them
  // (A0, B0 .. B(NI-1), A1 .. A(MI-1)).
  auto read_one = [&](const bf16_t* cA, const bf16_t* cB, int ks, int r, bf16x8 (&a)[MI], bf16x8 (&b)[NI]) {
    const int pa = ((2 * ks + lg) ^ swz) * 8;
    if (r == 0 || r > NI) {
      const int t = r == 0 ? 0 : r - NI;
      a[t] = *(const bf16x8*)(cA + a_rd + t * 32 * BK + pa);
    } else {
      const int t = r - 1;
      if (NT) {
        b[t] = *(const bf16x8*)(cB + bt_rd + t * 32 * BK + pa);
      } else {
        const int krow = ks * 16 + 8 * lg + kq;
        const int seg = (wn * (2 * NI) + 2 * t + lhalf) ^ (kq << 1);
        const bf16x4 lo = lds_read_tr(cB + krow * BN + seg * 16 + bn_col);
        const bf16x4 hi = lds_read_tr(cB + (krow + 4) * BN + seg * 16 + bn_col);
        b[t] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      }
    }
  };
  // FUSE: the accumulator of this wave's 32 x 32 block of X A_t (row block wn of the wave's rows, transposed like acc),
  // the fragment of the slab of A_t for step ks (lane (li, lg): column li of the slab, 8 consecutive k), and the X
  // fragment of row block wn.
  f32x16 hacc;
#pragma unroll
  for (int v = 0; v < 16; ++v) hacc[v] = 0.f;
  auto read_e = [&](const bf16_t* cE, int ks) -> bf16x8 {
    const int krow = ks * 16 + 8 * lg + kq;
    const bf16x4 lo = lds_read_tr(cE + krow * rank + lhalf * 16 + bn_col);
    const bf16x4 hi = lds_read_tr(cE + (krow + 4) * rank + lhalf * 16 + bn_col);
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  };
  // the product of this step's slab fragment with the X fragment of row block wn, picked by selects on the (uniform)
  // wn: an index would send the fragments through scratch memory, and a branch per row block makes the compiler copy
  // the accumulator behind each MFMA
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  auto mma_h = [&](const bf16x8& e, const bf16x8 (&a)[MI]) {
    u32x4 x = __builtin_bit_cast(u32x4, a[0]);
#pragma unroll
    for (int t = 1; t < MI; ++t) {
      const u32x4 y = __builtin_bit_cast(u32x4, a[t]);
#pragma unroll
      for (int c = 0; c < 4; ++c) x[c] = wn == t ? y[c] : x[c];
    }
    hacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(e, __builtin_bit_cast(bf16x8, x), hacc, 0, 0, 0);
  };
  // One MFMA step from (a, b) with the operand reads of step ks_next of (cA, cB) into (an, bn) issued one per
  // MFMA in its shadow (skipped when rd is false), and, when LOADS, the loads of one tile into (dA, dB, dE) spread
  // over the MFMAs after them.  FUSE: one more product, e with the X fragment of row block wn, and the read of the
  // next step's fragment en of the slab cE.
  auto fused_step = [&](const bf16x8 (&a)[MI], const bf16x8 (&b)[NI], const bf16_t* cA, const bf16_t* cB, int ks_next,
                        bf16x8 (&an)[MI], bf16x8 (&bn)[NI], bool rd, auto LOADS, bf16_t* dA, bf16_t* dB,
                        const bf16x8& e, bf16x8& en, const bf16_t* cE, bf16_t* dE, uint32_t dP = 0, int o0 = 0,
                        int o2 = 0) {
    constexpr bool loads = decltype(LOADS)::value;
    constexpr int NM = MI * NI, NR = MI + NI, NL = NLD;
    if (FUSE && fuse_h) en = read_e(cE, ks_next);
#pragma unroll
    for (int m = 0; m < NM; ++m) {
      mma_one(a, b, m);
      if (rd) {
        if (m < NR) read_one(cA, cB, ks_next, m, an, bn);
        if (m == NM - 1) {                                   // a narrower tile has more fragments than MFMAs
#pragma unroll
          for (int r = NM; r < NR; ++r) read_one(cA, cB, ks_next, r, an, bn);
        }
      }
      if (loads) {
#pragma unroll
        for (int d = (m * NL) / NM; d < ((m + 1) * NL) / NM; ++d) issue_one(dA, dB, dE, d, dP, o0, o2);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    if (FUSE && fuse_h) {
      mma_h(e, a);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  static_assert(!SPLIT || (2 * A_ELEMS <= BM * BK && 2 * BN * BK <= BM * BK), "two stages per array");
  auto stA = [&](int s) -> bf16_t* {
    if (SPLIT) return (s < 2 ? sA0 : sA1) + (s & 1) * A_ELEMS;
    return s == 0 ? sA0 : (s == 1 ? sA1 : (s == 2 ? sA2 : sA3));
  };
  auto stB = [&](int s) -> bf16_t* {
    if (SPLIT) return (s < 2 ? sB0 : sB1) + (s & 1) * (BN * BK);
    return s == 0 ? sB0 : (s == 1 ? sB1 : (s == 2 ? sB2 : sB3));
  };
  auto stE = [&](int s) -> bf16_t* { return s == 0 ? sE0 : (s == 1 ? sE1 : (s == 2 ? sE2 : sE3)); };
  auto tile_barrier = [&]() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  };

  auto ldsP = [&](int st) -> uint32_t { return sm.pk_lds + (uint32_t)st * 1024u; };
  typedef __attribute__((address_space(3))) uint32_t lds_u32;
  // DIFFP: the entries o0 .. o2 - 1 of a tile (o1: the first of its second bucket), the first 256 of them in cP, added to
  // the W side of the tile in stage cB (landed, visible to the workgroup)
  auto patch_tile = [&](bf16_t* cB, uint32_t cP, int o0, int o1, int o2) {
    auto add_entry = [&](uint32_t w, int pos) {
      const int j = (int)(w >> 23), line = (int)((w >> 16) & 127u) + ((SPAN == 2 && o0 + pos >= o1) ? 128 : 0);
      bf16_t* e = NT ? cB + line * BK + (((j >> 3) ^ swz_row<BK>(line)) * 8) + (j & 7)
                     : cB + j * BN + (((line >> 4) ^ ((j & 3) << 1)) * 16) + (line & 15);
      // (the packed bf16 add of the LDS atomic unit in place of this read-modify-write was 5 % slower)
      *e = f32_to_bf16(bf16_to_f32(*e) + __uint_as_float(w << 16));
    };
    static_assert(NTHR >= 256, "one entry a thread covers what was staged");
    if (tid < o2 - o0 && tid < 256) add_entry(*(const lds_u32*)(uintptr_t)(cP + 4u * (uint32_t)tid), tid);   // (an LDS address, said as such)
    // a bucket pair with more entries than were staged: the rest from memory, in a loop of its own so that the usual case
    // holds no memory load whose wait would also wait for the tiles in flight
    if (o2 - o0 > 256)
      for (int pos = 256 + tid; pos < o2 - o0; pos += NTHR) add_entry(dlist[o0 + pos], pos);
  };
  // ---- prologue: tiles 0 .. PRE-1 in flight; tile 0 landed and visible; its first operands in registers
  constexpr int PRE = BK == 64 ? NST : NST - 1;
#pragma unroll
  for (int s0 = 0; s0 < PRE; ++s0) {
    prepare();
    if (DIFFP) bucket_offsets(s0, ps0[s0], ps1[s0], ps2[s0]);
    issue(stA(s0), stB(s0), stE(s0), ldsP(s0), ps0[s0], ps2[s0]);
  }
  if (DIFFP) bucket_offsets(PRE, nx0, nx1, nx2);
  wait_vmcnt<(PRE - 1) * NLD>();
  wait_lgkm0();
  tile_barrier();
  if (DIFFP && patch && ps2[0] > ps0[0]) {
    patch_tile(sB0, ldsP(0), ps0[0], ps1[0], ps2[0]);
    wait_lgkm0();
    tile_barrier();
  }

  bf16x8 a0[MI], b0[NI], a1[MI], b1[NI];
  bf16x8 e0 = {}, e1 = {};
  read_ops(sA0, sB0, 0, a0, b0);
  if (FUSE && fuse_h) e0 = read_e(sE0, 0);
  // FUSE: the K loop ends with the backbone; the adapter tile (its B_t side is fetched like any tile) follows below
  const int KT_loop = fuse_h ? KT : KT_total;

  if (BK == 64) {
    // Steps 0..2 run from registers read one step ahead; before the last step every wave has read all of this
    // stage and tile kt+1 has landed (the loads of the NST-2 tiles after it may stay in flight): barrier; then,
    // under the last step's MFMAs, the first operands of tile kt+1 are read and all loads of tile kt+NST are
    // issued into the stage just freed.
    for (int kt2 = 0; kt2 < KT_loop; kt2 += NST) {
#pragma unroll
      for (int u = 0; u < NST; ++u) {
        const int kt = kt2 + u;
        if (kt < KT_loop) {
          bf16_t* cA = stA(u);
          bf16_t* cB = stB(u);
          bf16_t* cE = stE(u);
          prepare();
          __builtin_amdgcn_sched_barrier(0);
          fused_step(a0, b0, cA, cB, 1, a1, b1, true, std::false_type{}, nullptr, nullptr, e0, e1, cE, nullptr);
          fused_step(a1, b1, cA, cB, 2, a0, b0, true, std::false_type{}, nullptr, nullptr, e1, e0, cE, nullptr);
          fused_step(a0, b0, cA, cB, 3, a1, b1, true, std::false_type{}, nullptr, nullptr, e0, e1, cE, nullptr);
          wait_vmcnt<(NST - 2) * NLD>();
          wait_lgkm0();
          tile_barrier();
          __builtin_amdgcn_sched_barrier(0);
          if (DIFFP) {
            // Tile kt + 1 has landed: its masked entries, then a second barrier, then it may be read.  (Waiting for the
            // tile one step earlier and adding the entries under the MFMAs of the third step was slower.)
            const int un = (u + 1) % NST;
            if (patch && ps2[un] > ps0[un]) {
              patch_tile(stB(un), ldsP(un), ps0[un], ps1[un], ps2[un]);
              wait_lgkm0();
              tile_barrier();
            }
            // this stage is refilled with tile kt + NST (PRE == NST here): its entries, and the offsets of the tile after
            ps0[u] = nx0; ps1[u] = nx1; ps2[u] = nx2;
            bucket_offsets(kt + NST + 1, nx0, nx1, nx2);
            __builtin_amdgcn_sched_barrier(0);
          }
          fused_step(a1, b1, stA((u + 1) % NST), stB((u + 1) % NST), 0, a0, b0, true, std::true_type{}, cA, cB, e1, e0,
                     stE((u + 1) % NST), cE, ldsP(u), ps0[u], ps2[u]);   // past the last tile: read, unused
          issue_done();
        }
      }
    }
  } else {
    for (int kt4 = 0; kt4 < KT_total; kt4 += NST) {
#pragma unroll
      for (int u = 0; u < NST; ++u) {
        const int kt = kt4 + u;
        if (kt < KT_total) {
          bf16_t* cA = stA(u);
          bf16_t* cB = stB(u);
          prepare();
          __builtin_amdgcn_sched_barrier(0);
          // first MFMA step.  The operand reads of the second step go out first (their latency hides under the
          // MFMAs); the refill of the stage computed from in the previous iteration with tile kt+3 (past the last
          // tile: zeros nobody reads) is spread between the MFMA pairs.
          read_ops(cA, cB, 1, a1, b1);
          __builtin_amdgcn_sched_barrier(0);
          mma_with_loads(a0, b0, stA((u + NST - 1) % NST), stB((u + NST - 1) % NST));
          issue_done();
          // tile kt+1 must have landed (the two newer ones may stay in flight) and every read of this stage be done
          wait_vmcnt<(NST - 2) * NLD>();
          wait_lgkm0();
          tile_barrier();
          __builtin_amdgcn_sched_barrier(0);
          // second MFMA step, with the first operands of the next tile read under it
          if (kt + 1 < KT_total) read_ops(stA((u + 1) % NST), stB((u + 1) % NST), 0, a0, b0);
          __builtin_amdgcn_sched_barrier(0);
          mma(a1, b1);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
  }
  // the refills issued past the last tile (zeros) must have landed before the stages are reused below
  wait_vmcnt<0>();
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");

  if (FUSE && fuse_h) {
    // The adapter tile.  Its W-side operand (rows of B_t) was fetched like any K-tile into the stage after the last
    // backbone tile's; its A side is Hs = s_t (X A_t) of the tile's rows, which the waves hold in hacc: this lane has
    // row wn*32 + li of the wave's row half and columns 8 j + 4 lg .. + 3.  Scaled, masked beyond the rank, rounded to
    // bf16, it goes into that stage in the layout the operand reads expect (pieces 4..7 of a row, contraction
    // indices 32..63, are zero), and from the tiles of the first column to memory.
    const int sK = KT % NST;
    bf16_t* hA = stA(sK);
    const bf16_t* hB = stB(sK);
    const int row_l = wm * (32 * MI) + wn * 32 + li;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int col = 8 * j + 4 * lg;
      float v[4];
#pragma unroll
      for (int c4 = 0; c4 < 4; ++c4) v[c4] = (col + c4 < rank) ? tk.scale * hacc[4 * j + c4] : 0.f;
      uint2 pk;
      pk.x = pack_bf16x2(v[0], v[1]);
      pk.y = pack_bf16x2(v[2], v[3]);
      *(uint2*)(hA + row_l * BK + ((j ^ swz) * 8) + 4 * lg) = pk;
      if (c0 == 0 && p.HsOut != nullptr && row_l < nrows && col < p.RP)
        *(uint2*)(p.HsOut + (size_t)(row0 + row_l) * p.RP + col) = pk;
    }
#pragma unroll
    for (int q = 0; q < 2; ++q)
      *(uint4*)(hA + row_l * BK + (((4 + 2 * lg + q) ^ swz) * 8)) = make_uint4(0, 0, 0, 0);
    wait_lgkm0();
    tile_barrier();
    const int nks = (rank + 15) >> 4;               // steps that carry data (rank <= 32: one or two)
    for (int ks = 0; ks < nks; ++ks) {
      read_ops(hA, hB, ks, a0, b0);
      mma(a0, b0);
    }
    wait_lgkm0();
    tile_barrier();                                 // the stages are reused as staging below
  }

  // ---- epilogue: aggregate, mask, store; 32 rows of the wave tile at a time through this wave's own array.
  constexpr int AREA = NI == 2 ? 2560 : 1280;     // elements of a staging area (5 KB or 2.5 KB)
  constexpr int AREAS = A_ELEMS / AREA;           // staging areas per A stage
  static_assert(32 * EPW <= AREA && NW <= AREAS * NST, "every wave has its own staging area");
  bf16_t* stage = stA(wave / AREAS) + (wave % AREAS) * AREA;
  constexpr int PPR = WCOLS / 8;                 // 16-byte pieces per staged row
  constexpr int RPI = 64 / PPR;                  // rows one wave instruction moves
  const int e_row = lane / PPR, e_pc = (lane % PPR) * 8;
  const bool scale_out = !NT && ia3;             // IA3 forward: Z = x W is saved first, then Y = Z * l_t
  const int passes = (scale_out && p.Zsave) ? 2 : 1;
  const bool z_only = !NT && tuning && p.Zsave;  // TUNING forward: x W goes to the saved region, Y is written by the bottleneck kernels
  for (int pass = 0; pass < passes; ++pass) {
    const bool to_z = z_only || pass + 1 < passes;
    bf16_t* dst = to_z ? p.Zsave + (size_t)(tk.zrow0 - tk.row_begin) * p.Nc : p.Out;   // indexed by the row in the batch
    if (scale_out && !to_z) {
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int c = c0 + wn * WCOLS + ni * 32 + 8 * j + 4 * lg;
          const bool in = c < p.Nc;                           // Nc is a multiple of 8: the four columns together
          const float l0 = in ? bf16_to_f32(Lvec[c]) : 0.f, l1 = in ? bf16_to_f32(Lvec[c + 1]) : 0.f;
          const float l2 = in ? bf16_to_f32(Lvec[c + 2]) : 0.f, l3 = in ? bf16_to_f32(Lvec[c + 3]) : 0.f;
#pragma unroll
          for (int mi = 0; mi < MI; ++mi) {
            acc[mi][ni][4 * j + 0] *= l0;
            acc[mi][ni][4 * j + 1] *= l1;
            acc[mi][ni][4 * j + 2] *= l2;
            acc[mi][ni][4 * j + 3] *= l3;
          }
        }
    }
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          uint2 v;
          v.x = pack_bf16x2(acc[mi][ni][4 * j + 0], acc[mi][ni][4 * j + 1]);
          v.y = pack_bf16x2(acc[mi][ni][4 * j + 2], acc[mi][ni][4 * j + 3]);
          *(uint2*)(stage + li * EPW + ni * 32 + 8 * j + 4 * lg) = v;
        }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int rr = 0; rr < 32 / RPI; ++rr) {
        const int ml = rr * RPI + e_row;
        const int m = wm * (32 * MI) + mi * 32 + ml;
        const int c = c0 + wn * WCOLS + e_pc;
        if (m < nrows && c < p.Nc) {
          uint4 v = *(const uint4*)(stage + ml * EPW + e_pc);
          if (sRow[m] == 0) v = make_uint4(0, 0, 0, 0);
          *(uint4*)(dst + (size_t)(row0 + m) * p.Nc + c) = v;
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      __builtin_amdgcn_wave_barrier();
    }
  }
}

// Workgroups 0 .. n_full-1 compute full tiles, slot by slot with the XCD in the low three bits of the index (the
// hardware deals consecutive workgroups round-robin to the eight XCDs, so one XCD's L2 sees neighbouring tiles).
// The workgroups after them compute the remaining tiles in pieces (tail_split = 2: two half-width tiles each;
// 4: four 128 x 128 quarters each); all pieces of a tile run on the same XCD.  The dispatcher hands out workgroups
// in index order, so the pieces start as the compute units finish their last full tile.
template <bool NT, int BK, bool FUSE, bool DIFFP>
__global__ __launch_bounds__(512, 1) void k_gemm_dma(const GemmParams p) {
  constexpr int STAGE_ELEMS = BM * BK;            // 16 KB (BK = 32, four stages) or 32 KB (BK = 64, two) per operand
  __shared__ __attribute__((aligned(1024))) bf16_t sA0[STAGE_ELEMS];
  __shared__ __attribute__((aligned(1024))) bf16_t sA1[STAGE_ELEMS];
  __shared__ __attribute__((aligned(1024))) bf16_t sA2[BK == 32 ? STAGE_ELEMS : 8];
  __shared__ __attribute__((aligned(1024))) bf16_t sA3[BK == 32 ? STAGE_ELEMS : 8];
  __shared__ __attribute__((aligned(1024))) bf16_t sB0[STAGE_ELEMS];
  __shared__ __attribute__((aligned(1024))) bf16_t sB1[STAGE_ELEMS];
  __shared__ __attribute__((aligned(1024))) bf16_t sB2[BK == 32 ? STAGE_ELEMS : 8];
  __shared__ __attribute__((aligned(1024))) bf16_t sB3[BK == 32 ? STAGE_ELEMS : 8];
  __shared__ __attribute__((aligned(1024))) bf16_t sE0[FUSE ? 2048 : 8];   // FUSE: [64][rank <= 32] slabs of A_t, 4 KB a stage
  __shared__ __attribute__((aligned(1024))) bf16_t sE1[FUSE ? 2048 : 8];
  __shared__ __attribute__((aligned(1024))) bf16_t sE2[FUSE ? 2048 : 8];
  __shared__ __attribute__((aligned(1024))) bf16_t sE3[FUSE ? 2048 : 8];
  __shared__ __attribute__((aligned(1024))) uint32_t sP[DIFFP ? 4 * 256 : 2];   // DIFFP: 256 packed entries a stage
  __shared__ int sOff[DIFFP ? 3 * 1024 : 2];                                      // DIFFP: K < 65536, so at most 1023 K-tiles
  __shared__ int sRow[256];
  const Smem sm = {sA0, sA1, sA2, sA3, sB0, sB1, sB2, sB3, sRow, sE0, sE1, sE2, sE3, (uint32_t)(uintptr_t)(lds_void_ptr)sP, sOff};
  const int b = blockIdx.x;
  // the start stamps wait in the buffer itself (words 2, 3), so that nothing stays live across the tile
  if (p.clk != nullptr && b == 0 && threadIdx.x == 0) { p.clk[2] = clock64(); p.clk[3] = wall_clock64(); }
  if (!FUSE && b < p.n_full) {                    // a launch with the down-projection in the loop has pieces only
    gemm_tile<NT, 4, 4, 2, BK, false, DIFFP>(p, b, 0, 0, sm);
  } else if (p.tail_split == 2) {
    const int t = b - p.n_full;                                       // n_full is a multiple of 8
    gemm_tile<NT, 4, 4, 1, BK, FUSE, DIFFP>(p, p.n_full + (((t >> 4) << 3) | (t & 7)), (t >> 3) & 1, 0, sm);
  } else {
    const int t = b - p.n_full;
    gemm_tile<NT, 2, 2, 2, BK, FUSE, DIFFP>(p, p.n_full + (((t >> 5) << 3) | (t & 7)), (t >> 3) & 1, (t >> 4) & 1, sm);
  }
  if (p.clk != nullptr && blockIdx.x == 0 && threadIdx.x == 0) {
    atomicAdd(p.clk, (unsigned long long)clock64() - p.clk[2]);
    atomicAdd(p.clk + 1, (unsigned long long)wall_clock64() - p.clk[3]);
  }
}

// Number of compute units, asked once.
int compute_units() {
  static int n = 0;
  if (n == 0) {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0) n = v;
    else n = 256;
  }
  return n;
}

// The tile plan of a launch: whole tiles for the full rounds of workgroups, the rest as halves or quarters.
struct TilePlan { int n_m, n_n, per_xcd, n_full, tail_split, grid; bool narrow; };
TilePlan plan_tiles(const CallCtx& c, int Kc, int Nc) {
  TilePlan t{};
  t.n_m = (int)c.st->items[TS256].size();
  t.n_n = (Nc + TILE_N - 1) / TILE_N;
  const int total = t.n_m * t.n_n;
  t.per_xcd = (total + 7) / 8;
  // One workgroup per compute unit at a time: the tiles left after the last full round would keep a fraction of
  // the units busy for a whole tile time.  When they fit four times, they run as quarters, when twice, as
  // half-width tiles.
  static const bool no_halves = getenv("MUX_GEMM_NO_HALF_TILES") != nullptr;
  static const bool no_quarters = getenv("MUX_GEMM_NO_QUARTER_TILES") != nullptr;
  static const bool narrow = getenv("MUX_GEMM_BK32") != nullptr;
  const int ncu = compute_units();
  const int full_slots = (total / ncu) * (ncu / 8);          // per-XCD slots covered by whole rounds
  const int rem = total - full_slots * 8;
  int tail_slots = 0;
  if (!no_halves && ncu % 8 == 0 && rem > 0 && 2 * rem <= ncu) tail_slots = t.per_xcd - full_slots;
  t.tail_split = (!no_quarters && 4 * rem <= ncu) ? 4 : 2;
  t.n_full = 8 * (t.per_xcd - tail_slots);
  t.grid = t.n_full + 8 * t.tail_split * tail_slots;
  t.narrow = narrow || Kc % 64 != 0;
  return t;
}

template <bool NT>
mux_status launch(const CallCtx& c, const bf16_t* Ain, const bf16_t* Ext, bf16_t* Out, bf16_t* Zsave, int Kc, int Nc,
                  bool fuse_down) {
  GemmParams p;
  p.dtab = c.dtab; p.tasks = *c.tref; p.Ain = Ain; p.W = (const bf16_t*)c.W; p.ldw = c.ldw; p.Ext = Ext; p.Out = Out;
  p.Zsave = Zsave; p.Kc = Kc; p.Nc = Nc; p.RP = c.RP;
  p.HsOut = fuse_down ? (bf16_t*)Ext : nullptr;
  const TilePlan t = plan_tiles(c, Kc, Nc);
  p.n_m = t.n_m; p.n_n = t.n_n; p.per_xcd = t.per_xcd; p.n_full = t.n_full; p.tail_split = t.tail_split;
  p.AinScaled = (const bf16_t*)c.dYs;
  p.Wdiff = (const bf16_t*)c.diffW; p.wdiff_stride = c.diffW_stride;
  p.DiffPack = (const uint32_t*)c.diffPack;
  p.clk = diag_clock_buffer();
  if (t.n_m * t.n_n == 0) return MUX_OK;
  if (fuse_down && (NT || t.narrow || t.n_full != 0)) return fail(MUX_ERR_UNSUPPORTED, "gemm: this launch cannot carry the down-projection");
  if (p.DiffPack != nullptr && (t.narrow || fuse_down)) return fail(MUX_ERR_UNSUPPORTED, "gemm: this launch cannot add masked entries in the tile loop");
  if (!t.narrow) {
    if (!NT && fuse_down) MUX_LAUNCH("gemm_nn", (k_gemm_dma<false, 64, true, false>), dim3(t.grid), dim3(512), 0, c.stream, p);
    else if (p.DiffPack != nullptr) MUX_LAUNCH(NT ? "gemm_nt" : "gemm_nn", (k_gemm_dma<NT, 64, false, true>), dim3(t.grid), dim3(512), 0, c.stream, p);
    else MUX_LAUNCH(NT ? "gemm_nt" : "gemm_nn", (k_gemm_dma<NT, 64, false, false>), dim3(t.grid), dim3(512), 0, c.stream, p);
  } else {
    MUX_LAUNCH(NT ? "gemm_nt" : "gemm_nn", (k_gemm_dma<NT, 32, false, false>), dim3(t.grid), dim3(512), 0, c.stream, p);
  }
  return MUX_OK;
}

}  // namespace

// The pipelined kernel needs what the register-staged one needs, a contraction length that is a multiple of 32,
// and in the backward every LoRA rank a multiple of 8 (rows of A_t are read in 16-byte pieces).
bool gemm_dma_supported(const CallCtx& c, bool backward) {
  if (!gemm_mfma_supported(c)) return false;
  if ((backward ? c.N : c.K) % 32 != 0) return false;      // no K-tail masks in the pipelined loop
  if (backward)
    for (const HostTask& ht : c.st->tasks)
      if (ht.kind == MUX_ADAPTER_LORA && (ht.rank & 7) != 0) return false;
  return true;
}

// Can the forward of this call form Hs = s_t X A_t inside the backbone tile loop?  The kernel can when the launch is
// made of half or quarter tiles only, with 64-deep stages, LoRA ranks up to 32 that are multiples of 8 (A_t is read in
// place) and no Adapter-Tuning task.  It is chosen for launches of quarter tiles (at most a quarter of the compute
// units' worth of 256 x 256 tiles): there the loop waits on loads, the extra product per step costs about 0.13 us per
// 64 of K, and the launch it saves costs 9 to 25 us; in launches of half tiles the extra product costs more than the
// launch (measured 4 to 13 % slower).  MUX_GEMM_FUSE_DOWN (read once): 0 never, 2 in launches of half tiles as well.
bool gemm_dma_fuses_down(const CallCtx& c) {
  static const int mode = [] { const char* e = getenv("MUX_GEMM_FUSE_DOWN"); return e == nullptr ? 1 : atoi(e); }();
  if (mode == 0 || !gemm_dma_supported(c, false)) return false;
  if (c.st->n_lora == 0 || c.st->n_tuning > 0 || !c.lora_natural || c.st->r_max > 32 || c.diffPack != nullptr) return false;
  const TilePlan t = plan_tiles(c, c.K, c.N);
  if (t.narrow || t.n_full != 0 || t.n_m * t.n_n == 0) return false;
  return t.tail_split == 4 || mode == 2;
}

mux_status gemm_dma_forward(const CallCtx& c, const void* X, const void* Hs, void* Y, void* Z, bool fuse_down) {
  return launch<false>(c, (const bf16_t*)X, (const bf16_t*)Hs, (bf16_t*)Y, (bf16_t*)Z, c.K, c.N, fuse_down);
}

mux_status gemm_dma_backward(const CallCtx& c, const void* dY, const void* Gs, void* dX) {
  return launch<true>(c, (const bf16_t*)dY, (const bf16_t*)Gs, (bf16_t*)dX, nullptr, c.N, c.K, false);
}

}  // namespace mux
