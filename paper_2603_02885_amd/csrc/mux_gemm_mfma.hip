// Backbone GEMM on the matrix cores (bf16 in, fp32 accumulate), with the adapter's up-projection
// folded in as one extra K-tile and the aggregate / padding mask applied in the epilogue.
//
//   forward  (NN):  Y[T,N]  = mask * ( X[T,K] W[K,N]      + Hs[T,r] B_t[r,N] )      Eq. 1 + LoRA + Add
//   backward (NT):  dX[T,K] = mask * ( dY[T,N] W[K,N]^T   + Gs[T,r] A_t[K,r]^T )    Eq. 2 + LoRA
//
// Hs = s_t (x A_t) and Gs = s_t (g B_t^T) are bf16 and already carry the scale, so the adapter
// branch is literally more contraction steps of the same tile:  [X | Hs] [W ; B_t].
//
// Tiling for gfx950: 256x256 output tile per workgroup of 4 waves (2x2), 128x128 per wave as 4x4
// v_mfma_f32_32x32x16_bf16 tiles (256 accumulator registers per lane), BK = 64, two LDS stages
// (147 KB of the 160 KB), register-staged global prefetch of the next K-tile.
// W is stored [K,N]: the forward needs it k-major per lane, which ds_read_b64_tr_b16 delivers
// straight from the natural [k][n] LDS tile; the backward reads W rows as they are.
// Workgroup ids are dealt round-robin to the 8 XCDs, so each XCD gets a contiguous range of a
// grouped tile order and its L2 sees a compact block of tiles.
#include "mux_device_utils.h"

namespace mux {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int PITCH_K = BK + 8;     // elements; rows of a [rows][BK] tile (144 B: conflict-free 16 B reads)
constexpr int PITCH_N = BN + 32;    // elements; rows of the forward's [BK][BN] tile (576 B)
constexpr int TILE_ELEMS = BM * PITCH_K;                       // == BK * PITCH_N == 18432
static_assert(BM * PITCH_K == BK * PITCH_N, "both tile layouts use the same LDS footprint");
constexpr int SMEM_BYTES = 2 * 2 * TILE_ELEMS * 2 + 256 * 4;   // 2 stages x (A,B) + row flags
constexpr int TS256 = 2;
constexpr int EP_PITCH = 128 + 8;    // elements; epilogue staging rows of one wave (4 x 128 x 136 x 2 B = 139264 B)

struct GemmParams {
  const int32_t* dtab;
  const bf16_t* Ain;   // [T, Kc]  activations (X or dY)
  const bf16_t* W;     // [K, ldw]
  int64_t ldw;
  const bf16_t* Ext;   // [T, RP]  Hs or Gs (may be null without LoRA tasks)
  bf16_t* Out;         // [T, Nc]
  bf16_t* Zsave;       // forward: x W of IA3_OUT rows (may be null)
  int Kc, Nc, RP;
  int n_m, n_n, per_xcd;
  int only_ia3;        // process IA3_OUT items only (the pipelined kernel took the rest)
  const bf16_t* Wdiff; // merged weights W + M_t * delta_t of the Diff-Pruning tasks, `wdiff_stride` elements apart (or null)
  int64_t wdiff_stride;
  const bf16_t* Prep;  // backward: prepared input rows of the TUNING tasks (dY + p D_t^T), [z_rows, Kc], indexed like the saved x W
  TaskRef tasks;
};

__device__ __forceinline__ uint4 zero4() { return make_uint4(0, 0, 0, 0); }

// 8 bf16 scaled elementwise by 8 bf16, rounded back to bf16
__device__ __forceinline__ uint4 mul_bf16x8(uint4 a, uint4 b) {
  uint4 r;
  const uint32_t* pa = (const uint32_t*)&a;
  const uint32_t* pb = (const uint32_t*)&b;
  uint32_t* pr = (uint32_t*)&r;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const float lo = __uint_as_float(pa[e] << 16) * __uint_as_float(pb[e] << 16);
    const float hi = __uint_as_float(pa[e] & 0xffff0000u) * __uint_as_float(pb[e] & 0xffff0000u);
    pr[e] = pack_bf16x2(lo, hi);
  }
  return r;
}

typedef __amdgpu_buffer_rsrc_t rsrc_t;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
constexpr uint32_t OOB = 0x80000000u;   // beyond any num_records: the load returns zeros

// raw buffer (stride 0) over `bytes` bytes starting at p
__device__ __forceinline__ rsrc_t make_rsrc(const void* p, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc((void*)p, 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ uint4 buf_load16(rsrc_t r, uint32_t byte_off) {
  const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)byte_off, 0, 0);
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ uint16_t buf_load2(rsrc_t r, uint32_t byte_off) {
  return (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(r, (int)byte_off, 0, 0);
}

__device__ __forceinline__ bf16x4 lds_read_tr(const bf16_t* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4bf16((__attribute__((address_space(3))) bf16x4*)p);
}

template <bool NT>
__global__ __launch_bounds__(256, 1) void k_gemm(const GemmParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16_t* sA = (bf16_t*)smem_raw;                 // [2][TILE_ELEMS]
  bf16_t* sB = sA + 2 * TILE_ELEMS;               // [2][TILE_ELEMS]
  int* sRow = (int*)(sB + 2 * TILE_ELEMS);        // [256] 1 = row is a real token of this item

  // ---- which tile: XCD-aware grouped order
  const int total = p.n_m * p.n_n;
  const int L = (blockIdx.x & 7) * p.per_xcd + (blockIdx.x >> 3);
  if (L >= total) return;
  constexpr int GROUP = 4;
  const int width = GROUP * p.n_n;
  const int first_m = (L / width) * GROUP;
  const int gsize = p.n_m - first_m < GROUP ? p.n_m - first_m : GROUP;
  const int tm = first_m + (L % width) % gsize;
  const int tn = (L % width) / gsize;

  const ItemView it = load_item(p.dtab, TS256, tm);
  const int c0 = tn * BN;                          // first output column
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  if (p.only_ia3 && !(it.task >= 0 && it.nvalid > 0 && get_task_kind(p.tasks, it.task) == MUX_ADAPTER_IA3_OUT)) return;

  {
    const int row = it.row0 + tid;
    sRow[tid] = (it.task >= 0 && tid < it.nrows && row_is_valid(p.dtab, row)) ? 1 : 0;
  }

  if (it.task < 0 || it.nvalid == 0) {             // rows of no task, or padding only: zeros out
    for (int e = tid; e < it.nrows * (BN / 8); e += 256) {
      const int m = e / (BN / 8), c = c0 + (e % (BN / 8)) * 8;
      if (c < p.Nc) *(uint4*)(p.Out + (size_t)(it.row0 + m) * p.Nc + c) = zero4();
    }
    return;
  }

  const DevTask tk = get_task(p.tasks, it.task);
  const bool lora = tk.kind == MUX_ADAPTER_LORA;
  const bool ia3 = tk.kind == MUX_ADAPTER_IA3_OUT;
  const bool tuning = tk.kind == MUX_ADAPTER_TUNING;   // forward: only x W is produced here (saved); backward: rows from Prep
  const int rank = tk.rank;
  const bf16_t* adapterB = NT ? (const bf16_t*)tk.A : (const bf16_t*)tk.B;  // the operand paired with Ext
  const bf16_t* Lvec = (const bf16_t*)tk.L;

  // ---- per-thread load geometry.  All global reads are buffer loads: a masked-off piece gets an
  // out-of-range offset and the hardware returns zeros, so the loop has no branches.
  // [rows][BK] tiles: 8 rows per thread (row = tid/8 + 32 q), one 16-byte piece (8 elements) per row
  const int a_r = tid >> 3, a_pc = (tid & 7) * 8;
  // forward's [BK][BN] tile: 8 k-rows per thread (k = tid/32 + 8 q), piece n = (tid%32)*8
  const int b_k = tid >> 5, b_pc = (tid & 31) * 8;

  uint32_t a_ok = 0;     // bit q: A row a_r + 32 q is a real token of this item
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    const int m = a_r + 32 * q, row = it.row0 + m;
    if (m < it.nrows && row_is_valid(p.dtab, row)) a_ok |= 1u << q;
  }
  uint32_t b_ok = 0;     // NT: bit q: output column c0 + a_r + 32 q exists
#pragma unroll
  for (int q = 0; q < 8; ++q)
    if (c0 + a_r + 32 * q < p.Nc) b_ok |= 1u << q;
  const bool bcol_ok = c0 + b_pc < p.Nc;   // NN: this thread's 8 output columns exist

  const int KT = (p.Kc + BK - 1) / BK;
  const int KT_total = KT + (lora ? 1 : 0);

  // buffer resources (byte offsets must stay below 2^31: checked on the host)
  const rsrc_t rA = make_rsrc((NT && tuning) ? p.Prep + (size_t)(tk.zrow0 + it.row0 - tk.row_begin) * p.Kc : p.Ain + (size_t)it.row0 * p.Kc,
                              (uint32_t)it.nrows * (uint32_t)p.Kc * 2u);
  const bf16_t* Wt = task_weight(tk, p.W, p.Wdiff, p.wdiff_stride);
  const rsrc_t rW = NT ? make_rsrc(Wt + (size_t)c0 * p.ldw, (uint32_t)((size_t)(p.Nc - c0 < BN ? p.Nc - c0 : BN) * p.ldw * 2))
                       : make_rsrc(Wt + c0, (uint32_t)(((size_t)(p.Kc - 1) * p.ldw + (p.Nc - c0)) * 2));
  const rsrc_t rE = make_rsrc(lora ? p.Ext + (size_t)it.row0 * p.RP : p.Ain, lora ? (uint32_t)it.nrows * (uint32_t)p.RP * 2u : 0u);
  const rsrc_t rP = NT ? make_rsrc(lora ? adapterB + (size_t)c0 * rank : p.Ain,
                                   lora ? (uint32_t)(p.Nc - c0 < BN ? p.Nc - c0 : BN) * (uint32_t)rank * 2u : 0u)
                       : make_rsrc(lora ? adapterB + c0 : p.Ain, lora ? (uint32_t)(((size_t)(rank - 1) * p.Nc + (p.Nc - c0)) * 2) : 0u);
  const uint32_t a_off = ((uint32_t)a_r * (uint32_t)p.Kc + (uint32_t)a_pc) * 2u;     // + q * 32 rows + k0
  const uint32_t a_rowstep = 32u * (uint32_t)p.Kc * 2u;
  const uint32_t wt_off = (uint32_t)(((size_t)a_r * p.ldw + a_pc) * 2);               // NT
  const uint32_t wt_rowstep = (uint32_t)(32 * p.ldw * 2);
  const uint32_t wn_off = (uint32_t)(((size_t)b_k * p.ldw + b_pc) * 2);               // NN
  const uint32_t wn_rowstep = (uint32_t)(8 * p.ldw * 2);

  uint4 ra[8], rb[8];

  auto load_global = [&](int kt) {
    if (kt < KT) {
      const int k0 = kt * BK;
      const bool kin = k0 + a_pc < p.Kc;          // this piece is inside the contraction range
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const bool ok = ((a_ok >> q) & 1u) && kin;
        ra[q] = buf_load16(rA, ok ? a_off + q * a_rowstep + (uint32_t)k0 * 2u : OOB);
      }
      if (NT) {   // rows of W are output columns, contraction contiguous
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          const bool ok = ((b_ok >> q) & 1u) && kin;
          rb[q] = buf_load16(rW, ok ? wt_off + q * wt_rowstep + (uint32_t)k0 * 2u : OOB);
        }
      } else {    // natural [k][n] rows of W
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          const bool ok = bcol_ok && (k0 + b_k + 8 * q < p.Kc);
          rb[q] = buf_load16(rW, ok ? wn_off + q * wn_rowstep + (uint32_t)((size_t)k0 * p.ldw * 2) : OOB);
        }
      }
    } else {
      // adapter tile: contraction index j < rank (Ext holds zeros on padding rows and beyond rank)
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const bool ok = (a_r + 32 * q < it.nrows) && a_pc < p.RP;
        ra[q] = buf_load16(rE, ok ? (uint32_t)(((a_r + 32 * q) * p.RP + a_pc) * 2) : OOB);
      }
      if (NT) {   // A_t[c][j], row pitch = rank elements
        if ((rank & 7) == 0) {
#pragma unroll
          for (int q = 0; q < 8; ++q) {
            const bool ok = ((b_ok >> q) & 1u) && a_pc < rank;
            rb[q] = buf_load16(rP, ok ? (uint32_t)(((a_r + 32 * q) * rank + a_pc) * 2) : OOB);
          }
        } else {  // rows of A_t are not 16-byte aligned: element loads
#pragma unroll
          for (int q = 0; q < 8; ++q) {
            uint32_t w[4];
#pragma unroll
            for (int e = 0; e < 8; e += 2) {
              const bool ok0 = ((b_ok >> q) & 1u) && a_pc + e < rank, ok1 = ((b_ok >> q) & 1u) && a_pc + e + 1 < rank;
              const uint32_t o = (uint32_t)(((a_r + 32 * q) * rank + a_pc + e) * 2);
              w[e >> 1] = (uint32_t)buf_load2(rP, ok0 ? o : OOB) | ((uint32_t)buf_load2(rP, ok1 ? o + 2u : OOB) << 16);
            }
            rb[q] = make_uint4(w[0], w[1], w[2], w[3]);
          }
        }
      } else {    // B_t[j][n], row pitch = Nc
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          const bool ok = bcol_ok && (b_k + 8 * q < rank);
          rb[q] = buf_load16(rP, ok ? (uint32_t)(((size_t)(b_k + 8 * q) * p.Nc + b_pc) * 2) : OOB);
        }
      }
    }
  };

  auto store_lds = [&](int buf, int kt) {
    bf16_t* dA = sA + buf * TILE_ELEMS;
    bf16_t* dB = sB + buf * TILE_ELEMS;
    if (NT && ia3 && kt < KT) {      // backward of the output scale: g * l_t along the contraction
      const int k0 = kt * BK;
      const uint4 lv = (k0 + a_pc < p.Kc) ? *(const uint4*)(Lvec + k0 + a_pc) : zero4();
#pragma unroll
      for (int q = 0; q < 8; ++q) ra[q] = mul_bf16x8(ra[q], lv);
    }
#pragma unroll
    for (int q = 0; q < 8; ++q) *(uint4*)(dA + (a_r + 32 * q) * PITCH_K + a_pc) = ra[q];
    if (NT) {
#pragma unroll
      for (int q = 0; q < 8; ++q) *(uint4*)(dB + (a_r + 32 * q) * PITCH_K + a_pc) = rb[q];
    } else {
#pragma unroll
      for (int q = 0; q < 8; ++q) *(uint4*)(dB + (b_k + 8 * q) * PITCH_N + b_pc) = rb[q];
    }
  };

  f32x16 acc[4][4];
#pragma unroll
  for (int mi = 0; mi < 4; ++mi)
#pragma unroll
    for (int ni = 0; ni < 4; ++ni)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;

  const int li = lane & 31, lg = lane >> 5;
  const int l16 = lane & 15, lhalf = (lane >> 4) & 1;

  auto compute = [&](int buf) {
    const bf16_t* cA = sA + buf * TILE_ELEMS + (wm * 128 + li) * PITCH_K + 8 * lg;
    const bf16_t* cBk = sB + buf * TILE_ELEMS + (wn * 128 + li) * PITCH_K + 8 * lg;                      // NT
    const bf16_t* cBn = sB + buf * TILE_ELEMS + (8 * lg + (l16 >> 2)) * PITCH_N + wn * 128 + 16 * lhalf + 4 * (l16 & 3);  // NN
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 a[4], b[4];
#pragma unroll
      for (int mi = 0; mi < 4; ++mi) a[mi] = *(const bf16x8*)(cA + mi * 32 * PITCH_K + ks * 16);
#pragma unroll
      for (int ni = 0; ni < 4; ++ni) {
        if (NT) {
          b[ni] = *(const bf16x8*)(cBk + ni * 32 * PITCH_K + ks * 16);
        } else {
          const bf16x4 lo = lds_read_tr(cBn + (ks * 16) * PITCH_N + ni * 32);
          const bf16x4 hi = lds_read_tr(cBn + (ks * 16 + 4) * PITCH_N + ni * 32);
          b[ni] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        }
      }
#pragma unroll
      for (int mi = 0; mi < 4; ++mi)
#pragma unroll
        for (int ni = 0; ni < 4; ++ni)
          acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mi], b[ni], acc[mi][ni], 0, 0, 0);
    }
  };

  // ---- pipeline: global -> registers -> LDS stage, compute from the other stage
  load_global(0);
  store_lds(0, 0);
  __syncthreads();
  for (int kt = 0; kt < KT_total; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < KT_total) load_global(kt + 1);
    compute(buf);
    if (kt + 1 < KT_total) store_lds(buf ^ 1, kt + 1);
    __syncthreads();
  }

  // ---- epilogue: aggregate, mask, store.  Each wave stages its 128x128 tile as bf16 in its own
  // LDS region (the K-loop stages are free now), then writes rows with 16-byte coalesced stores.
  bf16_t* stage = (bf16_t*)smem_raw + wave * (128 * EP_PITCH);
  float lcol[4];
#pragma unroll
  for (int ni = 0; ni < 4; ++ni) {
    const int c = c0 + wn * 128 + ni * 32 + li;
    lcol[ni] = (!NT && ia3 && c < p.Nc) ? bf16_to_f32(Lvec[c]) : 1.f;
  }
  const int passes = (!NT && ia3 && p.Zsave) ? 2 : 1;     // IA3 forward also saves x W before the scale
  const bool z_only = !NT && tuning && p.Zsave;           // TUNING forward: x W goes to the saved region, Y is written later
  for (int pass = 0; pass < passes; ++pass) {
    const bool to_z = z_only || (passes == 2 && pass == 0);
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
      for (int ni = 0; ni < 4; ++ni)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int m = mi * 32 + 8 * (v >> 2) + 4 * lg + (v & 3);
          const float y = to_z ? acc[mi][ni][v] : acc[mi][ni][v] * lcol[ni];
          stage[m * EP_PITCH + ni * 32 + li] = f32_to_bf16(y);
        }
    __syncthreads();
    bf16_t* dst = to_z ? p.Zsave + (size_t)(tk.zrow0 - tk.row_begin) * p.Nc : p.Out;
#pragma unroll 4
    for (int rr = 0; rr < 32; ++rr) {
      const int ml = rr * 4 + (lane >> 4);            // row inside the wave tile
      const int m = wm * 128 + ml;                    // row inside the workgroup tile
      const int c = c0 + wn * 128 + (lane & 15) * 8;
      if (m < it.nrows && c < p.Nc) {
        uint4 v = *(const uint4*)(stage + ml * EP_PITCH + (lane & 15) * 8);
        if (sRow[m] == 0) v = zero4();
        *(uint4*)(dst + (size_t)(it.row0 + m) * p.Nc + c) = v;
      }
    }
    __syncthreads();
  }
}

template <bool NT>
mux_status launch(const CallCtx& c, const bf16_t* Ain, const bf16_t* Ext, bf16_t* Out, bf16_t* Zsave, int Kc, int Nc,
                  int only_ia3) {
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)k_gemm<NT>, hipFuncAttributeMaxDynamicSharedMemorySize, SMEM_BYTES);
    if (e != hipSuccess) return fail(MUX_ERR_DEVICE, std::string("hipFuncSetAttribute: ") + hipGetErrorString(e));
    attr_set = true;
  }
  GemmParams p;
  p.dtab = c.dtab; p.tasks = *c.tref; p.Ain = Ain; p.W = (const bf16_t*)c.W; p.ldw = c.ldw; p.Ext = Ext; p.Out = Out;
  p.Zsave = Zsave; p.Kc = Kc; p.Nc = Nc; p.RP = c.RP;
  p.Wdiff = (const bf16_t*)c.diffW; p.wdiff_stride = c.diffW_stride;
  p.n_m = (int)c.st->items[TS256].size();
  p.n_n = (Nc + BN - 1) / BN;
  const int total = p.n_m * p.n_n;
  if (total == 0) return MUX_OK;
  p.per_xcd = (total + 7) / 8;
  p.only_ia3 = only_ia3;
  p.Prep = (const bf16_t*)c.dYs;
  MUX_LAUNCH(NT ? (only_ia3 ? "gemm_nt_ia3" : "gemm_nt_regstaged") : "gemm_nn_regstaged", k_gemm<NT>, dim3(p.per_xcd * 8), dim3(256), SMEM_BYTES, c.stream, p);
  return MUX_OK;
}

}  // namespace

bool gemm_mfma_supported(const CallCtx& c) {
  // 16-byte global loads need rows of X, dY, W, Hs and B_t to start 16-byte aligned
  // and the 32-bit buffer offsets need W and the largest row group a kernel builds one descriptor over (1024 rows of
  // activations; rows parked at offset 2^31 must stay out of range) below 2 GiB
  const int64_t big = (int64_t)1 << 31;
  return (c.K % 8 == 0) && (c.N % 8 == 0) && (c.ldw % 8 == 0) && (((uintptr_t)c.W & 15) == 0) &&
         ((int64_t)c.K * c.ldw * 2 < big) && ((int64_t)1024 * (c.K > c.N ? c.K : c.N) * 2 < big);
}

mux_status gemm_mfma_forward(const CallCtx& c, const void* X, const void* Hs, void* Y, void* Z) {
  return launch<false>(c, (const bf16_t*)X, (const bf16_t*)Hs, (bf16_t*)Y, (bf16_t*)Z, c.K, c.N, 0);
}

mux_status gemm_mfma_backward(const CallCtx& c, const void* dY, const void* Gs, void* dX, int only_ia3) {
  return launch<true>(c, (const bf16_t*)dY, (const bf16_t*)Gs, (bf16_t*)dX, nullptr, c.N, c.K, only_ia3);
}

}  // namespace mux
