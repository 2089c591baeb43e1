// Attention step of a chunk-aligned batch (section 3.5): causal softmax attention of every sequence on its own,
// forward and backward, bf16 storage, fp32 accumulation on the matrix cores (v_mfma_f32_32x32x16_bf16).
//
// Work item = a block of 128 tokens of one sequence x one head; four waves, 32 tokens each.  All three kernels keep
// the wave's own tokens on the N side of every product (lane l owns token l % 32; its two half-waves split the
// other index), so that softmax statistics, log-sum-exp and the dO.O term are per-lane scalars and a probability
// tile leaves the accumulators already in the layout of the next product's B operand:
//   forward   S^T = K Q^T (keys x queries)      -> P^T -> O^T  += V^T P^T          online softmax over key tiles
//   dQ        S^T, dP^T = V dO^T                -> dS^T -> dQ^T += K^T dS^T
//   dK, dV    S = Q K^T, dP = dO V^T (queries x keys, the wave owns keys) -> dV^T += dO^T P, dK^T += Q^T dS
// The operand that has to be read across rows (V^T, K^T, dO^T, Q^T) comes from a row-major LDS tile through
// ds_read_b64_tr_b16.  A sum over 16 tokens may take them in any order as long as both operands agree; the order
// used is the one the accumulator layout gives: slot i of half-wave h <-> token 8 (i / 4) + 4 h + i % 4.
// Every output element has one owner; nothing is accumulated across workgroups, results repeat bit for bit.
#include "mux_attn.h"
#include "mux_device_utils.h"

namespace mux {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int BLK = kAttnBlockRows;
constexpr int TILE = 64;        // tokens of the other side staged per step
// What follows from the head dimension D (a multiple of 16 up to 128; built for 64, 80, 96 and 128).
template <int D>
struct Dim {
  static_assert(D % 16 == 0 && D >= 32 && D <= 128, "head dimension");
  static constexpr int KS = D / 16;          // contraction steps of 16 over the head dimension
  static constexpr int DT = (D + 31) / 32;   // 32-column tiles of an output row (the last may be half used)
  static constexpr int DP = 32 * DT;         // columns of a staged tile; those from D on stay zero
  static constexpr int KP = DP + 8;          // LDS row pitch (elements) of a tile that is only read along rows
  static constexpr int TP = DP + 16;         // ... of a tile that is also read across rows
};
constexpr float LOG2E = 1.4426950408889634f, LN2 = 0.6931471805599453f;

// A wave in a run of matrix products is served before the other wave of its SIMD, whose vector instructions then
// fill the issue slots between the products (forward and dQ: 2 % faster; dK/dV: no change, not used there).
#define ATTN_PRIO_HIGH() __builtin_amdgcn_s_setprio(2)
#define ATTN_PRIO_LOW() __builtin_amdgcn_s_setprio(0)

struct AttnParams {
  const int32_t* dtab;
  const bf16_t *Q, *K, *V, *O, *dO;
  bf16_t *Out, *dQ, *dK, *dV;
  float* lse;         // [H][T], natural log
  float* delta;       // [H][T]
  int64_t ldq, ldk, ldv, ldo;
  int T, H, Hkv;      // query heads, key/value heads (H = group * Hkv: query head h reads key/value head h / group)
  float scale;
};

__device__ __forceinline__ bf16x4 lds_read_tr(const bf16_t* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4bf16((__attribute__((address_space(3))) bf16x4*)p);
}
__device__ __forceinline__ f32x16 mma(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
// 2^x by the hardware instruction (arguments here are <= 0 or masked afterwards; denormal results may flush to zero)
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ bf16x8 zero8() { return __builtin_bit_cast(bf16x8, uint4{0u, 0u, 0u, 0u}); }
// accumulator elements 8u .. 8u+7 as a B operand
__device__ __forceinline__ bf16x8 pack8(const f32x16& v, int u) {
  uint4 r;
  r.x = pack_bf16x2(v[8 * u + 0], v[8 * u + 1]);
  r.y = pack_bf16x2(v[8 * u + 2], v[8 * u + 3]);
  r.z = pack_bf16x2(v[8 * u + 4], v[8 * u + 5]);
  r.w = pack_bf16x2(v[8 * u + 6], v[8 * u + 7]);
  return __builtin_bit_cast(bf16x8, r);
}
// A operand read across the rows of a row-major tile: column c0 + lane % 32, the 8 rows 4h + {0..3}, 8 + 4h + {0..3} from row0
template <int TP>
__device__ __forceinline__ bf16x8 read_across(const bf16_t* tile, int row0, int c0, int lane) {
  const int j = lane & 15, grp = lane >> 4;
  const bf16_t* p = tile + (row0 + 4 * (grp >> 1) + (j >> 2)) * TP + c0 + 16 * (grp & 1) + 4 * (j & 3);
  const bf16x4 lo = lds_read_tr(p), hi = lds_read_tr(p + 8 * TP);
  return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}
// token of accumulator element j for half-wave h inside a 32-token tile
__device__ __forceinline__ int tok(int j, int half) { return 8 * (j >> 2) + 4 * half + (j & 3); }

// Work item of a workgroup: (block of the list, head).  Workgroups go to the eight XCDs round-robin; with a multiple of
// eight heads every XCD takes its own heads and walks the list in order, so that the blocks running on an XCD at one
// time belong to two or three sequences of one head and find their keys and values in that XCD's L2.
__device__ __forceinline__ void work_item(int n_blocks, int n_heads, int& block, int& head) {
  const unsigned id = blockIdx.x;
  if ((n_heads & 7) == 0) {
    const unsigned j = id >> 3;
    head = (int)(id & 7) + 8 * (int)(j / (unsigned)n_blocks);
    block = (int)(j % (unsigned)n_blocks);
  } else {
    head = (int)(id / (unsigned)n_blocks);
    block = (int)(id % (unsigned)n_blocks);
  }
}

// ROWS rows x D columns of one head from global memory (rows past `limit` read as zero) into registers, then LDS.
// The tile is cut into 16-byte pieces, D / 8 a row.  Where the pieces of a row divide evenly among the 256 / ROWS
// threads that a row can have, a thread takes consecutive pieces of one row (one address, constant offsets);
// otherwise the 256 threads take the pieces of the tile in order, 256 at a time.
template <int ROWS, int D>
struct TileLoadT {
  static constexpr int PPR = D / 8, NP = ROWS * PPR, TPR = 256 / ROWS;
  static constexpr bool RUNS = PPR % TPR == 0;
  static constexpr int N = RUNS ? PPR / TPR : (NP + 255) / 256;
  uint4 r[N];
  __device__ __forceinline__ void load(const bf16_t* base, int64_t ld, int first, int row0, int limit, int hc, int tid) {
    if (RUNS) {
      const int row = row0 + tid / TPR;
      const uint4* src = (const uint4*)(base + (size_t)(first + row) * ld + hc + (tid % TPR) * (8 * N));
#pragma unroll
      for (int i = 0; i < N; ++i) r[i] = row < limit ? src[i] : uint4{0u, 0u, 0u, 0u};
    } else {
#pragma unroll
      for (int i = 0; i < N; ++i) {
        const int e = tid + 256 * i, row = row0 + e / PPR, pc = e % PPR;
        const bool ok = (NP % 256 == 0 || e < NP) && row < limit;
        r[i] = ok ? *(const uint4*)(base + (size_t)(first + row) * ld + hc + pc * 8) : uint4{0u, 0u, 0u, 0u};
      }
    }
  }
  __device__ __forceinline__ void store(bf16_t* tile, int pitch, int tid) const {
    if (RUNS) {
      uint4* dst = (uint4*)(tile + (tid / TPR) * pitch + (tid % TPR) * (8 * N));
#pragma unroll
      for (int i = 0; i < N; ++i) dst[i] = r[i];
    } else {
#pragma unroll
      for (int i = 0; i < N; ++i) {
        const int e = tid + 256 * i;
        if (NP % 256 == 0 || e < NP) *(uint4*)(tile + (e / PPR) * pitch + (e % PPR) * 8) = r[i];
      }
    }
  }
};
// Zero in the columns D .. DP-1 of a staged tile of `rows` rows (nothing is ever stored there afterwards).
template <int D, int DP>
__device__ __forceinline__ void zero_pad_columns(bf16_t* tile, int rows, int pitch, int tid) {
  if constexpr (DP > D) {
    constexpr int PIECES = (DP - D) / 8;       // 16-byte pieces a row
    for (int e = tid; e < rows * PIECES; e += 256)
      *(uint4*)(tile + (e / PIECES) * pitch + D + (e % PIECES) * 8) = uint4{0u, 0u, 0u, 0u};
  }
}

// ------------------------------------------------------------------------------------------------ forward
template <int D>
__global__ __launch_bounds__(256, 2) void k_attn_fwd(AttnParams p) {
  constexpr int KS = Dim<D>::KS, DT = Dim<D>::DT, DP = Dim<D>::DP, KP = Dim<D>::KP, TP = Dim<D>::TP;
  __shared__ __align__(16) bf16_t sK[TILE * KP];
  __shared__ __align__(16) bf16_t sV[TILE * TP];
  int wi_block, wi_head;
  work_item(p.dtab[DH_ATT_NBLK], p.H, wi_block, wi_head);
  const int32_t* blk = p.dtab + p.dtab[DH_ATT_OFF_FWD] + wi_block * DA_WORDS;
  const int first = blk[DA_FIRST_ROW], len = blk[DA_LEN], q0 = blk[DA_BLOCK0];
  const int hc = wi_head * D;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, li = lane & 31, half = lane >> 5;
  const int ql = q0 + 32 * wave + li;          // this lane's query inside the sequence
  const bool qok = ql < len;
  zero_pad_columns<D, DP>(sV, TILE, TP, tid);
  bf16x8 qf[KS];
  {
    const bf16_t* qrow = p.Q + (size_t)(first + ql) * p.ldq + hc + 8 * half;
#pragma unroll
    for (int s = 0; s < KS; ++s) qf[s] = qok ? *(const bf16x8*)(qrow + 16 * s) : zero8();
  }
  f32x16 o[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int j = 0; j < 16; ++j) o[dt][j] = 0.f;
  float m = -INFINITY, m_prev = -INFINITY, l = 0.f;
  const float c = p.scale * LOG2E;
  const float lazy = 8.f / c;                   // 8 in the exponent, in units of the raw score
  const int kend = min(len, q0 + BLK);          // keys [0, kend) are visible to some query of the block
  const int wq_first = q0 + 32 * wave, wq_last = wq_first + 31;
  TileLoadT<TILE, D> tk, tv;
  const int hck = wi_head / (p.H / p.Hkv) * D;  // this head's key/value columns
  tk.load(p.K, p.ldk, first, 0, len, hck, tid);
  tv.load(p.V, p.ldv, first, 0, len, hck, tid);
  for (int kb = 0; kb < kend; kb += TILE) {
    __syncthreads();
    tk.store(sK, KP, tid);
    tv.store(sV, TP, tid);
    __syncthreads();
    if (kb + TILE < kend) {
      tk.load(p.K, p.ldk, first, kb + TILE, len, hck, tid);
      tv.load(p.V, p.ldv, first, kb + TILE, len, hck, tid);
    }
    if (kb > wq_last) continue;                 // no key of this tile is visible to this wave's queries
    f32x16 s[2];
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int j = 0; j < 16; ++j) s[kt][j] = 0.f;
    {
      // the K fragments of the first 32 keys are fetched up front; each is refilled for the second 32 keys as
      // soon as its product is issued, so that an LDS read has the other products to land behind
      const bf16_t* kp = sK + li * KP + 8 * half;
      bf16x8 kf[KS];
#pragma unroll
      for (int st = 0; st < KS; ++st) kf[st] = *(const bf16x8*)(kp + 16 * st);
      __builtin_amdgcn_sched_barrier(0);        // (the scheduler would otherwise sink every read next to its use)
      ATTN_PRIO_HIGH();
#pragma unroll
      for (int st = 0; st < KS; ++st) {
        s[0] = mma(kf[st], qf[st], s[0]);
        kf[st] = *(const bf16x8*)(kp + 32 * KP + 16 * st);
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int st = 0; st < KS; ++st) s[1] = mma(kf[st], qf[st], s[1]);
      ATTN_PRIO_LOW();
    }
    const bool diag = kb + TILE - 1 > wq_first;
    // running maximum on the raw scores (the scale is positive), then one fused multiply-add per element: m is kept in
    // units of the raw score, exp2 arguments are s c - m c
    float mx = -INFINITY;
    if (diag) {                                 // only the tiles on the diagonal pay for the mask
      const int rel = ql - kb - 4 * half;       // key 32 kt + 8 (j / 4) + j % 4 is hidden iff it exceeds rel
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int j = 0; j < 16; ++j)
          if (32 * kt + 8 * (j >> 2) + (j & 3) > rel) s[kt][j] = -INFINITY;
    }
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int j = 0; j < 16; ++j) mx = fmaxf(mx, s[kt][j]);
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    // The reference point of the exponentials follows the running maximum lazily: it moves only when the maximum
    // has grown by more than 8 in the exponent (probabilities then stay below 2^8, harmless in fp32 and bf16, and
    // the final division by the row sum cancels the choice), so the rescaling of the output is rare.
    if (!(mx <= m + lazy)) m = mx;              // also the first tile (m = -inf) and never for mx = -inf
    const float ms = m == -INFINITY ? 0.f : m;
    const float alpha = fast_exp2((m_prev - ms) * c);
    m_prev = m;
    const float msc = ms * c;
    float rs = 0.f;
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        const float e = fast_exp2(fmaf(s[kt][j], c, -msc));
        s[kt][j] = e;
        rs += e;
      }
    l = l * alpha + rs;
    if (__any(alpha != 1.f)) {                  // the running maximum of some query moved
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int j = 0; j < 16; ++j) o[dt][j] *= alpha;
    }
    ATTN_PRIO_HIGH();
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const bf16x8 pb = pack8(s[kt], u);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) o[dt] = mma(read_across<TP>(sV, 32 * kt + 16 * u, 32 * dt, lane), pb, o[dt]);
      }
    ATTN_PRIO_LOW();
  }
  l += __shfl_xor(l, 32);
  if (qok) {
    const float inv = 1.f / l;
    bf16_t* orow = p.Out + (size_t)(first + ql) * p.ldo + hc;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int jg = 0; jg < 4; ++jg) {
        if (32 * dt + 8 * jg >= D) continue;      // the unused half of the last 32 columns
        uint2 v;
        v.x = pack_bf16x2(o[dt][4 * jg + 0] * inv, o[dt][4 * jg + 1] * inv);
        v.y = pack_bf16x2(o[dt][4 * jg + 2] * inv, o[dt][4 * jg + 3] * inv);
        *(uint2*)(orow + 32 * dt + 8 * jg + 4 * half) = v;
      }
    if (p.lse && half == 0) p.lse[(size_t)wi_head * p.T + first + ql] = (m * c + log2f(l)) * LN2;
  }
}

// Rows that belong to no sequence: zero in `n_out` outputs.  grid = (64-row items, slabs of 2048 elements).
struct ZeroParams {
  const int32_t* dtab;
  bf16_t* out[3];
  int64_t ld[3];
  int n_out;
  int width[3];
};
__global__ __launch_bounds__(256) void k_attn_zero_pad(ZeroParams p) {
  const ItemView it = load_item(p.dtab, 0, blockIdx.x);
  if (it.task >= 0 && it.nvalid == it.nrows) return;
  // wave w takes the rows w, w + 4, ..; the workgroup covers a slab of 256 vectors (4 KB) of the row width
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int slab = (int)blockIdx.y * 256 + lane;
  for (int r = wave; r < it.nrows; r += 4) {
    if (it.task >= 0 && row_is_valid(p.dtab, it.row0 + r)) continue;
    for (int o = 0; o < p.n_out; ++o) {
      uint4* dst = (uint4*)(p.out[o] + (size_t)(it.row0 + r) * p.ld[o]);
#pragma unroll
      for (int k = 0; k < 4; ++k)
        if (slab + 64 * k < p.width[o] / 8) dst[slab + 64 * k] = uint4{0u, 0u, 0u, 0u};
    }
  }
}

// delta[h][row] = sum_d dO[row][h, d] * O[row][h, d] for the rows of sequences.  Sixteen lanes per (row, head), a
// 16-byte piece each (a wave instruction then reads whole runs of the row); a group of sixteen takes four
// consecutive heads, all loads issued before the sums.
template <int D>
__global__ __launch_bounds__(256) void k_attn_delta(AttnParams p) {
  constexpr int PPR = D / 8, U = 4;
  const int l16 = threadIdx.x & 15;
  const size_t group = ((size_t)blockIdx.x * 256 + threadIdx.x) >> 4;
  const size_t n = (size_t)p.T * p.H;
  uint4 x[U], y[U];
  bool ok[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const size_t idx = group * U + u;
    const int row = idx < n ? (int)(idx / p.H) : 0, h = (int)(idx % p.H);
    ok[u] = idx < n && l16 < PPR && row_is_valid(p.dtab, row);
    x[u] = y[u] = uint4{0u, 0u, 0u, 0u};
    if (ok[u]) {
      x[u] = *(const uint4*)(p.dO + (size_t)row * p.ldo + h * D + 8 * l16);
      y[u] = *(const uint4*)(p.O + (size_t)row * p.ldo + h * D + 8 * l16);
    }
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const uint32_t xs[4] = {x[u].x, x[u].y, x[u].z, x[u].w}, ys[4] = {y[u].x, y[u].y, y[u].z, y[u].w};
    float s = 0.f;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      s = fmaf(__uint_as_float(xs[q] << 16), __uint_as_float(ys[q] << 16), s);
      s = fmaf(__uint_as_float(xs[q] & 0xffff0000u), __uint_as_float(ys[q] & 0xffff0000u), s);
    }
    s += __shfl_xor(s, 8);
    s += __shfl_xor(s, 4);
    s += __shfl_xor(s, 2);
    s += __shfl_xor(s, 1);
    const size_t idx = group * U + u;
    if (idx < n && l16 == 0) p.delta[(size_t)(idx % p.H) * p.T + idx / p.H] = s;
  }
}

// ------------------------------------------------------------------------------------------------ dQ
template <int D>
__global__ __launch_bounds__(256, 2) void k_attn_bwd_q(AttnParams p) {
  constexpr int KS = Dim<D>::KS, DT = Dim<D>::DT, DP = Dim<D>::DP, KP = Dim<D>::KP, TP = Dim<D>::TP;
  __shared__ __align__(16) bf16_t sK[TILE * TP];
  __shared__ __align__(16) bf16_t sV[TILE * KP];
  int wi_block, wi_head;
  work_item(p.dtab[DH_ATT_NBLK], p.H, wi_block, wi_head);
  const int32_t* blk = p.dtab + p.dtab[DH_ATT_OFF_FWD] + wi_block * DA_WORDS;
  const int first = blk[DA_FIRST_ROW], len = blk[DA_LEN], q0 = blk[DA_BLOCK0];
  const int hc = wi_head * D;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, li = lane & 31, half = lane >> 5;
  const int ql = q0 + 32 * wave + li;
  const bool qok = ql < len;
  zero_pad_columns<D, DP>(sK, TILE, TP, tid);
  bf16x8 qf[KS], df[KS];
  {
    const bf16_t* qrow = p.Q + (size_t)(first + ql) * p.ldq + hc + 8 * half;
    const bf16_t* drow = p.dO + (size_t)(first + ql) * p.ldo + hc + 8 * half;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      qf[s] = qok ? *(const bf16x8*)(qrow + 16 * s) : zero8();
      df[s] = qok ? *(const bf16x8*)(drow + 16 * s) : zero8();
    }
  }
  const float c = p.scale * LOG2E;
  const float lse2 = qok ? p.lse[(size_t)wi_head * p.T + first + ql] * LOG2E : INFINITY;    // exp2(x - inf) = 0
  const float dl = qok ? p.delta[(size_t)wi_head * p.T + first + ql] : 0.f;
  f32x16 dq[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int j = 0; j < 16; ++j) dq[dt][j] = 0.f;
  const int kend = min(len, q0 + BLK);
  const int wq_first = q0 + 32 * wave, wq_last = wq_first + 31;
  TileLoadT<TILE, D> tk, tv;
  const int hck = wi_head / (p.H / p.Hkv) * D;  // this head's key/value columns
  tk.load(p.K, p.ldk, first, 0, len, hck, tid);
  tv.load(p.V, p.ldv, first, 0, len, hck, tid);
  for (int kb = 0; kb < kend; kb += TILE) {
    __syncthreads();
    tk.store(sK, TP, tid);
    tv.store(sV, KP, tid);
    __syncthreads();
    if (kb + TILE < kend) {
      tk.load(p.K, p.ldk, first, kb + TILE, len, hck, tid);
      tv.load(p.V, p.ldv, first, kb + TILE, len, hck, tid);
    }
    if (kb > wq_last) continue;
    const bool diag = kb + TILE - 1 > wq_first;
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {            // one half of the tile at a time keeps the live registers down
      f32x16 s, dp;
#pragma unroll
      for (int j = 0; j < 16; ++j) { s[j] = 0.f; dp[j] = 0.f; }
      ATTN_PRIO_HIGH();
#pragma unroll
      for (int st = 0; st < KS; ++st) {
        s = mma(*(const bf16x8*)(sK + (32 * kt + li) * TP + 16 * st + 8 * half), qf[st], s);
        dp = mma(*(const bf16x8*)(sV + (32 * kt + li) * KP + 16 * st + 8 * half), df[st], dp);
      }
      ATTN_PRIO_LOW();
#pragma unroll
      for (int j = 0; j < 16; ++j) s[j] = fast_exp2(fmaf(s[j], c, -lse2));        // P^T (zero for a lane without query)
      if (diag) {                               // only the tiles on the diagonal pay for the mask
        const int rel = ql - kb - 32 * kt - 4 * half;
#pragma unroll
        for (int j = 0; j < 16; ++j)
          if (8 * (j >> 2) + (j & 3) > rel) s[j] = 0.f;
      }
#pragma unroll
      for (int j = 0; j < 16; ++j) s[j] *= dp[j] - dl;                           // dS^T
      ATTN_PRIO_HIGH();
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const bf16x8 ds = pack8(s, u);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) dq[dt] = mma(read_across<TP>(sK, 32 * kt + 16 * u, 32 * dt, lane), ds, dq[dt]);
      }
      ATTN_PRIO_LOW();
    }
  }
  if (qok) {
    bf16_t* orow = p.dQ + (size_t)(first + ql) * p.ldq + hc;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int jg = 0; jg < 4; ++jg) {
        if (32 * dt + 8 * jg >= D) continue;      // the unused half of the last 32 columns
        uint2 v;
        v.x = pack_bf16x2(dq[dt][4 * jg + 0] * p.scale, dq[dt][4 * jg + 1] * p.scale);
        v.y = pack_bf16x2(dq[dt][4 * jg + 2] * p.scale, dq[dt][4 * jg + 3] * p.scale);
        *(uint2*)(orow + 32 * dt + 8 * jg + 4 * half) = v;
      }
  }
}

// ------------------------------------------------------------------------------------------------ dK, dV
template <int D>
__global__ __launch_bounds__(256, 2) void k_attn_bwd_kv(AttnParams p) {
  constexpr int KS = Dim<D>::KS, DT = Dim<D>::DT, DP = Dim<D>::DP, KP = Dim<D>::KP, TP = Dim<D>::TP;
  constexpr int QT = 32;                       // queries staged per step
  __shared__ __align__(16) bf16_t sQ[QT * TP];
  __shared__ __align__(16) bf16_t sD[QT * TP];
  __shared__ __align__(16) bf16_t sVf[BLK * KP];   // the block's own V rows (B operand of dO V^T), kept here to save registers
  __shared__ float sLse[QT], sDelta[QT];
  int wi_block, wi_head;                       // wi_head: a key/value head
  work_item(p.dtab[DH_ATT_NBLK], p.Hkv, wi_block, wi_head);
  const int32_t* blk = p.dtab + p.dtab[DH_ATT_OFF_BWD] + wi_block * DA_WORDS;
  const int first = blk[DA_FIRST_ROW], len = blk[DA_LEN], k0 = blk[DA_BLOCK0];
  const int hc = wi_head * D;
  const int group = p.H / p.Hkv;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, li = lane & 31, half = lane >> 5;
  const int kl = k0 + 32 * wave + li;          // this lane's key inside the sequence
  const bool kok = kl < len;
  zero_pad_columns<D, DP>(sQ, QT, TP, tid);
  zero_pad_columns<D, DP>(sD, QT, TP, tid);
  bf16x8 kf[KS];
  {
    const bf16_t* krow = p.K + (size_t)(first + kl) * p.ldk + hc + 8 * half;
#pragma unroll
    for (int s = 0; s < KS; ++s) kf[s] = kok ? *(const bf16x8*)(krow + 16 * s) : zero8();
    TileLoadT<TILE, D> t;
    t.load(p.V, p.ldv, first, k0, len, hc, tid);
    t.store(sVf, KP, tid);
    t.load(p.V, p.ldv, first, k0 + TILE, len, hc, tid);
    t.store(sVf + TILE * KP, KP, tid);
  }
  const bf16_t* vfrag = sVf + (32 * wave + li) * KP + 8 * half;
  const float c = p.scale * LOG2E;
  f32x16 dk[DT], dv[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int j = 0; j < 16; ++j) { dk[dt][j] = 0.f; dv[dt][j] = 0.f; }
  const int wk_first = k0 + 32 * wave;
  TileLoadT<QT, D> tq, td;
  float r_lse = 0.f, r_delta = 0.f;
  for (int g = 0; g < group; ++g) {             // every query head that reads this key/value head
  const int hq = wi_head * group + g, hcq = hq * D;
  auto load_stats = [&](int qb) {
    if (tid < QT) {
      const bool ok = qb + tid < len;
      r_lse = ok ? p.lse[(size_t)hq * p.T + first + qb + tid] * LOG2E : INFINITY;   // exp2(x - inf) = 0
      r_delta = ok ? p.delta[(size_t)hq * p.T + first + qb + tid] : 0.f;
    }
  };
  tq.load(p.Q, p.ldq, first, k0, len, hcq, tid);
  td.load(p.dO, p.ldo, first, k0, len, hcq, tid);
  load_stats(k0);
  for (int qb = k0; qb < len; qb += QT) {       // queries before the block see none of its keys
    __syncthreads();
    tq.store(sQ, TP, tid);
    td.store(sD, TP, tid);
    if (tid < QT) { sLse[tid] = r_lse; sDelta[tid] = r_delta; }
    __syncthreads();
    if (qb + QT < len) {
      tq.load(p.Q, p.ldq, first, qb + QT, len, hcq, tid);
      td.load(p.dO, p.ldo, first, qb + QT, len, hcq, tid);
      load_stats(qb + QT);
    }
    if (qb + QT - 1 < wk_first) continue;     // every query of the tile lies before this wave's keys
    const bool diag = qb < wk_first + 32;        // some query of the tile lies before some key of the wave
    {
      constexpr int qt = 0;
      f32x16 s, dp;
#pragma unroll
      for (int j = 0; j < 16; ++j) { s[j] = 0.f; dp[j] = 0.f; }
#pragma unroll
      for (int st = 0; st < KS; ++st) {
        s = mma(*(const bf16x8*)(sQ + (32 * qt + li) * TP + 16 * st + 8 * half), kf[st], s);
        dp = mma(*(const bf16x8*)(sD + (32 * qt + li) * TP + 16 * st + 8 * half), *(const bf16x8*)(vfrag + 16 * st), dp);
        if (st % 2 == 1) __builtin_amdgcn_sched_barrier(0);
      }
      // P (a lane without key computes on zeros and is not stored)
#pragma unroll
      for (int j = 0; j < 16; ++j) s[j] = fast_exp2(fmaf(s[j], c, -sLse[32 * qt + tok(j, half)]));
      if (diag) {                               // only the tiles on the diagonal pay for the mask
        const int rel = kl - qb - 32 * qt - 4 * half;      // query 8 (j / 4) + j % 4 sees the key iff it is >= rel
#pragma unroll
        for (int j = 0; j < 16; ++j)
          if (8 * (j >> 2) + (j & 3) < rel) s[j] = 0.f;
      }
#pragma unroll
      for (int j = 0; j < 16; ++j) dp[j] = s[j] * (dp[j] - sDelta[32 * qt + tok(j, half)]);   // dS
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const bf16x8 pb = pack8(s, u), ds = pack8(dp, u);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          dv[dt] = mma(read_across<TP>(sD, 32 * qt + 16 * u, 32 * dt, lane), pb, dv[dt]);
          dk[dt] = mma(read_across<TP>(sQ, 32 * qt + 16 * u, 32 * dt, lane), ds, dk[dt]);
        }
        __builtin_amdgcn_sched_barrier(0);      // keeps the operand reads of the next group from piling up in registers
      }
    }
  }
  }                                             // next query head of the group
  if (kok) {
    bf16_t* krow = p.dK + (size_t)(first + kl) * p.ldk + hc;
    bf16_t* vrow = p.dV + (size_t)(first + kl) * p.ldv + hc;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int jg = 0; jg < 4; ++jg) {
        if (32 * dt + 8 * jg >= D) continue;      // the unused half of the last 32 columns
        uint2 a, b;
        a.x = pack_bf16x2(dk[dt][4 * jg + 0] * p.scale, dk[dt][4 * jg + 1] * p.scale);
        a.y = pack_bf16x2(dk[dt][4 * jg + 2] * p.scale, dk[dt][4 * jg + 3] * p.scale);
        b.x = pack_bf16x2(dv[dt][4 * jg + 0], dv[dt][4 * jg + 1]);
        b.y = pack_bf16x2(dv[dt][4 * jg + 2], dv[dt][4 * jg + 3]);
        *(uint2*)(krow + 32 * dt + 8 * jg + 4 * half) = a;
        *(uint2*)(vrow + 32 * dt + 8 * jg + 4 * half) = b;
      }
  }
}

mux_status check(const char* fn, const mux_attn_desc* d, const mux_segtab* st) {
  if (!d || !st) return fail(MUX_ERR_INVALID_ARG, std::string(fn) + ": null descriptor or table");
  if (d->n_heads < 1 || d->n_kv_heads < 1 || d->head_dim < 1) return fail(MUX_ERR_INVALID_ARG, std::string(fn) + ": bad head counts");
  if (d->n_heads % d->n_kv_heads) return fail(MUX_ERR_INVALID_ARG, std::string(fn) + ": n_kv_heads must divide n_heads");
  const int D = d->head_dim;
  if (d->dtype != MUX_DT_BF16 || (D != 64 && D != 80 && D != 96 && D != 128))
    return fail(MUX_ERR_UNSUPPORTED, std::string(fn) + ": only bf16 and head_dim 64, 80, 96 and 128 are built");
  const int64_t w = (int64_t)d->n_heads * D, wkv = (int64_t)d->n_kv_heads * D;
  const int64_t lds[4] = {d->ldq, d->ldk, d->ldv, d->ldo};
  for (int i = 0; i < 4; ++i) {
    const int64_t ld = lds[i];
    if (ld < (i == 1 || i == 2 ? wkv : w)) return fail(MUX_ERR_SHAPE, std::string(fn) + ": a leading dimension is smaller than its heads * head_dim");
    if (ld % 8) return fail(MUX_ERR_UNSUPPORTED, std::string(fn) + ": leading dimensions must be multiples of 8");
    if ((int64_t)st->T * ld >= ((int64_t)1 << 40)) return fail(MUX_ERR_SHAPE, std::string(fn) + ": problem too large");
  }
  if ((int64_t)st->n_attn_blocks * d->n_heads >= ((int64_t)1 << 31)) return fail(MUX_ERR_SHAPE, std::string(fn) + ": too many work items");
  if (!(d->scale >= 0.f)) return fail(MUX_ERR_INVALID_ARG, std::string(fn) + ": negative scale");
  return MUX_OK;
}

bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

// One launch of kernel template K<D> for the head dimension of the call.
#define ATTN_LAUNCH(name, K, D, grid, stream, p)                                           \
  do {                                                                                     \
    if ((D) == 128) MUX_LAUNCH(name, K<128>, grid, dim3(256), 0, stream, p);               \
    else if ((D) == 96) MUX_LAUNCH(name, K<96>, grid, dim3(256), 0, stream, p);            \
    else if ((D) == 80) MUX_LAUNCH(name, K<80>, grid, dim3(256), 0, stream, p);            \
    else MUX_LAUNCH(name, K<64>, grid, dim3(256), 0, stream, p);                           \
  } while (0)

mux_status last_hip(const char* fn) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(MUX_ERR_DEVICE, std::string(fn) + ": " + hipGetErrorString(e));
  return MUX_OK;
}

}  // namespace
}  // namespace mux

using namespace mux;

extern "C" size_t mux_attn_saved_bytes(const mux_attn_desc* desc, const mux_segtab* st) {
  if (!desc || !st || desc->n_heads < 1) return 0;
  return align256((size_t)st->T * (size_t)desc->n_heads * sizeof(float));
}

extern "C" size_t mux_attn_workspace_bytes(const mux_attn_desc* desc, const mux_segtab* st) {
  return mux_attn_saved_bytes(desc, st);
}

extern "C" mux_status mux_attn_forward(const mux_attn_desc* desc, const mux_segtab* st, const void* dev_segtab,
                                       const void* Q, const void* K, const void* V, void* O, void* saved,
                                       void* hip_stream) {
  static const char* fn = "mux_attn_forward";
  if (mux_status s = check(fn, desc, st)) return s;
  if (st->T == 0) return MUX_OK;
  if (!dev_segtab || !Q || !K || !V || !O) return fail(MUX_ERR_INVALID_ARG, std::string(fn) + ": null device pointer");
  if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O))
    return fail(MUX_ERR_UNSUPPORTED, std::string(fn) + ": pointers must be 16-byte aligned");
  hipStream_t stream = (hipStream_t)hip_stream;
  const int D = desc->head_dim;
  AttnParams p{};
  p.dtab = (const int32_t*)dev_segtab;
  p.Q = (const bf16_t*)Q; p.K = (const bf16_t*)K; p.V = (const bf16_t*)V; p.Out = (bf16_t*)O;
  p.lse = (float*)saved;
  p.ldq = desc->ldq; p.ldk = desc->ldk; p.ldv = desc->ldv; p.ldo = desc->ldo;
  p.T = st->T; p.H = desc->n_heads; p.Hkv = desc->n_kv_heads;
  p.scale = desc->scale > 0.f ? desc->scale : 1.f / sqrtf((float)D);
  ZeroParams z{};
  z.dtab = p.dtab; z.out[0] = (bf16_t*)O; z.ld[0] = desc->ldo; z.n_out = 1; z.width[0] = desc->n_heads * D;
  MUX_LAUNCH("attn_zero_pad", k_attn_zero_pad, dim3((unsigned)st->items[0].size(), (unsigned)((z.width[0] + 2047) / 2048)), dim3(256), 0, stream, z);
  if (st->n_attn_blocks > 0)
    ATTN_LAUNCH("attn_fwd", k_attn_fwd, D, dim3((unsigned)st->n_attn_blocks * (unsigned)desc->n_heads), stream, p);
  return last_hip(fn);
}

extern "C" mux_status mux_attn_backward(const mux_attn_desc* desc, const mux_segtab* st, const void* dev_segtab,
                                        const void* Q, const void* K, const void* V, const void* O, const void* dO,
                                        const void* saved, void* dQ, void* dK, void* dV, void* ws, size_t ws_bytes,
                                        void* hip_stream) {
  static const char* fn = "mux_attn_backward";
  if (mux_status s = check(fn, desc, st)) return s;
  if (st->T == 0) return MUX_OK;
  if (!dev_segtab || !Q || !K || !V || !O || !dO || !saved || !dQ || !dK || !dV || !ws)
    return fail(MUX_ERR_INVALID_ARG, std::string(fn) + ": null device pointer");
  const void* ptrs[8] = {Q, K, V, O, dO, dQ, dK, dV};
  for (const void* q : ptrs)
    if (!aligned16(q)) return fail(MUX_ERR_UNSUPPORTED, std::string(fn) + ": pointers must be 16-byte aligned");
  if (ws_bytes < mux_attn_workspace_bytes(desc, st)) return fail(MUX_ERR_WORKSPACE, std::string(fn) + ": workspace too small");
  hipStream_t stream = (hipStream_t)hip_stream;
  const int D = desc->head_dim;
  AttnParams p{};
  p.dtab = (const int32_t*)dev_segtab;
  p.Q = (const bf16_t*)Q; p.K = (const bf16_t*)K; p.V = (const bf16_t*)V; p.O = (const bf16_t*)O; p.dO = (const bf16_t*)dO;
  p.dQ = (bf16_t*)dQ; p.dK = (bf16_t*)dK; p.dV = (bf16_t*)dV;
  p.lse = (float*)saved; p.delta = (float*)ws;
  p.ldq = desc->ldq; p.ldk = desc->ldk; p.ldv = desc->ldv; p.ldo = desc->ldo;
  p.T = st->T; p.H = desc->n_heads; p.Hkv = desc->n_kv_heads;
  p.scale = desc->scale > 0.f ? desc->scale : 1.f / sqrtf((float)D);
  ZeroParams z{};
  z.dtab = p.dtab; z.n_out = 3;
  z.width[0] = desc->n_heads * D; z.width[1] = z.width[2] = desc->n_kv_heads * D;
  z.out[0] = p.dQ; z.ld[0] = desc->ldq; z.out[1] = p.dK; z.ld[1] = desc->ldk; z.out[2] = p.dV; z.ld[2] = desc->ldv;
  MUX_LAUNCH("attn_zero_pad", k_attn_zero_pad, dim3((unsigned)st->items[0].size(), (unsigned)((z.width[0] + 2047) / 2048)), dim3(256), 0, stream, z);
  const size_t n = (size_t)st->T * desc->n_heads;
  ATTN_LAUNCH("attn_delta", k_attn_delta, D, dim3((unsigned)(((n + 3) / 4 * 16 + 255) / 256)), stream, p);
  if (st->n_attn_blocks > 0) {
    ATTN_LAUNCH("attn_bwd_kv", k_attn_bwd_kv, D, dim3((unsigned)st->n_attn_blocks * (unsigned)desc->n_kv_heads), stream, p);
    ATTN_LAUNCH("attn_bwd_q", k_attn_bwd_q, D, dim3((unsigned)st->n_attn_blocks * (unsigned)desc->n_heads), stream, p);
  }
  return last_hip(fn);
}
