/*
 * mux.h -- C ABI of the multiplexed multi-task PEFT linear layer for AMD MI355X (gfx950).
 *
 * One frozen backbone weight W is shared by several independent fine-tuning tasks
 * (paper section 3.2).  Their token batches are chunk-aligned and concatenated along the
 * token dimension (section 3.5), pushed through ONE backbone GEMM (Eq. 1), and every task's
 * adapter is applied to that task's rows only (sections 3.2, 3.4.3).  The backward pass
 * returns the input gradient (Eq. 2) and per-task adapter gradients; a gradient of W is
 * never formed (sections 1 and 2.2).
 *
 * Conventions
 *   - Plain C, no exceptions.  Every function returns a mux_status (or a size/count);
 *     mux_last_error() gives a thread-local text for the last non-OK status.
 *   - "host" pointers are ordinary CPU memory, "device" pointers are HIP device memory of the
 *     current device.  The caller owns every device buffer, including workspace, saved
 *     activations and the uploaded table; the library allocates only the host-side mux_segtab.
 *   - All GPU work is enqueued on the given hipStream_t (passed as void*); no call
 *     synchronises.  Argument checks happen on the host before anything is launched; a call
 *     that returns an error has launched nothing.
 *   - Same inputs give bit-identical outputs (no floating-point atomics anywhere).
 *   - Tensors are row-major and dense unless a leading dimension is given.
 *     X[T,K], W[K,N] (Y = X W, the orientation of Eq. 1), Y[T,N], dY[T,N], dX[T,K],
 *     A_t[K,r_t], B_t[r_t,N], l_t[N].  T = mux_segtab_rows().
 *   - Diagnostics (per-kernel timing, probes of the box, measurement switches) are declared in mux_diag.h; none
 *     of them is needed in normal use.
 */
#ifndef MUX_H_
#define MUX_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MUX_OK = 0,
  MUX_ERR_INVALID_ARG = 1, /* null pointer, non-positive size, bad enum, bad flag          */
  MUX_ERR_SHAPE = 2,       /* sizes inconsistent with the table or with each other          */
  MUX_ERR_UNSUPPORTED = 3, /* valid request the library does not implement                   */
  MUX_ERR_WORKSPACE = 4,   /* workspace / destination buffer too small                       */
  MUX_ERR_HOST_NOMEM = 5,  /* host allocation failed                                         */
  MUX_ERR_DEVICE = 6       /* a HIP runtime call failed (text in mux_last_error)             */
} mux_status;

/* Adapter kinds.  LORA: y = x W + s (x A) B (sections 2.1, 2.2; aggregate = add, 3.4.3).
 * IA3_OUT: y = (x W) * l, a per-task elementwise output scale (aggregate = multiply).
 * TUNING: the additive type of section 2.1 (Adapter-Tuning, one of the three implemented types of
 * section 5), a bottleneck inserted after the BaseOp: z = x W, y = z + s gelu(z D) U with D [N, r],
 * U [r, N] and gelu(u) = u/2 (1 + erf(u / sqrt 2)).  D is passed in the A slot, U in the B slot.
 * DIFF: the selective type of section 2.1 (Diff-Pruning, also among the implemented types of section 5):
 * y = x (W + M * delta) with a fixed 0/1 mask M over the entries of W and trainable values delta on the
 * masked entries only.  The values are passed in the A slot (one per masked entry, in the row-major order
 * of the mask), the mask itself as a mux_sparse_mask in mux_layer_desc.masks.
 * NONE: y = x W. */
typedef enum {
  MUX_ADAPTER_NONE = 0,
  MUX_ADAPTER_LORA = 1,
  MUX_ADAPTER_IA3_OUT = 2,
  MUX_ADAPTER_TUNING = 3,
  MUX_ADAPTER_DIFF = 4
} mux_adapter_kind;

/* Storage type of activations, weights and adapters.  BF16: bfloat16 storage, fp32
 * accumulation on the matrix cores.  F32: fp32 storage and arithmetic (a correctness mode).
 * Adapter gradients are fp32 in both modes. */
typedef enum { MUX_DT_BF16 = 0, MUX_DT_F32 = 1 } mux_dtype;

#define MUX_MAX_RANK 64
#define MUX_MAX_TASKS 1024

/* One fine-tuning task: its adapter type and the sequence lengths of its batch (host). */
typedef struct {
  int32_t kind;            /* mux_adapter_kind                                              */
  int32_t rank;            /* LORA, TUNING: 1..MUX_MAX_RANK; ignored otherwise              */
  float scale;             /* LORA, TUNING: s_t; ignored otherwise                          */
  int32_t n_seqs;          /* may be 0 (a task with no tokens has no rows, zero gradients)  */
  const int32_t* seq_lens; /* host, n_seqs entries, each >= 1                               */
} mux_task_desc;

typedef struct mux_segtab mux_segtab; /* host object, opaque */

/* mux_segtab_build flags */
#define MUX_SEGTAB_DENSE 1u /* tasks back to back, only the tail of the batch padded         */

/* Chunk-size rule of section 3.5: the greatest power of two dividing every length, not
 * below `floor_` (the paper's typical floor is 64).  lens: host, n entries.  Lengths <= 0
 * are ignored; with no length left the result is floor_. */
mux_status mux_choose_chunk_size(const int32_t* lens, int32_t n, int32_t floor_, int32_t* out);

/* Chunk-based alignment (section 3.5).  Step 1 packs each task's sequences in order inside
 * that task's own batch (max_pack_len = 0: one pack per task; > 0: a pack is closed when the
 * next sequence would make it longer; a longer sequence is a pack by itself).  Step 2 cuts
 * every pack into chunks of `chunk` rows, consecutive for a long pack; the last chunk of a
 * pack is zero padded.  Tasks keep the caller's order.  chunk must be a power of two.
 * With MUX_SEGTAB_DENSE packs are laid back to back instead and a chunk may hold rows of
 * two tasks.  *out is allocated by the library; release with mux_segtab_free. */
mux_status mux_segtab_build(const mux_task_desc* tasks, int32_t n_tasks, int32_t chunk,
                            int32_t max_pack_len, uint32_t flags, mux_segtab** out);
void mux_segtab_free(mux_segtab* st);

int32_t mux_segtab_rows(const mux_segtab* st);         /* T = n_chunks * chunk              */
int32_t mux_segtab_n_chunks(const mux_segtab* st);
int32_t mux_segtab_n_tasks(const mux_segtab* st);
int32_t mux_segtab_valid_tokens(const mux_segtab* st); /* rows that are real tokens         */

/* Canonical little-endian int32 image (what "bit-exact table" means):
 *   header[16] = magic 'MUXT', version, flags, n_tasks, chunk, max_pack_len, n_chunks, T,
 *                valid_total, n_packs, n_segments, n_seqs, 0, 0, 0, 0
 *   per task    [row_begin, row_count, valid_tokens, chunk_begin, chunk_count,
 *                pack_begin, pack_count, seq_begin]
 *   per pack    [task, row_begin, valid_tokens, chunk_begin, chunk_count, seg_begin]
 *   per chunk   [valid_rows, seg_begin, seg_count, first_task]
 *   per segment [task, pack, chunk, row_begin, n_rows, index_in_pack]
 *               (segment = the rows of one pack inside one chunk, in row order)
 *   per sequence[task, pack, first_row, len]
 * Row i is a real token iff (i mod chunk) < valid_rows[i div chunk]. */
size_t mux_segtab_serialized_bytes(const mux_segtab* st);
mux_status mux_segtab_serialize(const mux_segtab* st, void* host_dst, size_t cap);
/* row -> task map: host_dst[i] = task of row i, or -1 for a padding row (T entries). */
mux_status mux_segtab_row_task(const mux_segtab* st, int32_t* host_dst, size_t cap_entries);

/* Device image of the table (tile work lists derived from it; layout private to the
 * library version).  Upload once per table; the copy is enqueued on `hip_stream` from
 * memory owned by `st`, so `st` must outlive the copy. */
size_t mux_segtab_device_bytes(const mux_segtab* st);
mux_status mux_segtab_upload(const mux_segtab* st, void* dev_dst, size_t cap, void* hip_stream);

/* Fixed sparse mask of one DIFF task over W[K,N] (host struct, device arrays of int32).  The masked entries
 * are numbered in row-major order (by k, then n, no duplicates): entry e of row k has column col_idx[e],
 * row_ptr[k] <= e < row_ptr[k+1].  The same entries are listed a second time column by column:
 * col_ent[2*i] = row k and col_ent[2*i+1] = number e of the i-th listed entry, col_ptr[n] <= i < col_ptr[n+1],
 * k ascending inside a column.  The mask is fixed during training, so both listings are built once.
 * Optional (all four or none; NULL: the library takes another route for this task's rows): the entries once more by
 * tiles, for the backbone products that add them to their tiles of W on the way.  Forward: bucket (k / 64, n / 128)
 * has number (k / 64) * ceil(N / 128) + n / 128 and holds the entries i with fwd_ptr[b] <= i < fwd_ptr[b+1],
 * fwd_ent[2*i] = number e, fwd_ent[2*i+1] = (k % 64) << 7 | (n % 128).  Backward: bucket (n / 64, k / 128) has number
 * (n / 64) * ceil(K / 128) + k / 128, bwd_ent[2*i] = e, bwd_ent[2*i+1] = (n % 64) << 7 | (k % 128). */
typedef struct mux_sparse_mask {
  int32_t nnz;
  const int32_t* row_ptr;  /* device, K+1 */
  const int32_t* col_idx;  /* device, nnz */
  const int32_t* col_ptr;  /* device, N+1 */
  const int32_t* col_ent;  /* device, 2*nnz */
  const int32_t* fwd_ptr;  /* device, ceil(K/64)*ceil(N/128)+1, or NULL */
  const int32_t* fwd_ent;  /* device, 2*nnz */
  const int32_t* bwd_ptr;  /* device, ceil(N/64)*ceil(K/128)+1, or NULL */
  const int32_t* bwd_ent;  /* device, 2*nnz */
} mux_sparse_mask;

/* Lays out both listings of a mask on the host from its entries (k[e], n[e]), e = 0 .. nnz-1, which must be sorted
 * by (k, n) without duplicates and lie inside W[K,N]: row_ptr [K+1], col_idx [nnz], col_ptr [N+1], col_ent [2 nnz], all
 * host arrays of the caller, who copies them to the device and points a mux_sparse_mask at the copies.  Index work
 * only; nothing is launched. */
mux_status mux_sparse_mask_layout(const int32_t* k, const int32_t* n, int32_t nnz, int32_t K, int32_t N,
                                  int32_t* row_ptr, int32_t* col_idx, int32_t* col_ptr, int32_t* col_ent);

/* The listing by tiles of the same entries (same preconditions): fwd_ptr [ceil(K/64)*ceil(N/128)+1], fwd_ent [2 nnz],
 * bwd_ptr [ceil(N/64)*ceil(K/128)+1], bwd_ent [2 nnz], host arrays of the caller.  Inside a bucket the entries keep
 * their (k, n) order.  Index work only; nothing is launched. */
mux_status mux_sparse_mask_tile_layout(const int32_t* k, const int32_t* n, int32_t nnz, int32_t K, int32_t N,
                                       int32_t* fwd_ptr, int32_t* fwd_ent, int32_t* bwd_ptr, int32_t* bwd_ent);

/* One multiplexed layer call.  All pointers inside are device pointers, except the three
 * arrays A, B, L themselves, which are host arrays of n_tasks device pointers (entry NULL
 * where the task's kind does not use it).  Ranks, scales and kinds come from the table. */
typedef struct {
  int32_t K, N;          /* in / out features                                               */
  int32_t dtype;         /* mux_dtype                                                       */
  uint32_t flags;        /* MUX_LAYER_* below                                               */
  const void* W;         /* device, [K, ldw] row-major, frozen                              */
  int64_t ldw;           /* elements between rows of W, >= N                                */
  int32_t n_tasks;       /* must equal the table's                                          */
  const void* const* A;  /* host array of device pointers, LORA: A_t[K, r_t]; TUNING: D_t[N, r_t] */
  const void* const* B;  /* LORA: B_t[r_t, N]; TUNING: U_t[r_t, N]                          */
  const void* const* L;  /* IA3_OUT: l_t[N]                                                 */
  const struct mux_sparse_mask* const* masks; /* host array of n_tasks host pointers, DIFF: the task's mask
                            (NULL entries for the other kinds; the array may be NULL without DIFF tasks)   */
} mux_layer_desc;

#define MUX_LAYER_REFERENCE_KERNELS 1u /* run the plain (non matrix-core) HIP kernels       */

/* Bytes of `saved` (forward -> backward: scaled adapter activations s_t (x A_t); x W of the
 * IA3_OUT and TUNING rows; the pre-activations z D_t of the TUNING rows) and of `ws` (scratch,
 * contents undefined between calls).  Both follow from the layer description and the table alone
 * (for DIFF tasks also from what their masks bring: with the listing by tiles the call packs the
 * entries, 4 bytes each; without it, it may hold a copy of W per such task). */
size_t mux_lora_saved_bytes(const mux_layer_desc* layer, const mux_segtab* st);
size_t mux_lora_workspace_bytes(const mux_layer_desc* layer, const mux_segtab* st);

/* Forward (Eq. 1 + adapters + aggregate):  for row i of task t
 *     Y_i = x_i W + s_t (x_i A_t) B_t      (LORA)
 *     Y_i = (x_i W) * l_t                  (IA3_OUT)
 *     Y_i = z_i + s_t gelu(z_i D_t) U_t ,  z_i = x_i W        (TUNING)
 *     Y_i = x_i (W + M_t * delta_t)        (DIFF)
 *     Y_i = x_i W                          (NONE)
 * Padding rows: their X content is ignored (never multiplied) and Y_i = 0.
 * X: device [T,K]; Y: device [T,N]; saved: device, mux_lora_saved_bytes, may be NULL only if
 * no backward follows and no task is LORA; ws: device, >= mux_lora_workspace_bytes. */
mux_status mux_lora_forward(const mux_layer_desc* layer, const mux_segtab* st,
                            const void* dev_segtab, const void* X, void* Y, void* saved,
                            void* ws, size_t ws_bytes, void* hip_stream);

/* Backward (Eq. 2 + adapter gradients), g_i = dY_i (zero on padding rows):
 *     dX_i = g_i W^T + s_t (g_i B_t^T) A_t^T ,  dA_t = s_t sum_i x_i^T (g_i B_t^T) ,
 *     dB_t = s_t sum_i (x_i A_t)^T g_i                                        (LORA)
 *     dX_i = (g_i * l_t) W^T ,  dl_t = sum_i g_i * (x_i W)                    (IA3_OUT)
 *     p_i = s_t (g_i U_t^T) * gelu'(z_i D_t) ,  dX_i = (g_i + p_i D_t^T) W^T ,
 *     dD_t = sum_i z_i^T p_i  (returned in dA[t], [N,r_t]) ,
 *     dU_t = s_t sum_i gelu(z_i D_t)^T g_i  (returned in dB[t], [r_t,N])      (TUNING)
 *     dX_i = g_i (W + M_t * delta_t)^T ,  d delta_t[e] = sum_i x_i[k_e] g_i[n_e]  (returned in dA[t], [nnz],
 *     the masked entries of x^T g: the one place where entries of a weight gradient are formed)   (DIFF)
 *     dX_i = g_i W^T                                                          (NONE)
 * sums over the rows of task t only.  dX of padding rows = 0.  No gradient of W.
 * dA, dB, dL: host arrays of n_tasks device pointers to fp32 buffers ([K,r_t], [r_t,N], [N]);
 * an entry may be NULL to skip that gradient.  accumulate = 0 overwrites, 1 adds to what the
 * buffers hold (micro-batch accumulation).  dX may be NULL to skip the input gradient.
 * `saved` must be the buffer the matching forward filled with the same layer and table. */
mux_status mux_lora_backward(const mux_layer_desc* layer, const mux_segtab* st,
                             const void* dev_segtab, const void* X, const void* dY,
                             const void* saved, void* dX, void* const* dA, void* const* dB,
                             void* const* dL, int accumulate, void* ws, size_t ws_bytes,
                             void* hip_stream);

/* mux_lora_backward for callers that cannot allocate device memory or hand over a workspace: code running under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and results (bit for bit)
 * as mux_lora_backward without `ws` / `ws_bytes`: the workspace is a device array of MUX_STATIC_WS_BYTES bytes inside
 * the library, one copy per GPU, held from the loading of the library until the process ends.  The call allocates
 * nothing and frees nothing; its first call on a device looks the array's address up once (make that call outside a
 * capture).  A call whose mux_lora_workspace_bytes() exceeds MUX_STATIC_WS_BYTES returns MUX_ERR_WORKSPACE and
 * launches nothing.  All calls on one GPU share that GPU's array: the array keeps the last call's contents (every
 * call writes what it reads, nothing has to start at zero), and two such calls that overlap in time on one GPU (two
 * streams, two threads) race on it; order them on one stream or with events. */
#define MUX_STATIC_WS_BYTES ((size_t)32 << 20)
mux_status mux_lora_backward_static_ws(const mux_layer_desc* layer, const mux_segtab* st,
                                       const void* dev_segtab, const void* X, const void* dY,
                                       const void* saved, void* dX, void* const* dA, void* const* dB,
                                       void* const* dL, int accumulate, void* hip_stream);

const char* mux_last_error(void);
const char* mux_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MUX_H_ */
