// Internal declarations shared by the host code and the kernels of the library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string>
#include <vector>

#include "mux.h"
#include "mux_diag.h"

namespace mux {

// ---- device image of the segment table (int32 words) ------------------------------------
// hdr[32] followed by the sections whose word offsets the header gives.
enum : int {
  DH_MAGIC = 0, DH_T, DH_CHUNK, DH_LOG2C, DH_NTASKS, DH_NCHUNKS, DH_OFF_TASKS, DH_OFF_CHUNK_VALID,
  DH_NITEMS0,            // + 3*i : n_items, off_items, off_task_items for tile size kTileRows[i]
  DH_ZROWS = DH_NITEMS0 + 12, DH_RMAX, DH_WORDS, DH_OFF_ROWBITS,
  DH_ATT_NBLK,           // attention work lists: number of 128-row blocks of sequences, then the word offsets of the
  DH_ATT_OFF_FWD,        // list ordered for the passes that walk the keys before a block (longest walk first) and of the
  DH_ATT_OFF_BWD,        // list ordered for the pass that walks the queries after a block; 4 words an entry (DA_*)
  DH_OFF_ITEM_TOK0,      // per 64-row work item: how many tokens of its task lie on the rows before it
  DH_OFF_ITEM_BITS,      // per 64-row work item: two words, bit r = row row0 + r of the item is a real token
  DH_HDR_WORDS = 32
};
constexpr int kNumTileSizes = 4;
constexpr int kTileRows[kNumTileSizes] = {64, 128, 256, 1024};
constexpr uint32_t kDevMagic = 0x4458554Du;  // "MUXD"

// per task, 8 words
enum : int { DT_ROW_BEGIN = 0, DT_ROW_COUNT, DT_VALID, DT_KIND, DT_RANK, DT_SCALE_BITS, DT_ZROW0, DT_ITEM_PAD, DT_WORDS };
// per attention block, 4 words: the sequence's first row and length, the block's first token inside the sequence
enum : int { DA_FIRST_ROW = 0, DA_LEN, DA_BLOCK0, DA_PAD, DA_WORDS };
constexpr int kAttnBlockRows = 128;
// per work item, 4 words: rows [row0, row0+nrows) all belong to `task` (-1: rows of no task)
enum : int { DI_TASK = 0, DI_ROW0, DI_NROWS, DI_NVALID, DI_WORDS };

// Per-call task parameters in device memory (filled by a small kernel from launch arguments).
struct DevTask {
  const void* A;
  const void* B;
  const void* L;
  float* dA;
  float* dB;
  float* dL;
  float scale;
  int32_t kind;
  int32_t rank;
  int32_t row_begin;
  int32_t row_count;
  int32_t zrow0;      // first row of this task inside the saved x W region (IA3_OUT, TUNING) or inside the
                      // block-transposed copies (DIFF, a multiple of 64), else -1
  int64_t at_off;     // element offset of this task's transposed A_t inside the workspace region
                      // DIFF tasks: A = values, dA = their gradient, B = row_ptr, L = col_idx, dB = col_ptr, dL = col_ent
                      // (all int32 arrays), at_off = number of masked entries; rank = index of the task's merged
                      // weight W + M_t * delta_t in the workspace when the call builds them, or the element offset of
                      // the task's packed entries when the backbone product adds them in LDS, else -1
};
static_assert(sizeof(DevTask) == 80, "DevTask layout");

// The task parameters of a call as the kernels see them: up to kArgTasks tasks travel by value in the kernel
// arguments (no kernel has to write a table first); more tasks than that, and the kernels that take a plain pointer,
// read the table a small kernel wrote into the workspace.
constexpr int kArgTasks = 32;
struct TaskTable { DevTask t[kArgTasks]; };
struct TaskRef {
  const DevTask* mem;   // device table, or null: then `arg` holds the tasks
  TaskTable arg;
};

struct HostTask {
  int32_t kind, rank;
  float scale;
  int32_t row_begin, row_count, valid, zrow0;
};

struct Item { int32_t task, row0, nrows, nvalid; };

}  // namespace mux

struct mux_segtab {
  int32_t n_tasks = 0, chunk = 0, log2c = 0, n_chunks = 0, T = 0, valid_total = 0;
  int32_t max_pack_len = 0;
  uint32_t flags = 0;
  int32_t d_rows = 0;               // rows of the block-transposed copies of the DIFF tasks (each task rounded up to 64)
  int32_t r_max = 0, z_rows = 0, n_lora = 0, n_ia3 = 0, n_tuning = 0, n_diff = 0;   // r_max over the LORA and TUNING tasks
  std::vector<int32_t> image;       // canonical serialisation
  std::vector<int32_t> dev_image;   // device image (host copy, source of the upload)
  std::vector<int32_t> row_task;    // T entries
  std::vector<mux::HostTask> tasks;
  int32_t n_attn_blocks = 0;        // 128-row blocks of sequences (attention work items)
  std::vector<mux::Item> items[mux::kNumTileSizes];
  std::vector<int32_t> task_item_begin[mux::kNumTileSizes], task_item_count[mux::kNumTileSizes];
};

namespace mux {

mux_status fail(mux_status s, const std::string& msg);
void clear_error();

// Optional event bracketing of kernel launches (see mux_profile_enable).
void prof_note_bytes(double bytes);   // bytes the next bracketed launch moves (kernels the method itself asks no bytes of)
void prof_begin(const char* name, hipStream_t stream);
void prof_end(hipStream_t stream);
struct ProfScope {
  hipStream_t s;
  ProfScope(const char* name, hipStream_t stream) : s(stream) { prof_begin(name, stream); }
  ~ProfScope() { prof_end(s); }
};

// Device buffer of two 64-bit words set by mux_diag_set_clock_buffer (null when off): see mux_diag.h.
unsigned long long* diag_clock_buffer();

#define MUX_LAUNCH(name, kernel, grid, block, smem, stream, ...)         \
  do {                                                                   \
    ::mux::ProfScope mux_prof_scope_(name, stream);                      \
    hipLaunchKernelGGL(kernel, grid, block, smem, stream, __VA_ARGS__);  \
  } while (0)

inline int round_up(int v, int m) { return (v + m - 1) / m * m; }
inline size_t align256(size_t v) { return (v + 255) & ~size_t(255); }

// Everything a kernel launcher needs about one call.
struct CallCtx {
  const mux_segtab* st;
  const int32_t* dtab;     // device image
  const DevTask* dtasks;   // device table in the workspace (null when no kernel of this call reads it)
  const TaskRef* tref;     // what the matrix-core kernels take: that table, or the tasks by value
  int K, N;
  int64_t ldw;
  int RP;                  // row pitch (elements) of the H / G buffers
  void* AT;                // workspace: per-task A_t^T [round_up(r_t,16)][K] bf16 (forward, fast path)
  void* dYs;               // workspace [z_rows][N]: the backbone backward's input rows of the kinds that change it
                           // (IA3_OUT: dY * l_t, fast path only; TUNING: dY + p D_t^T)
  const void* W;
  hipStream_t stream;
  void* U2;                // saved: pre-activations z D_t of the TUNING rows, [T][RP] (null without such tasks)
  bool lora_natural;       // every LoRA rank is a multiple of 8: the down-projection reads A_t [K, r] as it is
  bool tune_natural;       // likewise every Adapter-Tuning rank: D_t [N, r] is read as it is, forward and backward
  int diff_max_nnz;        // largest mask of the DIFF tasks of this call
  void* diffT[2];          // workspace: block-transposed copies of the DIFF rows of X ([0]) and of dY ([1])
  void* diffW;             // workspace: per DIFF task with entries, W + M_t * delta_t [K][ldw] bf16 (matrix-core path;
                           // null: the sparse updates run after the backbone products instead)
  int64_t diffW_stride;    // elements between the merged weights of two tasks
  int diffW_slots;         // how many tasks have one
  void* diffPack;          // workspace: the masks' entries packed for the backbone product of this call, which adds
                           // them to the tiles of W in LDS (index << 16 | bf16 value; null: another route is taken)
};

// H / G row pitch in elements
inline int rank_pitch(const mux_segtab* st) { return (st->n_lora + st->n_tuning) > 0 ? round_up(st->r_max, 16) : 0; }

// plain (non matrix-core) kernels, both storage types
mux_status ref_forward(const CallCtx& c, int dtype, const void* X, void* Y, void* H, void* Z);
mux_status ref_backward(const CallCtx& c, int dtype, const void* X, const void* dY, const void* H,
                        const void* Z, void* G, void* dX, int accumulate);


// the same plain kernels, step by step (bit mask)
enum : unsigned {
  REF_DOWN = 1, REF_FWD = 2, REF_G = 4, REF_DB = 8, REF_DA = 16, REF_DL = 32, REF_DX = 64,
  REF_TUNE_DOWN = 128,   // TUNING forward, after z is saved: u = z D_t, Hs = s_t gelu(u)
  REF_TUNE_UP = 256,     // TUNING forward: Y = z + Hs U_t
  REF_TUNE_DZ = 512,     // TUNING backward, after Gs: dYs = dY + Gs D_t^T
  REF_ONLY_TUNING = 1024  // REF_G, REF_DB, REF_DA touch the TUNING tasks only (the LORA ones ran on the matrix cores)
};
void ref_steps(const CallCtx& c, int dtype, unsigned which, const void* X, const void* dY, void* Y, void* dX, void* H,
               void* Z, void* G, int accumulate);

// Diff-Pruning tasks, both storage types: the masked sparse update after the backbone GEMM, and the masked gradient
size_t diff_transposed_bytes(int K, int N, const mux_segtab* st, size_t esz);
size_t diff_merged_bytes(int K, int64_t ldw);      // one task's merged weight, bf16
void diff_pack(const CallCtx& c, bool backward);   // the packed entries the backbone product of this call adds in LDS
void diff_merge(const CallCtx& c, int slots);                                                                        // W + M_t * delta_t per task
void diff_forward(const CallCtx& c, int dtype, const void* X, void* Y);                                       // Y += x (M_t * delta_t)
void diff_backward(const CallCtx& c, int dtype, const void* X, const void* dY, void* dX, int accumulate);     // dX, d delta_t

// matrix-core backbone GEMM (bf16)
bool gemm_mfma_supported(const CallCtx& c);
mux_status gemm_mfma_forward(const CallCtx& c, const void* X, const void* Hs, void* Y, void* Z);
mux_status gemm_mfma_backward(const CallCtx& c, const void* dY, const void* Gs, void* dX, int only_ia3);
// pipelined variant (direct-to-LDS loads, 4 stages)
bool gemm_dma_supported(const CallCtx& c, bool backward);
bool fast_gemm_patches_diff(const CallCtx& c, bool backward);   // the backbone product of this call can add masked entries in LDS
bool gemm_dma_fuses_down(const CallCtx& c);   // the forward launch would be half / quarter tiles only: Hs is formed in its K loop
mux_status gemm_dma_forward(const CallCtx& c, const void* X, const void* Hs, void* Y, void* Z, bool fuse_down);
mux_status gemm_dma_backward(const CallCtx& c, const void* dY, const void* Gs, void* dX);

// matrix-core adapter kernels (bf16): down-projections and per-task gradient reductions
mux_status adapter_down_x(const CallCtx& c, const void* X, void* Hs);                       // S1
mux_status adapter_dy_pass(const CallCtx& c, const void* dY, const void* Hs, void* Gs, void* part);   // S4: Gs, dB partials
mux_status adapter_down_tune(const CallCtx& c, const void* Z, void* Hs);                    // Adapter-Tuning forward
mux_status adapter_tune_add(const CallCtx& c, const void* In, const void* Small, void* Out, int backward);
mux_status adapter_grads(const CallCtx& c, const void* X, const void* dY, const void* Hs, const void* Gs, const void* Z,
                         void* part, int accumulate);                                       // S6, and the sums of S4
size_t adapter_partial_bytes(int K, int N, const mux_segtab* st);

// matrix-core (MFMA) kernels, bf16 storage
size_t fast_partial_bytes(int K, int N, const mux_segtab* st);
bool fast_supported(const CallCtx& c, const void* p0, const void* p1, const void* p2, const void* p3, const void* p4,
                    const void* p5);   // shapes and pointers the 16-byte loads of the matrix-core kernels can take
mux_status fast_forward(const CallCtx& c, const void* X, void* Y, void* H, void* Z, void* part);
mux_status fast_backward(const CallCtx& c, const void* X, const void* dY, const void* H, const void* Z, void* G, void* dX,
                         int accumulate, void* part);

}  // namespace mux
