/*
 * mux_attn.h -- C ABI of the attention step of a chunk-aligned batch (paper section 3.5).
 *
 * Between the q/k/v projections and the o projection of the multiplexed layer every sequence attends to itself:
 * the batch holds each task's sequences packed one after the other and cut along the chunk grid, a pack longer
 * than a chunk continues in the following chunks, and those chunks reuse the keys and values of the earlier ones.
 * What is computed is causal softmax attention of every sequence on its own -- token i of a sequence sees tokens
 * 0..i of that sequence, never another sequence of its pack, another task or a padding row:
 *     O_i = sum_{j <= i} softmax_j(scale * q_i . k_j) v_j          per head
 * The sequences come from the same table (mux_segtab) as the linear layers; rows follow its layout.
 *
 * Conventions as in mux.h.  Q, O, dO, dQ are device, bf16, [T, n_heads * head_dim] row-major, K, V, dK, dV
 * [T, n_kv_heads * head_dim], with the given leading dimensions (elements between rows; head h in columns
 * h*head_dim ..), so the three slices of a fused QKV buffer can be passed as they are.  n_kv_heads divides n_heads
 * (grouped-query attention: query head h reads key/value head h / (n_heads / n_kv_heads); dK, dV collect the
 * contributions of every query head of the group).  Rows of padding are written as zero in every output.
 * Supported now: MUX_DT_BF16, head_dim 64, 80, 96 or 128, leading dimensions that are multiples of 8 and 16-byte aligned
 * pointers; anything else returns MUX_ERR_UNSUPPORTED and launches nothing.
 */
#ifndef MUX_ATTN_H_
#define MUX_ATTN_H_

#include <stddef.h>
#include <stdint.h>

#include "mux.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
  int32_t n_heads;
  int32_t n_kv_heads; /* divides n_heads */
  int32_t head_dim;   /* 64, 80, 96 or 128 */
  int32_t dtype;      /* MUX_DT_BF16 */
  float scale;        /* 0: 1 / sqrt(head_dim) */
  int64_t ldq, ldk, ldv, ldo; /* elements between rows of Q (and dQ), K (and dK), V (and dV), O (and dO) */
} mux_attn_desc;

/* Bytes of `saved` (forward -> backward: the log of every row's softmax denominator, fp32 [n_heads][T]) and of the
 * backward's workspace (fp32 [n_heads][T]: sum_d dO * O per row and head). */
size_t mux_attn_saved_bytes(const mux_attn_desc* desc, const mux_segtab* st);
size_t mux_attn_workspace_bytes(const mux_attn_desc* desc, const mux_segtab* st);

/* Forward.  `saved` may be NULL when no backward pass follows.  O may not alias Q, K or V. */
mux_status mux_attn_forward(const mux_attn_desc* desc, const mux_segtab* st, const void* dev_segtab, const void* Q,
                            const void* K, const void* V, void* O, void* saved, void* hip_stream);

/* Backward of sum(O * dO): with P the softmax probabilities of a sequence and head,
 *     dV = P^T dO,   dS = P * (dO V^T - rowsum(dO * O)),   dQ = scale dS K,   dK = scale dS^T Q.
 * O and `saved` are the forward's.  Every output row is written (no accumulation); results repeat bit for bit
 * (every output element has one owner, no atomics). */
mux_status mux_attn_backward(const mux_attn_desc* desc, const mux_segtab* st, const void* dev_segtab, const void* Q,
                             const void* K, const void* V, const void* O, const void* dO, const void* saved, void* dQ,
                             void* dK, void* dV, void* ws, size_t ws_bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* MUX_ATTN_H_ */
