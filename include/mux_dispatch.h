/*
 * mux_dispatch.h -- C ABI of the Dispatch step (paper section 3.2: the rules that prepare the inputs of the batched
 * BaseOp; section 3.5: where a token sits in the chunk-aligned batch).
 *
 * A task hands over its tokens densely packed, [valid_t, width] row-major: its sequences one after the other in the
 * order of its seq_lens.  In the aligned batch those tokens occupy the task's valid rows in ascending order; every
 * other row is padding.  mux_dispatch_gather lays the aligned batch out (padding rows written as zero),
 * mux_dispatch_scatter brings the valid rows back.  Pure placement, bit-exact, any element type of 2 or 4 bytes.
 *
 * Conventions as in mux.h.  `task_ptrs` is a host array of n_tasks device pointers (NULL allowed for a task without
 * tokens); `ld_task` and `ld_aligned` are the elements between rows of the packed buffers and of the aligned one
 * (>= width); elem_bytes is 2 or 4.  Work is enqueued on the stream; nothing is allocated.
 */
#ifndef MUX_DISPATCH_H_
#define MUX_DISPATCH_H_

#include <stddef.h>
#include <stdint.h>

#include "mux.h"

#ifdef __cplusplus
extern "C" {
#endif

mux_status mux_dispatch_gather(const mux_segtab* st, const void* dev_segtab, const void* const* task_ptrs,
                               int64_t ld_task, void* aligned, int64_t ld_aligned, int32_t width, int32_t elem_bytes,
                               void* hip_stream);
mux_status mux_dispatch_scatter(const mux_segtab* st, const void* dev_segtab, const void* aligned, int64_t ld_aligned,
                                void* const* task_ptrs, int64_t ld_task, int32_t width, int32_t elem_bytes,
                                void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* MUX_DISPATCH_H_ */
