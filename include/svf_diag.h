/*
 * libsvf diagnostics - not part of the method's boundary (include/svf.h is).
 *
 * svf_verify_attn picks its kernel from the shape: the matrix-core kernel for bf16 with head
 * dimension 128, the vector-ALU kernel otherwise.  For measuring that choice (the packed query
 * rows per KV head, gamma x G of them, are few: whether the matrix cores pay at that size is a
 * question for the profiler) the call below runs the same attention (Sec. 3.1 / 3.3, same
 * arguments, same result within the output tolerance) with the kernel named by the caller.
 * Stateless like the rest of the library.
 */
#ifndef SVF_DIAG_H_
#define SVF_DIAG_H_

#include "svf.h"

#ifdef __cplusplus
extern "C" {
#endif

#define SVF_KERNEL_AUTO 0        /* what svf_verify_attn would run                       */
#define SVF_KERNEL_VECTOR_ALU 1  /* the vector-ALU kernel whatever the shape (and its merge launch) */

/* Workspace bytes svf_diag_verify_attn needs for `kernel` (>= svf_workspace_bytes; 0 if invalid). */
size_t svf_diag_workspace_bytes(const svf_shape_t* shape, int kernel);

/* svf_verify_attn with the kernel chosen by the caller; SVF_ERR_SHAPE for an unknown kernel. */
int svf_diag_verify_attn(const svf_shape_t* shape, int kernel, const void* q, const void* K, const void* V,
                         const int32_t* block_table, const int32_t* seq_lens, const void* k_draft,
                         const void* v_draft, const uint64_t* draft_mask_or_null, const int32_t* sel_idx,
                         const int32_t* sel_cnt, void* out, float* lse_or_null, void* ws, size_t ws_bytes,
                         void* stream);

/*
 * How often the bounded waits between the workgroups of a group ran out since the workspace was
 * last cleared (svf_workspace_init): counts[0] = workgroups that scored all blocks themselves after
 * waiting in vain for the others' block keys (anchor layers), counts[1] = wavefronts that left their
 * slice of the rows to the workgroup arriving last after waiting in vain for the others' partial
 * results.  The results are the same bits either way; a fallback costs time (microseconds per
 * launch), which is what this is for.  `counts`: two uint64 in device memory, written on `stream`.
 */
int svf_diag_wait_fallbacks(const svf_shape_t* shape, const void* ws, size_t ws_bytes, uint64_t* counts, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SVF_DIAG_H_ */
