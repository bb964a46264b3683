/*
 * libsvf - sparse feed-forward verification for speculative decoding on AMD MI355X (gfx950).
 *
 * C ABI of the sparse FFN of "Accelerate Speculative Decoding with Sparse Computation in
 * Verification" (Sec. 3.4, Eq. 10-14): while the draft tokens of a step are verified, hidden
 * channels whose gate activation is small are left out of the up and down projections.
 *
 * Conventions as in svf.h: shape and option structs are HOST pointers, every other pointer is
 * a DEVICE pointer owned by the caller; work is enqueued on `stream` and the call returns
 * immediately; 0 on success, a negative SVF_ERR_* code (svf.h) otherwise, checked before any
 * launch; inputs must be finite.
 *
 * Tensors (last index fastest; weights and activations bf16, biases fp32):
 *   x         bf16 [M][d_model]      hidden states of the M draft tokens (or draft-tree nodes)
 *   w_gate    bf16 [d_ff][d_model]   gate projection, one row per hidden channel
 *   w_up      bf16 [d_ff][d_model]   up projection, one row per hidden channel
 *   w_down_t  bf16 [d_ff][d_model]   down projection TRANSPOSED: row i is what hidden channel i
 *                                    adds to the output (column i of W_down), so that leaving a
 *                                    channel out leaves a contiguous row unread
 *   b_gate, b_up  fp32 [d_ff], b_down fp32 [d_model]; each may be NULL (= zeros)
 *   y         bf16 [M][d_model]
 *   active    uint64 [d_ff] (optional output): bit m set = channel i is used for token m
 */
#ifndef SVF_FFN_H_
#define SVF_FFN_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SVF_ACT_SILU 0 /* z / (1 + exp(-z)): the gate of SwiGLU */
#define SVF_ACT_GELU 1 /* 0.5 z (1 + erf(z / sqrt 2))           */

/* How the gate and the up matrix are read.  TOGETHER: one pass over both (x fetched once for both, no
 * pause between the passes); every row of w_up is read and only w_down_t skips the rows of
 * channels no token keeps.  GATE_FIRST: the gate matrix, then only the rows of w_up that some
 * token keeps; pays off when well over half of the channels are dropped by all tokens.  AUTO
 * currently means TOGETHER.  The outputs are the same up to the order of fp32 additions. */
#define SVF_FFN_WALK_AUTO 0
#define SVF_FFN_WALK_GATE_FIRST 1
#define SVF_FFN_WALK_TOGETHER 2

typedef struct svf_ffn_shape {
  int32_t M;       /* tokens verified together, 1..64                                  */
  int32_t d_model; /* model dimension, a multiple of 128                               */
  int32_t d_ff;    /* hidden channels, a multiple of 32                                */
  int32_t act;     /* SVF_ACT_*: sigma of Eq. 10                                       */
  float tau;       /* threshold of Eq. 12, >= 0; 0 keeps every channel (the dense FFN) */
  int32_t walk;    /* SVF_FFN_WALK_*: how the gate and up matrices are read (same result) */
} svf_ffn_shape_t;

/* Bytes of device workspace svf_sparse_ffn needs (multiple of 256; 0 if the shape is invalid).
 * The workspace needs no initialisation; calls sharing one must be ordered on one stream. */
size_t svf_ffn_workspace_bytes(const svf_ffn_shape_t* shape);

/*
 * Sparse feed-forward layer for M tokens (Eq. 10, 12-14), per token m:
 *   h      = act(W_gate x_m + b_gate)                          fp32 accumulation, fp32 h
 *   S_m    = { i : |h_i| < tau }                               (strict; decided on the fp32 h)
 *   y_m    = sum over i not in S_m of  h_i (W_up[i] . x_m + b_up[i]) W_down[:, i]  + b_down
 * The per-channel products h_i (..) are rounded to bf16 before the down projection and y to
 * bf16 at the end; all sums are fp32.  A weight row of w_down_t (and, with SVF_FFN_WALK_GATE_FIRST,
 * of w_up) is read only if its channel is outside S_m for at least one of the M tokens.  With
 * tau = 0 this is the dense layer of Eq. 10-11.
 * SVF_ERR_NULL (x, weights, y or ws NULL), SVF_ERR_SHAPE (shape out of range, a pointer not
 * 16-byte aligned, act or walk unknown, tau negative or not a number), SVF_ERR_WORKSPACE.
 */
int svf_sparse_ffn(const svf_ffn_shape_t* shape, const void* x, const void* w_gate, const void* w_up,
                   const void* w_down_t, const float* b_gate, const float* b_up, const float* b_down,
                   void* y, uint64_t* active_or_null, void* ws, size_t ws_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SVF_FFN_H_ */
