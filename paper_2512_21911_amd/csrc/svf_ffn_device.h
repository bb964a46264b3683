// Internal declarations of the sparse feed-forward translation units (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "svf.h"
#include "svf_ffn.h"

namespace svf {

struct FfnParams {
  const void* x;            // bf16 [M][d_model]
  const void* w_gate;       // bf16 [d_ff][d_model]
  const void* w_up;         // bf16 [d_ff][d_model]
  const void* w_down_t;     // bf16 [d_ff][d_model]
  const float* b_gate;      // fp32 [d_ff] or NULL
  const float* b_up;        // fp32 [d_ff] or NULL
  const float* b_down;      // fp32 [d_model] or NULL
  void* y;                  // bf16 [M][d_model]
  uint64_t* active;         // [d_ff] or NULL
  void* h_up;               // bf16 [64][d_ff]: h * up per token, zero where the token does not use the channel
  uint8_t* rowany;          // [d_ff]: nonzero = the channel is used by some token
  float* partial;           // fp32 [k_splits][M][d_model]
  int32_t M, d_model, d_ff, act, k_splits;
  int32_t fused_walk;       // gate and up matrices walked together (every row of W_up is read)
  int32_t tile_rows;        // channels per tile of the fused walk (<= 32)
  float tau;
};

// Slices of the hidden dimension the down projection is cut into (partial sums in the workspace).
int ffn_k_splits(int d_model, int d_ff);
int ffn_fused_tile_rows(int d_ff, int M);
hipError_t launch_sparse_ffn(const FfnParams& p, hipStream_t st);

}  // namespace svf
