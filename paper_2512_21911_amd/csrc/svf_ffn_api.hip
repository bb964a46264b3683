// C ABI of the sparse feed-forward verification: argument checks, workspace layout, launches.
#include <cmath>

#include "svf_ffn_device.h"

namespace {

constexpr size_t kAlign = 256;
size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }
bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

int check_ffn_shape(const svf_ffn_shape_t* s) {
  if (!s) return SVF_ERR_NULL;
  if (s->M < 1 || s->M > 64) return SVF_ERR_SHAPE;
  if (s->d_model < 128 || s->d_model % 128 != 0 || s->d_model > (1 << 20)) return SVF_ERR_SHAPE;
  if (s->d_ff < 32 || s->d_ff % 32 != 0 || s->d_ff > (1 << 24)) return SVF_ERR_SHAPE;
  if (s->act != SVF_ACT_SILU && s->act != SVF_ACT_GELU) return SVF_ERR_SHAPE;
  if (!(s->tau >= 0.0f) || std::isinf(s->tau)) return SVF_ERR_SHAPE;
  if (s->walk != SVF_FFN_WALK_AUTO && s->walk != SVF_FFN_WALK_GATE_FIRST && s->walk != SVF_FFN_WALK_TOGETHER)
    return SVF_ERR_SHAPE;
  return SVF_OK;
}

struct FfnPlan {
  int k_splits;
  size_t off_h_up, off_rowmask, off_partial, bytes;
};

FfnPlan plan_ffn(const svf_ffn_shape_t& s) {
  FfnPlan pl;
  pl.k_splits = svf::ffn_k_splits(s.d_model, s.d_ff);
  size_t off = 0;
  pl.off_h_up = off;
  off += align_up((size_t)64 * s.d_ff * 2);
  pl.off_rowmask = off;
  off += align_up((size_t)s.d_ff);
  pl.off_partial = off;
  off += align_up((size_t)pl.k_splits * s.M * s.d_model * 4);
  pl.bytes = off;
  return pl;
}

}  // namespace

extern "C" {

size_t svf_ffn_workspace_bytes(const svf_ffn_shape_t* shape) {
  if (check_ffn_shape(shape) != SVF_OK) return 0;
  return plan_ffn(*shape).bytes;
}

int svf_sparse_ffn(const svf_ffn_shape_t* shape, const void* x, const void* w_gate, const void* w_up,
                   const void* w_down_t, const float* b_gate, const float* b_up, const float* b_down,
                   void* y, uint64_t* active_or_null, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_ffn_shape(shape);
  if (rc) return rc;
  if (!x || !w_gate || !w_up || !w_down_t || !y) return SVF_ERR_NULL;
  if (misaligned(x) || misaligned(w_gate) || misaligned(w_up) || misaligned(w_down_t) || misaligned(y) ||
      misaligned(b_gate) || misaligned(b_up) || misaligned(b_down) ||
      (reinterpret_cast<uintptr_t>(active_or_null) & 7u))
    return SVF_ERR_SHAPE;
  if (!ws || reinterpret_cast<uintptr_t>(ws) % kAlign) return SVF_ERR_WORKSPACE;
  const FfnPlan pl = plan_ffn(*shape);
  if (ws_bytes < pl.bytes) return SVF_ERR_WORKSPACE;
  svf::FfnParams p;
  p.x = x;
  p.w_gate = w_gate;
  p.w_up = w_up;
  p.w_down_t = w_down_t;
  p.b_gate = b_gate;
  p.b_up = b_up;
  p.b_down = b_down;
  p.y = y;
  p.active = active_or_null;
  char* w = static_cast<char*>(ws);
  p.h_up = w + pl.off_h_up;
  p.rowany = reinterpret_cast<uint8_t*>(w + pl.off_rowmask);
  p.partial = reinterpret_cast<float*>(w + pl.off_partial);
  p.M = shape->M;
  p.d_model = shape->d_model;
  p.d_ff = shape->d_ff;
  p.act = shape->act;
  p.k_splits = pl.k_splits;
  p.tau = shape->tau;
  p.fused_walk = shape->walk != SVF_FFN_WALK_GATE_FIRST;
  p.tile_rows = svf::ffn_fused_tile_rows(shape->d_ff, shape->M);
  return svf::launch_sparse_ffn(p, static_cast<hipStream_t>(stream)) == hipSuccess ? SVF_OK : SVF_ERR_HIP;
}

}  // extern "C"
