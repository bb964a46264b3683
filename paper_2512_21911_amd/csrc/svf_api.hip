// C ABI of libsvf: argument validation, workspace planning, kernel dispatch.
// Every check runs before the first launch; on error nothing has been enqueued.
#include <math.h>
#include <string.h>

#include <mutex>
#include <vector>

#include "svf_device.h"

namespace svf {

hipError_t launch_verify_attn_valu(const AttnParams& p, int dtype, hipStream_t st);
hipError_t launch_verify_attn_mfma(const AttnParams& p, hipStream_t st);
hipError_t launch_retrieve_only(const AttnParams& p, hipStream_t st);
bool mfma_supported(const svf_shape_t& s);
int mfma_splits(const svf_shape_t& s);
bool mfma_rows_mode(const svf_shape_t& s);
int mfma_rows_splits(const svf_shape_t& s);

namespace {

constexpr size_t kAlign = 256;

size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

int elem_bytes(int dtype) { return dtype == SVF_F32 ? 4 : 2; }

bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

int check_shape(const svf_shape_t* s) {
  if (!s) return SVF_ERR_NULL;
  if (s->dtype != SVF_F32 && s->dtype != SVF_BF16) return SVF_ERR_DTYPE;
  if (s->B < 1 || s->gamma < 1 || s->gamma > 64 || s->Hq < 1 || s->Hkv < 1 || s->Hq % s->Hkv != 0)
    return SVF_ERR_SHAPE;
  if (s->d != 64 && s->d != 128) return SVF_ERR_SHAPE;
  if (s->block_size < 1 || s->max_seq_len < 1 || s->page_size < 0) return SVF_ERR_SHAPE;
  const int vec = 16 / elem_bytes(s->dtype);
  if (s->kv_stride_tok < s->d || s->kv_stride_head < s->d || s->kv_stride_page < s->d) return SVF_ERR_SHAPE;
  if (s->kv_stride_tok % vec || s->kv_stride_head % vec || s->kv_stride_page % vec) return SVF_ERR_SHAPE;
  if (s->page_size > 0) {
    if (s->block_size % s->page_size != 0 && s->page_size % s->block_size != 0) return SVF_ERR_PAGING;
    if (s->max_pages_per_seq < 1 ||
        (int64_t)s->max_pages_per_seq * s->page_size < (int64_t)s->max_seq_len) return SVF_ERR_PAGING;
  }
  if (s->k_blocks < 1 || s->n_sink < 0 || s->n_local < 0 ||
      (int64_t)s->n_sink + s->n_local > s->k_blocks) return SVF_ERR_BUDGET;
  // (also keeps the number of splits per group, at most one per 8 tiles of 32 tokens, below 2^16:
  // the arrival counters of the attention kernels are 16 bits wide)
  if ((int64_t)s->k_blocks * s->block_size > (int64_t)1 << 23) return SVF_ERR_BUDGET;
  return SVF_OK;
}

int nb_max_of(const svf_shape_t& s) { return (s.max_seq_len + s.block_size - 1) / s.block_size; }

KvLayout layout_of(const svf_shape_t& s) {
  KvLayout kv;
  kv.stride_page = s.kv_stride_page;
  kv.stride_tok = s.kv_stride_tok;
  kv.stride_head = s.kv_stride_head;
  kv.page_size = s.page_size;
  kv.page_shift = -1;
  if (s.page_size > 0 && (s.page_size & (s.page_size - 1)) == 0) {
    int sh = 0;
    while ((1 << sh) < s.page_size) ++sh;
    kv.page_shift = sh;
  }
  kv.max_pages = s.max_pages_per_seq;
  return kv;
}

size_t scores_bytes(const svf_shape_t& s) {
  return align_up((size_t)s.B * s.Hkv * nb_max_of(s) * sizeof(float));
}

int check_ws(const svf_shape_t* s, const void* ws, size_t ws_bytes) {
  if (!ws) return SVF_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(ws) % kAlign) return SVF_ERR_WORKSPACE;
  if (ws_bytes < svf_workspace_bytes(s)) return SVF_ERR_WORKSPACE;
  return SVF_OK;
}

int hip_code(hipError_t e) { return e == hipSuccess ? SVF_OK : SVF_ERR_HIP; }

}  // namespace

// Workspace layout: [tickets | partial o | partial m, l / records | gather list | exchanged keys | epoch words],
// then (svf_workspace_bytes) the block scores of a selection whose caller does not ask for them
AttnPlan plan_attn(const svf_shape_t& s, bool allow_mfma) {
  AttnPlan pl;
  const int G = s.Hq / s.Hkv;
  pl.M = s.gamma * G;
  pl.Mpad = (pl.M + 31) / 32 * 32;
  pl.mfma = allow_mfma && mfma_supported(s);
  if (pl.mfma) {
    pl.n_splits = mfma_rows_mode(s) ? mfma_rows_splits(s) : mfma_splits(s);
  } else {
    const int64_t tiles = ((int64_t)s.k_blocks * s.block_size + 31) / 32 + (s.gamma + 31) / 32;
    const int64_t groups = (int64_t)s.B * s.Hkv * (pl.Mpad / 32);
    int64_t want = (512 + groups - 1) / groups;          // aim at ~2 workgroups per compute unit
    if (want > tiles) want = tiles;
    if (want < 1) want = 1;
    pl.n_splits = (int)want;
  }
  const size_t pairs = (size_t)s.B * s.Hkv;
  pl.groups = pairs * (pl.Mpad / 32);
  pl.slice_rows = (32 + (pl.n_splits < 16 ? pl.n_splits : 16) - 1) / (pl.n_splits < 16 ? pl.n_splits : 16);
  size_t off = 0;
  pl.off_tickets = off;
  off += align_up(pl.groups * kTicketWords * sizeof(uint64_t));
  // partial outputs: fp32 (vector-ALU kernel) or bf16 (matrix-core kernels) per split and row
  pl.off_o = off;
  off += align_up(pairs * pl.n_splits * pl.Mpad * s.d * (pl.mfma ? sizeof(uint16_t) : sizeof(float)));
  // maxima and denominators: two fp32 arrays for the vector-ALU kernel; 16 bytes per split and row
  // for the matrix-core kernels (a tagged record)
  pl.off_m = off;
  pl.off_l = off + pairs * pl.n_splits * pl.Mpad * sizeof(float);
  off += align_up((pl.mfma ? 4 : 2) * pairs * pl.n_splits * pl.Mpad * sizeof(float));
  pl.gather = pl.mfma && s.k_blocks <= kMaxGatherBlocks;
  pl.fused_select = pl.gather && nb_max_of(s) <= kMaxGatherBlocks;
  pl.gather_groups = pl.gather ? (int32_t)(((int64_t)s.k_blocks * s.block_size + 31) / 32 * 8) : 0;
  pl.off_gather = off;
  off += align_up(pairs * (size_t)pl.gather_groups * sizeof(uint64_t));
  // key exchange of the in-kernel retrieval: per (pair, row group)
  pl.off_xkeys = off;
  off += align_up(pl.fused_select ? pl.groups * (size_t)nb_max_of(s) * sizeof(uint64_t) : 0);
  pl.off_epochs = off;
  off += align_up(pl.groups * sizeof(uint64_t));
  pl.bytes = off;
  return pl;
}

namespace {

// high half of every group's epoch word: 0 (default wait budget) or the caller's number of polls plus one
__global__ void set_wait_polls_kernel(uint64_t* epochs, size_t n, uint32_t high_half) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) reinterpret_cast<uint32_t*>(epochs + i)[1] = high_half;
}

// zeroes up to three byte ranges (multiples of 16) of one buffer in one launch
struct ZeroRanges { size_t off[3], bytes[3]; };
__global__ void zero_ranges_kernel(char* base, ZeroRanges r) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (int k = 0; k < 3; ++k) {
    uint4* p = reinterpret_cast<uint4*>(base + r.off[k]);
    const size_t n16 = r.bytes[k] / 16;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) p[i] = make_uint4(0, 0, 0, 0);
  }
}

__global__ void fill_zero_kernel(uint4* p, size_t n16) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride)
    p[i] = make_uint4(0, 0, 0, 0);
}

}  // namespace

hipError_t launch_fill_zero(void* ptr, size_t bytes, hipStream_t st) {
  const size_t n16 = bytes / 16;
  if (n16 == 0) return hipSuccess;
  size_t blocks = (n16 + 255) / 256;
  if (blocks > 2048) blocks = 2048;
  hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)blocks), dim3(256), 0, st, static_cast<uint4*>(ptr), n16);
  return hipGetLastError();
}

}  // namespace svf

using namespace svf;

extern "C" {

int svf_version(void) { return 100; }

const char* svf_strerror(int code) {
  switch (code) {
    case SVF_OK: return "success";
    case SVF_ERR_NULL: return "a required pointer is NULL";
    case SVF_ERR_SHAPE: return "shape, stride or alignment out of range";
    case SVF_ERR_DTYPE: return "unsupported dtype";
    case SVF_ERR_PAGING: return "page size / block size / page table mismatch";
    case SVF_ERR_BUDGET: return "invalid block budget";
    case SVF_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case SVF_ERR_HIP: return "HIP launch failed";
    default: return "unknown error code";
  }
}

int32_t svf_budget_blocks(int64_t L, int64_t L0, double rho, int32_t block_size, int32_t* dense) {
  if (L < 1 || L0 < 0 || block_size < 1 || !(rho > 0.0 && rho < 1.0)) return SVF_ERR_SHAPE;
  const int64_t nb = (L + block_size - 1) / block_size;
  if (nb > INT32_MAX) return SVF_ERR_SHAPE;
  if (L <= L0) {
    if (dense) *dense = 1;
    return (int32_t)nb;
  }
  if (dense) *dense = 0;
  const double kept_tokens = (double)(L - L0) * rho + (double)L0;
  int64_t k = (int64_t)ceil(kept_tokens / (double)block_size - 1e-12);
  if (k < 1) k = 1;
  if (k > nb) k = nb;
  return (int32_t)k;
}

size_t svf_workspace_bytes(const svf_shape_t* shape) {
  if (check_shape(shape) != SVF_OK) return 0;
  return plan_attn(*shape).bytes + scores_bytes(*shape);
}

int svf_workspace_init(void* ws, size_t ws_bytes, void* stream) {
  if (!ws) return SVF_ERR_NULL;
  if (reinterpret_cast<uintptr_t>(ws) % kAlign || ws_bytes % 16) return SVF_ERR_WORKSPACE;
  return hip_code(launch_fill_zero(ws, ws_bytes, static_cast<hipStream_t>(stream)));
}

int svf_workspace_set_wait_polls(const svf_shape_t* shape, void* ws, size_t ws_bytes, int polls, void* stream) {
  int rc = check_shape(shape);
  if (rc) return rc;
  rc = check_ws(shape, ws, ws_bytes);
  if (rc) return rc;
  if (polls < -1 || polls > kMaxWaitPolls) return SVF_ERR_SHAPE;
  const AttnPlan pl = plan_attn(*shape);
  uint64_t* epochs = reinterpret_cast<uint64_t*>(static_cast<char*>(ws) + pl.off_epochs);
  hipLaunchKernelGGL(set_wait_polls_kernel, dim3((unsigned)((pl.groups + 255) / 256)), dim3(256), 0,
                     static_cast<hipStream_t>(stream), epochs, pl.groups, polls < 0 ? 0u : (uint32_t)polls + 1u);
  return hip_code(hipGetLastError());
}

static int block_reps_impl(const svf_shape_t* shape, const void* K, const int32_t* block_table,
                           const int32_t* seq_lens, int32_t first_block, int32_t n_blocks, void* reps,
                           void* stream, int minmax, int out_bf16) {
  int rc = check_shape(shape);
  if (rc) return rc;
  if (!K || !seq_lens || !reps || (shape->page_size > 0 && !block_table)) return SVF_ERR_NULL;
  if (misaligned(K) || misaligned(reps)) return SVF_ERR_SHAPE;
  const int nb_max = nb_max_of(*shape);
  if (first_block < 0 || first_block > nb_max || n_blocks < -1) return SVF_ERR_SHAPE;
  if (n_blocks == -1 || first_block + (int64_t)n_blocks > nb_max) n_blocks = nb_max - first_block;
  RepsParams p;
  p.kv = layout_of(*shape);
  p.K = K;
  p.table = block_table;
  p.seq_lens = seq_lens;
  p.reps = reps;
  p.Hkv = shape->Hkv;
  p.d = shape->d;
  p.block_size = shape->block_size;
  p.nb_max = nb_max;
  p.first_block = first_block;
  p.max_seq_len = shape->max_seq_len;
  p.n_blocks = n_blocks;
  p.minmax = minmax;
  p.out_bf16 = out_bf16;
  return hip_code(launch_block_reps(p, shape->dtype, shape->B, static_cast<hipStream_t>(stream)));
}

int svf_block_reps(const svf_shape_t* shape, const void* K, const int32_t* block_table,
                   const int32_t* seq_lens, int32_t first_block, int32_t n_blocks, float* reps,
                   void* stream) {
  return block_reps_impl(shape, K, block_table, seq_lens, first_block, n_blocks, reps, stream, 0, 0);
}

// block_table given (or the cache unpaged) and with_gather: the selection also leaves its gather
// list in the workspace
static int score_select_impl(const svf_shape_t* shape, const void* q, const float* reps,
                             const int32_t* seq_lens, int32_t* sel_idx, int32_t* sel_cnt,
                             float* scores_or_null, void* ws, size_t ws_bytes, void* stream,
                             bool with_gather, const int32_t* block_table) {
  int rc = check_shape(shape);
  if (rc) return rc;
  if (!q || !reps || !seq_lens || !sel_idx || !sel_cnt) return SVF_ERR_NULL;
  if (misaligned(q) || misaligned(reps)) return SVF_ERR_SHAPE;
  rc = check_ws(shape, ws, ws_bytes);
  if (rc) return rc;
  {
    // Shapes the retrieving attention kernel handles, when neither the scores nor a gather list
    // are asked for: its retrieval alone, one launch (the workgroups of a (sequence, KV head)
    // share the scoring), the same blocks bit for bit.
    const AttnPlan pl = plan_attn(*shape);
    if (pl.fused_select && !scores_or_null && !with_gather) {
      char* w = static_cast<char*>(ws);
      AttnParams a{};
      a.kv = layout_of(*shape);
      a.kv.page_size = 0;                                 // no page table in this call
      a.q = q;
      a.seq_lens = seq_lens;
      a.reps = reps;
      a.sel_idx_out = sel_idx;
      a.sel_cnt_out = sel_cnt;
      a.tickets = reinterpret_cast<uint64_t*>(w + pl.off_tickets);
      a.xkeys = reinterpret_cast<uint64_t*>(w + pl.off_xkeys);
      a.epochs = reinterpret_cast<uint64_t*>(w + pl.off_epochs);
      a.nb_max = nb_max_of(*shape);
      a.n_sink = shape->n_sink;
      a.n_local = shape->n_local;
      a.B = shape->B;
      a.gamma = shape->gamma;
      a.Hq = shape->Hq;
      a.Hkv = shape->Hkv;
      a.G = shape->Hq / shape->Hkv;
      a.d = shape->d;
      a.M = pl.M;
      a.Mpad = pl.Mpad;
      a.block_size = shape->block_size;
      a.k_blocks = shape->k_blocks;
      a.n_splits = pl.n_splits;
      a.max_seq_len = shape->max_seq_len;
      a.g_magic = (1ull << 32) / (uint64_t)a.G + 1ull;
      a.hkv_magic = (1ull << 32) / (uint64_t)a.Hkv + 1ull;
      return hip_code(launch_retrieve_only(a, static_cast<hipStream_t>(stream)));
    }
  }
  SelectParams p;
  p.q = q;
  p.reps = reps;
  p.seq_lens = seq_lens;
  p.scores = scores_or_null ? scores_or_null
                            : reinterpret_cast<float*>(static_cast<char*>(ws) + plan_attn(*shape).bytes);
  p.sel_idx = sel_idx;
  p.sel_cnt = sel_cnt;
  p.B = shape->B;
  p.gamma = shape->gamma;
  p.Hq = shape->Hq;
  p.Hkv = shape->Hkv;
  p.d = shape->d;
  p.block_size = shape->block_size;
  p.nb_max = nb_max_of(*shape);
  p.k_blocks = shape->k_blocks;
  p.n_sink = shape->n_sink;
  p.n_local = shape->n_local;
  p.max_seq_len = shape->max_seq_len;
  const AttnPlan pl = plan_attn(*shape);
  p.nq = 1;
  p.masks = nullptr;
  p.mask_words = 0;
  p.gather = nullptr;
  p.table = block_table;
  p.kv = layout_of(*shape);
  p.gather_groups = pl.gather_groups;
  if (with_gather && pl.gather) p.gather = reinterpret_cast<uint64_t*>(static_cast<char*>(ws) + pl.off_gather);
  return hip_code(launch_score_select(p, shape->dtype, static_cast<hipStream_t>(stream)));
}

int svf_score_select(const svf_shape_t* shape, const void* q, const float* reps,
                     const int32_t* seq_lens, int32_t* sel_idx, int32_t* sel_cnt,
                     float* scores_or_null, void* ws, size_t ws_bytes, void* stream) {
  return score_select_impl(shape, q, reps, seq_lens, sel_idx, sel_cnt, scores_or_null, ws, ws_bytes, stream,
                           false, nullptr);
}

// use_gather: the workspace holds the gather list of exactly this sel_idx / block_table / seq_lens
static int verify_attn_impl(const svf_shape_t* shape, const void* q, const void* K, const void* V,
                            const int32_t* block_table, const int32_t* seq_lens, const void* k_draft,
                            const void* v_draft, const uint64_t* draft_mask_or_null, const int32_t* sel_idx,
                            const int32_t* sel_cnt, void* out, float* lse_or_null, void* ws, size_t ws_bytes,
                            void* stream, bool use_gather, const float* reps_to_select_from = nullptr,
                            bool allow_mfma = true) {
  int rc = check_shape(shape);
  if (rc) return rc;
  if (!q || !K || !V || !seq_lens || !k_draft || !v_draft || !sel_idx || !sel_cnt || !out ||
      (shape->page_size > 0 && !block_table))
    return SVF_ERR_NULL;
  if (misaligned(q) || misaligned(K) || misaligned(V) || misaligned(k_draft) || misaligned(v_draft) ||
      misaligned(out))
    return SVF_ERR_SHAPE;
  rc = check_ws(shape, ws, ws_bytes);
  if (rc) return rc;
  const AttnPlan pl = plan_attn(*shape, allow_mfma);
  if (!allow_mfma && ws_bytes < pl.bytes) return SVF_ERR_WORKSPACE;
  char* w = static_cast<char*>(ws);
  AttnParams p;
  p.kv = layout_of(*shape);
  p.q = q;
  p.K = K;
  p.V = V;
  p.table = block_table;
  p.seq_lens = seq_lens;
  p.k_draft = k_draft;
  p.v_draft = v_draft;
  p.draft_mask = draft_mask_or_null;
  p.sel_idx = sel_idx;
  p.sel_cnt = sel_cnt;
  p.out = out;
  p.lse = lse_or_null;
  p.tickets = reinterpret_cast<uint64_t*>(w + pl.off_tickets);
  p.part_o = reinterpret_cast<float*>(w + pl.off_o);
  p.part_m = reinterpret_cast<float*>(w + pl.off_m);
  p.part_l = reinterpret_cast<float*>(w + pl.off_l);
  p.part_rec = reinterpret_cast<uint32_t*>(p.part_m);
  p.gather = (use_gather && pl.gather) ? reinterpret_cast<const uint64_t*>(w + pl.off_gather) : nullptr;
  p.gather_groups = pl.gather_groups;
  // retrieval inside the kernel: sel_idx / sel_cnt are then outputs (the caller passed them writable)
  p.reps = nullptr;
  p.sel_idx_out = nullptr;
  p.sel_cnt_out = nullptr;
  p.gather_out = nullptr;
  p.nb_max = nb_max_of(*shape);
  p.n_sink = shape->n_sink;
  p.n_local = shape->n_local;
  p.xkeys = reinterpret_cast<uint64_t*>(w + pl.off_xkeys);
  p.epochs = reinterpret_cast<uint64_t*>(w + pl.off_epochs);
  p.slice_rows = pl.slice_rows;
  if (reps_to_select_from && pl.fused_select) {
    p.reps = reps_to_select_from;
    p.sel_idx_out = const_cast<int32_t*>(sel_idx);
    p.sel_cnt_out = const_cast<int32_t*>(sel_cnt);
    p.gather_out = reinterpret_cast<uint64_t*>(w + pl.off_gather);
    p.gather = nullptr;
  }
  p.B = shape->B;
  p.gamma = shape->gamma;
  p.Hq = shape->Hq;
  p.Hkv = shape->Hkv;
  p.G = shape->Hq / shape->Hkv;
  p.d = shape->d;
  p.M = pl.M;
  p.Mpad = pl.Mpad;
  p.block_size = shape->block_size;
  p.k_blocks = shape->k_blocks;
  p.n_splits = pl.n_splits;
  p.mask_per_batch = shape->mask_per_batch;
  p.block_shift = -1;
  if ((shape->block_size & (shape->block_size - 1)) == 0)
    for (int sh = 0; sh < 31; ++sh)
      if ((1 << sh) == shape->block_size) p.block_shift = sh;
  p.g_magic = (1ull << 32) / (uint64_t)p.G + 1ull;
  p.hkv_magic = (1ull << 32) / (uint64_t)p.Hkv + 1ull;
  p.max_seq_len = shape->max_seq_len;
  const float scale = shape->sm_scale > 0.f ? shape->sm_scale : 1.0f / sqrtf((float)shape->d);
  p.scale_log2 = scale * 1.4426950408889634f;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (pl.mfma) return hip_code(launch_verify_attn_mfma(p, st));
  return hip_code(launch_verify_attn_valu(p, shape->dtype, st));
}

int svf_verify_attn(const svf_shape_t* shape, const void* q, const void* K, const void* V,
                    const int32_t* block_table, const int32_t* seq_lens, const void* k_draft,
                    const void* v_draft, const uint64_t* draft_mask_or_null, const int32_t* sel_idx,
                    const int32_t* sel_cnt, void* out, float* lse_or_null, void* ws, size_t ws_bytes,
                    void* stream) {
  return verify_attn_impl(shape, q, K, V, block_table, seq_lens, k_draft, v_draft, draft_mask_or_null, sel_idx,
                          sel_cnt, out, lse_or_null, ws, ws_bytes, stream, false);
}

// ---- the entry point that allocates nothing ---------------------------------------------------------
// Its workspace is this array (one copy per GPU, held until the process ends).  In host code the
// array's name is only a stand-in: the device address comes from hipGetSymbolAddress, once per device.
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices];          // per device, set on that device's first call

// Device address of `scratch` on the current device, or nullptr (with *rc set) on failure.
void* static_scratch(int* rc) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    *rc = SVF_ERR_HIP;
    return nullptr;
  }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
      *rc = SVF_ERR_HIP;
      return nullptr;
    }
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}
}  // namespace

size_t svf_static_workspace_bytes(void) { return kStaticScratchBytes; }

int svf_verify_attn_static_ws(const svf_shape_t* shape, const void* q, const void* K, const void* V,
                              const int32_t* block_table, const int32_t* seq_lens, const void* k_draft,
                              const void* v_draft, const uint64_t* draft_mask_or_null, const int32_t* sel_idx,
                              const int32_t* sel_cnt, void* out, float* lse_or_null, void* stream) {
  int rc = check_shape(shape);
  if (rc) return rc;
  if (!q || !K || !V || !seq_lens || !k_draft || !v_draft || !sel_idx || !sel_cnt || !out ||
      (shape->page_size > 0 && !block_table))
    return SVF_ERR_NULL;
  if (misaligned(q) || misaligned(K) || misaligned(V) || misaligned(k_draft) || misaligned(v_draft) ||
      misaligned(out))
    return SVF_ERR_SHAPE;
  // a shape whose workspace does not fit the array is refused
  if (svf_workspace_bytes(shape) > kStaticScratchBytes) return SVF_ERR_WORKSPACE;
  void* ws = static_scratch(&rc);
  if (!ws) return rc;
  // The array keeps what the last call left, of whatever shape: everything the kernels expect to
  // find zero (arrival words, call counters, exchanged keys, and the tagged records, whose tags
  // restart with the counters) is cleared first, by a fill kernel on the caller's stream.
  const AttnPlan pl = plan_attn(*shape);
  ZeroRanges zr;
  zr.off[0] = pl.off_tickets;
  zr.bytes[0] = pl.off_o - pl.off_tickets;
  zr.off[1] = pl.off_m;
  zr.bytes[1] = pl.off_gather - pl.off_m;
  zr.off[2] = pl.off_xkeys;
  zr.bytes[2] = pl.bytes - pl.off_xkeys;
  hipLaunchKernelGGL(zero_ranges_kernel, dim3(64), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<char*>(ws), zr);
  if (hipGetLastError() != hipSuccess) return SVF_ERR_HIP;
  return verify_attn_impl(shape, q, K, V, block_table, seq_lens, k_draft, v_draft, draft_mask_or_null, sel_idx,
                          sel_cnt, out, lse_or_null, ws, kStaticScratchBytes, stream, false);
}

// ---- diagnostics (include/svf_diag.h) ---------------------------------------------------------------
namespace {
// sums the statistics words of all groups into out[0] (exchange) and out[1] (merge); one workgroup
__global__ void sum_fallbacks_kernel(const uint64_t* tickets, size_t groups, uint64_t* out) {
  __shared__ unsigned long long acc[2];
  if (threadIdx.x < 2) acc[threadIdx.x] = 0ull;
  __syncthreads();
  unsigned long long a = 0ull, b = 0ull;
  for (size_t i = threadIdx.x; i < groups; i += blockDim.x) {
    a += tickets[i * svf::kTicketWords + svf::kTicketExchangeFallbacks];
    b += tickets[i * svf::kTicketWords + svf::kTicketMergeFallbacks];
  }
  atomicAdd(&acc[0], a);
  atomicAdd(&acc[1], b);
  __syncthreads();
  if (threadIdx.x < 2) out[threadIdx.x] = acc[threadIdx.x];
}
}  // namespace

int svf_diag_wait_fallbacks(const svf_shape_t* shape, const void* ws, size_t ws_bytes, uint64_t* counts, void* stream) {
  int rc = check_shape(shape);
  if (rc) return rc;
  rc = check_ws(shape, ws, ws_bytes);
  if (rc) return rc;
  if (!counts) return SVF_ERR_NULL;
  const AttnPlan pl = plan_attn(*shape);
  const uint64_t* tickets = reinterpret_cast<const uint64_t*>(static_cast<const char*>(ws) + pl.off_tickets);
  hipLaunchKernelGGL(sum_fallbacks_kernel, dim3(1), dim3(256), 0, static_cast<hipStream_t>(stream), tickets, pl.groups, counts);
  return hip_code(hipGetLastError());
}

// the attention with the kernel chosen by the caller
size_t svf_diag_workspace_bytes(const svf_shape_t* shape, int kernel) {
  if (check_shape(shape) != SVF_OK || (kernel != 0 && kernel != 1)) return 0;
  const size_t own = plan_attn(*shape, kernel == 0).bytes + scores_bytes(*shape);
  const size_t usual = svf_workspace_bytes(shape);
  return own > usual ? own : usual;
}

int svf_diag_verify_attn(const svf_shape_t* shape, int kernel, const void* q, const void* K, const void* V,
                         const int32_t* block_table, const int32_t* seq_lens, const void* k_draft,
                         const void* v_draft, const uint64_t* draft_mask_or_null, const int32_t* sel_idx,
                         const int32_t* sel_cnt, void* out, float* lse_or_null, void* ws, size_t ws_bytes,
                         void* stream) {
  if (kernel != 0 && kernel != 1) return SVF_ERR_SHAPE;
  return verify_attn_impl(shape, q, K, V, block_table, seq_lens, k_draft, v_draft, draft_mask_or_null, sel_idx,
                          sel_cnt, out, lse_or_null, ws, ws_bytes, stream, false, nullptr, kernel == 0);
}

int svf_verify_step(const svf_shape_t* shape, int mode, const void* q, const float* reps,
                    const void* K, const void* V, const int32_t* block_table, const int32_t* seq_lens,
                    const void* k_draft, const void* v_draft, const uint64_t* draft_mask_or_null,
                    int32_t* sel_idx, int32_t* sel_cnt, void* out, float* lse_or_null, void* ws,
                    size_t ws_bytes, void* stream) {
  // validate everything both halves need before enqueuing the first one
  if (mode != SVF_STEP_REUSE && mode != SVF_STEP_ANCHOR && mode != SVF_STEP_REUSE_GATHER) return SVF_ERR_SHAPE;
  const bool do_select = mode == SVF_STEP_ANCHOR;
  int rc = check_shape(shape);
  if (rc) return rc;
  if (!q || !K || !V || !seq_lens || !k_draft || !v_draft || !sel_idx || !sel_cnt || !out ||
      (shape->page_size > 0 && !block_table) || (do_select && !reps))
    return SVF_ERR_NULL;
  if (misaligned(q) || misaligned(K) || misaligned(V) || misaligned(k_draft) || misaligned(v_draft) ||
      misaligned(out) || (do_select && misaligned(reps)))
    return SVF_ERR_SHAPE;
  rc = check_ws(shape, ws, ws_bytes);
  if (rc) return rc;
  if (do_select && plan_attn(*shape).fused_select)
    return verify_attn_impl(shape, q, K, V, block_table, seq_lens, k_draft, v_draft, draft_mask_or_null, sel_idx,
                            sel_cnt, out, lse_or_null, ws, ws_bytes, stream, false, reps);
  if (do_select) {
    rc = score_select_impl(shape, q, reps, seq_lens, sel_idx, sel_cnt, nullptr, ws, ws_bytes, stream, true,
                           block_table);
    if (rc) return rc;
  }
  return verify_attn_impl(shape, q, K, V, block_table, seq_lens, k_draft, v_draft, draft_mask_or_null, sel_idx,
                          sel_cnt, out, lse_or_null, ws, ws_bytes, stream, mode != SVF_STEP_REUSE);
}

// ---- retrieval analytics -------------------------------------------------------------------

int32_t svf_mask_words(const svf_shape_t* shape) {
  if (check_shape(shape) != SVF_OK) return 0;
  return (nb_max_of(*shape) + 63) / 64;
}

size_t svf_analytics_workspace_bytes(const svf_shape_t* shape) {
  if (check_shape(shape) != SVF_OK) return 0;
  return align_up((size_t)shape->B * shape->gamma * shape->Hkv * nb_max_of(*shape) * sizeof(float));
}

int svf_select_per_draft(const svf_shape_t* shape, const void* q, const float* reps, const int32_t* seq_lens,
                         uint64_t* masks, float* scores_or_null, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_shape(shape);
  if (rc) return rc;
  if (!q || !reps || !seq_lens || !masks) return SVF_ERR_NULL;
  if (misaligned(q) || misaligned(reps)) return SVF_ERR_SHAPE;
  if (!scores_or_null) {
    if (!ws || reinterpret_cast<uintptr_t>(ws) % kAlign || ws_bytes < svf_analytics_workspace_bytes(shape))
      return SVF_ERR_WORKSPACE;
  }
  SelectParams p;
  p.q = q;
  p.reps = reps;
  p.seq_lens = seq_lens;
  p.scores = scores_or_null ? scores_or_null : static_cast<float*>(ws);
  p.sel_idx = nullptr;
  p.sel_cnt = nullptr;
  p.B = shape->B;
  p.gamma = shape->gamma;
  p.Hq = shape->Hq;
  p.Hkv = shape->Hkv;
  p.d = shape->d;
  p.block_size = shape->block_size;
  p.nb_max = nb_max_of(*shape);
  p.k_blocks = shape->k_blocks;
  p.n_sink = shape->n_sink;
  p.n_local = shape->n_local;
  p.max_seq_len = shape->max_seq_len;
  p.nq = shape->gamma;
  p.masks = masks;
  p.mask_words = (p.nb_max + 63) / 64;
  p.gather = nullptr;
  p.table = nullptr;
  p.kv = layout_of(*shape);
  p.gather_groups = 0;
  return hip_code(launch_score_select(p, shape->dtype, static_cast<hipStream_t>(stream)));
}

int svf_masks_from_selection(const svf_shape_t* shape, const int32_t* sel_idx, const int32_t* sel_cnt,
                             uint64_t* masks, void* stream) {
  int rc = check_shape(shape);
  if (rc) return rc;
  if (!sel_idx || !sel_cnt || !masks) return SVF_ERR_NULL;
  const int words = (nb_max_of(*shape) + 63) / 64;
  if ((size_t)words * 8 > 48 * 1024) return SVF_ERR_SHAPE;          // the mask of one pair is built in LDS
  return hip_code(launch_masks_from_selection(sel_idx, sel_cnt, masks, shape->B * shape->Hkv, shape->k_blocks, words,
                                              static_cast<hipStream_t>(stream)));
}

int svf_overlap_by_distance(const svf_shape_t* shape, const uint64_t* masks, const int32_t* pos, int32_t n_dist,
                            uint64_t* inter, void* stream) {
  int rc = check_shape(shape);
  if (rc) return rc;
  if (!masks || !pos || !inter) return SVF_ERR_NULL;
  const int words = (nb_max_of(*shape) + 63) / 64;
  if (n_dist < 1 || n_dist > 64 || words > 64 || shape->gamma > 64) return SVF_ERR_SHAPE;
  return hip_code(launch_overlap_by_distance(masks, pos, inter, shape->B, shape->Hkv, shape->gamma, words, n_dist,
                                             static_cast<hipStream_t>(stream)));
}

int svf_jaccard_adjacent(const svf_shape_t* shape, const uint64_t* masks_by_layer, int32_t n_layers,
                         uint64_t* inter_union, void* stream) {
  int rc = check_shape(shape);
  if (rc) return rc;
  if (!masks_by_layer || !inter_union) return SVF_ERR_NULL;
  if (n_layers < 1 || n_layers > 65535) return SVF_ERR_SHAPE;
  const int64_t words = (int64_t)shape->B * shape->Hkv * ((nb_max_of(*shape) + 63) / 64);
  return hip_code(launch_jaccard_adjacent(masks_by_layer, inter_union, n_layers, words,
                                          static_cast<hipStream_t>(stream)));
}

int svf_topk_anchors(const double* J, int32_t n_layers, int32_t K, int32_t* anchors) {
  if (!J || !anchors) return SVF_ERR_NULL;
  if (n_layers < 1 || K < 1 || K > n_layers) return SVF_ERR_SHAPE;
  for (int32_t l = 0; l < n_layers; ++l)
    if (!(J[l] >= 0.0 && J[l] <= 1.0)) return SVF_ERR_SHAPE;
  // K rounds of "largest 1 - J not taken yet, lowest layer first" (n_layers is a layer count)
  std::vector<char> taken((size_t)n_layers, 0);
  for (int32_t r = 0; r < K; ++r) {
    int32_t best = -1;
    for (int32_t l = 0; l < n_layers; ++l)
      if (!taken[l] && (best < 0 || 1.0 - J[l] > 1.0 - J[best])) best = l;
    taken[best] = 1;
  }
  int32_t n = 0;
  for (int32_t l = 0; l < n_layers; ++l)
    if (taken[l]) anchors[n++] = l;
  return SVF_OK;
}

/* ---- retrieval variants ------------------------------------------------------------------- */

static int check_retrieval(const svf_shape_t* shape, const svf_retrieval_t* r) {
  if (!r) return SVF_ERR_NULL;
  if (r->summary != SVF_SUMMARY_MEAN && r->summary != SVF_SUMMARY_MINMAX) return SVF_ERR_SHAPE;
  if (r->summary_dtype != SVF_F32 && r->summary_dtype != SVF_BF16) return SVF_ERR_DTYPE;
  if (r->group_rule != SVF_GROUP_MEAN && r->group_rule != SVF_GROUP_MAX) return SVF_ERR_SHAPE;
  if (r->budget_rule != SVF_BUDGET_PER_HEAD && r->budget_rule != SVF_BUDGET_GLOBAL) return SVF_ERR_SHAPE;
  if (r->budget_rule == SVF_BUDGET_GLOBAL) {
    const int64_t nb_max = nb_max_of(*shape);
    if (r->n_total < 1 || ((int64_t)shape->n_sink + shape->n_local) * shape->Hkv > r->n_total) return SVF_ERR_BUDGET;
    if (shape->k_blocks < (nb_max < r->n_total ? nb_max : (int64_t)r->n_total)) return SVF_ERR_BUDGET;
  }
  return SVF_OK;
}

static bool default_scores(const svf_retrieval_t& r) {
  return r.summary == SVF_SUMMARY_MEAN && r.summary_dtype == SVF_F32 && r.group_rule == SVF_GROUP_MEAN;
}

int svf_block_summaries(const svf_shape_t* shape, const svf_retrieval_t* retrieval, const void* K,
                        const int32_t* block_table, const int32_t* seq_lens, int32_t first_block,
                        int32_t n_blocks, void* summaries, void* stream) {
  int rc = check_shape(shape);
  if (rc) return rc;
  rc = check_retrieval(shape, retrieval);
  if (rc) return rc;
  return block_reps_impl(shape, K, block_table, seq_lens, first_block, n_blocks, summaries, stream,
                         retrieval->summary == SVF_SUMMARY_MINMAX, retrieval->summary_dtype == SVF_BF16);
}

int svf_retrieve(const svf_shape_t* shape, const svf_retrieval_t* retrieval, const void* q,
                 const void* summaries, const int32_t* seq_lens, int32_t* sel_idx, int32_t* sel_cnt,
                 float* scores_or_null, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_shape(shape);
  if (rc) return rc;
  rc = check_retrieval(shape, retrieval);
  if (rc) return rc;
  const svf_retrieval_t& r = *retrieval;
  if (default_scores(r) && r.budget_rule == SVF_BUDGET_PER_HEAD)
    return svf_score_select(shape, q, static_cast<const float*>(summaries), seq_lens, sel_idx, sel_cnt,
                            scores_or_null, ws, ws_bytes, stream);
  if (!q || !summaries || !seq_lens || !sel_idx || !sel_cnt) return SVF_ERR_NULL;
  if (misaligned(q) || misaligned(summaries)) return SVF_ERR_SHAPE;
  rc = check_ws(shape, ws, ws_bytes);
  if (rc) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  float* scores = scores_or_null ? scores_or_null
                                 : reinterpret_cast<float*>(static_cast<char*>(ws) + plan_attn(*shape).bytes);
  VariantParams v;
  v.q = q;
  v.summaries = summaries;
  v.seq_lens = seq_lens;
  v.scores = scores;
  v.sel_idx = sel_idx;
  v.sel_cnt = sel_cnt;
  v.B = shape->B;
  v.gamma = shape->gamma;
  v.Hq = shape->Hq;
  v.Hkv = shape->Hkv;
  v.d = shape->d;
  v.block_size = shape->block_size;
  v.nb_max = nb_max_of(*shape);
  v.k_blocks = shape->k_blocks;
  v.n_sink = shape->n_sink;
  v.n_local = shape->n_local;
  v.max_seq_len = shape->max_seq_len;
  v.minmax = r.summary == SVF_SUMMARY_MINMAX;
  v.summary_bf16 = r.summary_dtype == SVF_BF16;
  v.group_max = r.group_rule == SVF_GROUP_MAX;
  v.n_total = r.n_total;
  // the main path's own kernels wherever the rule is the main path's (same bits as svf_score_select)
  SelectParams p;
  p.q = q;
  p.reps = static_cast<const float*>(summaries);
  p.seq_lens = seq_lens;
  p.scores = scores;
  p.sel_idx = sel_idx;
  p.sel_cnt = sel_cnt;
  p.B = v.B; p.gamma = v.gamma; p.Hq = v.Hq; p.Hkv = v.Hkv; p.d = v.d;
  p.block_size = v.block_size; p.nb_max = v.nb_max; p.k_blocks = v.k_blocks;
  p.n_sink = v.n_sink; p.n_local = v.n_local; p.max_seq_len = v.max_seq_len;
  p.nq = 1;
  p.masks = nullptr;
  p.mask_words = 0;
  p.gather = nullptr;
  p.table = nullptr;
  p.kv = layout_of(*shape);
  p.gather_groups = 0;
  hipError_t e;
  if (default_scores(r)) e = launch_scores_only(p, shape->dtype, st);
  else e = launch_variant_scores(v, shape->dtype, st);
  if (e != hipSuccess) return SVF_ERR_HIP;
  if (r.budget_rule == SVF_BUDGET_PER_HEAD) return hip_code(launch_select_only(p, st));
  return hip_code(launch_select_global(v, st));
}

}  // extern "C"
