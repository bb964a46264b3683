// Internal declarations shared by the libsvf translation units (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "svf.h"

namespace svf {

// Cache addressing handed to kernels by value (Sec. 3.1: the cache is addressed per token
// and per KV head; paging is this library's generalisation of "the current KV cache").
struct KvLayout {
  int64_t stride_page, stride_tok, stride_head;  // elements
  int32_t page_size;                             // 0 = contiguous (page index = sequence index)
  int32_t page_shift;                            // log2(page_size) if a power of two, else -1
  int32_t max_pages;                             // row length of block_table
};

// Element offset (without the head / channel part) of logical token t of sequence b.
__device__ __forceinline__ int64_t token_offset(const KvLayout& kv, const int32_t* __restrict__ table,
                                                int b, int t) {
  if (kv.page_size == 0) return (int64_t)b * kv.stride_page + (int64_t)t * kv.stride_tok;
  int p, s;
  if (kv.page_shift >= 0) {
    p = t >> kv.page_shift;
    s = t & (kv.page_size - 1);
  } else {
    p = t / kv.page_size;
    s = t - p * kv.page_size;
  }
  const int phys = table[(int64_t)b * kv.max_pages + p];
  return (int64_t)phys * kv.stride_page + (int64_t)s * kv.stride_tok;
}

struct RepsParams {
  KvLayout kv;
  const void* K;
  const int32_t* table;
  const int32_t* seq_lens;
  float* reps;
  int32_t Hkv, d, block_size, nb_max, first_block, n_blocks, max_seq_len;
};

struct SelectParams {
  const void* q;            // [B][gamma][Hq][d]
  const float* reps;        // [B][Hkv][nb_max][d]
  const int32_t* seq_lens;
  float* scores;            // [B][Hkv][nb_max]
  int32_t* sel_idx;         // [B][Hkv][k]
  int32_t* sel_cnt;         // [B][Hkv]
  int32_t B, gamma, Hq, Hkv, d, block_size, nb_max, k_blocks, n_sink, n_local, max_seq_len;
};

struct AttnParams {
  KvLayout kv;
  const void* q;
  const void* K;
  const void* V;
  const int32_t* table;
  const int32_t* seq_lens;
  const void* k_draft;
  const void* v_draft;
  const uint64_t* draft_mask;  // may be null
  const int32_t* sel_idx;
  const int32_t* sel_cnt;
  void* out;
  float* lse;                  // may be null
  float* part_o;               // [B][Hkv][S][Mpad][d]   unnormalised partial outputs
  float* part_m;               // [B][Hkv][S][Mpad]      running maxima (log2 domain)
  float* part_l;               // [B][Hkv][S][Mpad]      partial denominators
  float* part_ml;              // [B][Hkv][S][Mpad][2]   (maximum, denominator) pairs; aliases part_m / part_l
  uint64_t* tickets;           // [B][Hkv][row groups]   arrival counters, zero between calls
  int32_t B, gamma, Hq, Hkv, G, d, M, Mpad, block_size, k_blocks, n_splits, mask_per_batch, max_seq_len;
  int32_t block_shift;         // log2(block_size) if a power of two, else -1
  uint64_t g_magic;            // floor(2^32 / G) + 1: n / G == (n * g_magic) >> 32 for n, G < 65536
  uint64_t hkv_magic;          // the same for Hkv
  float scale_log2;            // sm_scale * log2(e)
};

// Prefix length of sequence b, clamped to what the shape allows so that a corrupt length
// cannot send a kernel outside the page table.
__device__ __forceinline__ int clamped_len(const int32_t* __restrict__ seq_lens, int b, int max_seq_len) {
  const int L = seq_lens[b];
  return L < 0 ? 0 : (L > max_seq_len ? max_seq_len : L);
}

// Launchers (each validates nothing: the C ABI layer has already done so).
hipError_t launch_block_reps(const RepsParams& p, int dtype, int B, hipStream_t st);
hipError_t launch_score_select(const SelectParams& p, int dtype, hipStream_t st);
hipError_t launch_fill_zero(void* ptr, size_t bytes, hipStream_t st);

// Host-side planning shared by svf_workspace_bytes and the attention launcher.
struct AttnPlan {
  int32_t M, Mpad, n_splits;
  bool mfma;                 // bf16, d = 128: matrix-core kernel; otherwise the vector-ALU kernel
  size_t off_o, off_m, off_l, off_tickets, bytes;
};
AttnPlan plan_attn(const svf_shape_t& s);

}  // namespace svf
