// Internal declarations shared by the libsvf translation units (not part of the C ABI).
#pragma once

#include <hip/hip_bf16.h>
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
  void* reps;               // [B][Hkv][nb_max][d], or [B][Hkv][nb_max][2][d] (minimum, maximum)
  int32_t Hkv, d, block_size, nb_max, first_block, n_blocks, max_seq_len;
  int32_t minmax, out_bf16;  // 0, 0: fp32 mean keys
};

// Gather list (an optional by-product of block selection that the matrix-core attention kernel
// can consume instead of walking sel_idx and the page table itself): for every (sequence, KV
// head), entry e describes the four consecutive selected-token slots 4e .. 4e+3 (slot = position
// in the concatenation of the kept blocks): bits [55:0] = byte offset of the first slot's K row
// from the start of the K pool (head offset included; V uses the same offset in its pool),
// bits [58:56] = number of those slots that hold a real token (0..4, a prefix of the four).
constexpr int kGatherCountShift = 56;
constexpr uint64_t kGatherOffsetMask = (1ull << kGatherCountShift) - 1ull;
constexpr int kMaxGatherBlocks = 1024;   // block budgets above this do without a gather list
constexpr int kTicketWords = 8;          // 64-bit words per (pair, row group) in AttnParams::tickets
// (statistics only, svf_diag_wait_fallbacks: they count up until the workspace is cleared)
constexpr int kTicketExchangeFallbacks = 3;   // workgroups that scored all blocks themselves after a starved key exchange
constexpr int kTicketMergeFallbacks = 6;      // wavefronts that gave a slice of rows up to the last arriver
constexpr int kDefaultWaitPolls = 64;    // polls a workgroup spends waiting for the others of its group
constexpr int kMaxWaitPolls = 4096;

struct SelectParams {
  const void* q;            // [B][gamma][Hq][d]
  const float* reps;        // [B][Hkv][nb_max][d]
  const int32_t* seq_lens;
  float* scores;            // [B][Hkv][nb_max]
  int32_t* sel_idx;         // [B][Hkv][k]
  int32_t* sel_cnt;         // [B][Hkv]
  int32_t B, gamma, Hq, Hkv, d, block_size, nb_max, k_blocks, n_sink, n_local, max_seq_len;
  // Retrieval per draft token (analytics, Sec. 2.2): nq = gamma queries per (sequence, KV head)
  // instead of the first one only; scores are then [B][nq][Hkv][nb_max], sel_idx (may be NULL)
  // [B][nq][Hkv][k], and the kept blocks can come out as bit masks [B][Hkv][nq][mask_words]
  // (block j = bit j % 64 of word j / 64).  nq = 1 is the method's own retrieval.
  int32_t nq;
  uint64_t* masks;          // NULL: none
  int32_t mask_words;
  // optional gather list output (NULL: none); needs the cache addressing of the layer
  uint64_t* gather;         // [B][Hkv][gather_groups]
  const int32_t* table;
  KvLayout kv;
  int32_t gather_groups;
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
  // split partials.  Vector-ALU kernel: fp32 unnormalised outputs [B][Hkv][S][Mpad][d] with their
  // running maxima (log2 domain) and denominators in part_m / part_l.  Matrix-core kernels: outputs
  // normalised by their own denominator and rounded to bf16, [B][Hkv][S][Mpad][d] 2-byte elements
  // in part_o, and 16-byte records (maximum, tag, denominator, tag) in part_rec, valid for the call
  // whose tag both halves carry.  part_m and part_rec name the same region.
  float* part_o;
  float* part_m;               // [B][Hkv][S][Mpad]
  float* part_l;               // [B][Hkv][S][Mpad]
  uint32_t* part_rec;          // [B][Hkv][S][Mpad][4]
  // per (pair, row group) eight 64-bit words: [0], [1] arrival word of calls with an even / odd
  // tag (bits 15:0 arrivals, bits 31:16 slices given up), [2] arrival counter of the kernels that
  // reset it themselves, [4], [5] (even / odd tag) where the group's workgroups run: eight 8-bit
  // counters, one per XCD, to which every workgroup adds one when it starts; [3], [6] statistics
  // (kTicketExchangeFallbacks, kTicketMergeFallbacks); [7] unused
  uint64_t* tickets;
  const uint64_t* gather;      // [B][Hkv][gather_groups] gather list matching sel_idx, or NULL
  int32_t gather_groups;
  // in-kernel retrieval (matrix-core kernel on anchor layers): reps != NULL switches it on
  const float* reps;           // [B][Hkv][nb_max][d]
  int32_t* sel_idx_out;        // [B][Hkv][k_blocks]
  int32_t* sel_cnt_out;        // [B][Hkv]
  uint64_t* gather_out;        // [B][Hkv][gather_groups]
  int32_t nb_max, n_sink, n_local;
  // exchange of block keys between the workgroups of a (pair, row group): one 64-bit word per
  // block (key in the low half, the call's tag in the high half)
  uint64_t* xkeys;             // [groups][nb_max]
  // per group: low half = calls completed on this group (the tag of a call is that count plus
  // one), high half = 0 or 1 + the number of polls a workgroup spends waiting for other workgroups
  // (svf_workspace_set_wait_polls)
  uint64_t* epochs;            // [groups]
  int32_t slice_rows;          // rows of a row group that one workgroup merges: ceil(32 / min(n_splits, 16))
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

// ---- block scores (Sec. 3.1, Eq. 5): pieces shared by the stand-alone scores kernel and the
// attention kernel that retrieves for itself, so that both produce the same bits ---------------

// Larger score <=> larger key; -0 and +0 map to the same key.
__device__ __forceinline__ uint32_t score_key(float s) {
  uint32_t u = __float_as_uint(s + 0.0f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Eight consecutive lanes own one block: lane s of the group holds the 16-byte channel chunks
// s, s + 8, s + 16, ... of the representative (so that each load instruction of the group covers
// 128 contiguous bytes).  Sum over the group, every lane receiving the total; fixed pairing
// lane ^ 1, lane ^ 2, mirror inside 8, all three cross-lane operand modifiers of the add itself.
constexpr int kScoreLanes = 8;
__device__ __forceinline__ float lane8_sum(float v) {
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xf, 0xf, true));    // quad_perm [1,0,3,2]
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xf, 0xf, true));    // quad_perm [2,3,0,1]
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xf, 0xf, true));   // row_half_mirror
  return v;
}

// q0 . representative for this lane's chunks, then over the lane group: a fixed chain of fused
// multiply-adds followed by lane8_sum.  NCH = d / 32 chunks per lane.
template <int NCH>
__device__ __forceinline__ float block_score(const float4 (&r)[NCH], const float4 (&q)[NCH]) {
  float acc = r[0].x * q[0].x;
  acc = __builtin_fmaf(r[0].y, q[0].y, acc);
  acc = __builtin_fmaf(r[0].z, q[0].z, acc);
  acc = __builtin_fmaf(r[0].w, q[0].w, acc);
#pragma unroll
  for (int i = 1; i < NCH; ++i) {
    acc = __builtin_fmaf(r[i].x, q[i].x, acc);
    acc = __builtin_fmaf(r[i].y, q[i].y, acc);
    acc = __builtin_fmaf(r[i].z, q[i].z, acc);
    acc = __builtin_fmaf(r[i].w, q[i].w, acc);
  }
  return lane8_sum(acc);
}

// Inclusive prefix sum over the 64 lanes with cross-lane operand modifiers only: shifts by
// 1, 2, 4, 8 inside each row of 16 lanes (lanes without a source add zero), then the last lane
// of row 0 / row 2 into rows 1 / 3, then the last lane of row 1 into rows 2 and 3.
__device__ __forceinline__ uint32_t wave_inclusive_sum(uint32_t x) {
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x111, 0xf, 0xf, true);   // row_shr:1
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x112, 0xf, 0xf, true);   // row_shr:2
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x114, 0xf, 0xf, true);   // row_shr:4
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x118, 0xf, 0xf, true);   // row_shr:8
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x142, 0xa, 0xf, false);  // row_bcast:15 -> rows 1, 3
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x143, 0xc, 0xf, false);  // row_bcast:31 -> rows 2, 3
  return x;
}

__device__ __forceinline__ float query_value(float x) { return x; }
__device__ __forceinline__ float query_value(__hip_bfloat16 x) { return __bfloat162float(x); }

// Channel c of the first draft token's query averaged over the G query heads of a KV head:
// heads added in order, then one division.  q points at channel c of the group's first head,
// heads are D elements apart.  In two steps so that a caller can put other loads between the
// (unconditional) loads of the first eight heads and the arithmetic that waits for them.
template <typename T>
struct QueryHeads { T v[8]; };
template <typename T>
__device__ __forceinline__ QueryHeads<T> load_query_heads(const T* q, int G, int D) {
  QueryHeads<T> h;
#pragma unroll
  for (int u = 0; u < 8; ++u) h.v[u] = q[(int64_t)min(u, G - 1) * D];
  return h;
}
template <typename T>
__device__ __forceinline__ float mean_query_channel(const QueryHeads<T>& h, const T* q, int G, int D) {
  float s = 0.f;
#pragma unroll
  for (int u = 0; u < 8; ++u)
    if (u < G) s += query_value(h.v[u]);
  for (int g = 8; g < G; ++g) s += query_value(q[(int64_t)g * D]);
  return s / (float)G;
}

// Retrieval variants (retrieval_variants.hip): scores of the first draft token per query head
// against mean-key or min/max summaries (fp32 or bf16), combined per KV head by mean or maximum;
// kept blocks per KV head (the selection kernel of score_select.hip) or over all KV heads of a
// sequence.
struct VariantParams {
  const void* q;            // [B][gamma][Hq][d]
  const void* summaries;
  const int32_t* seq_lens;
  float* scores;            // [B][Hkv][nb_max]
  int32_t* sel_idx;         // [B][Hkv][k_blocks]
  int32_t* sel_cnt;         // [B][Hkv]
  int32_t B, gamma, Hq, Hkv, d, block_size, nb_max, k_blocks, n_sink, n_local, max_seq_len;
  int32_t minmax, summary_bf16, group_max, n_total;
};
hipError_t launch_variant_scores(const VariantParams& p, int dtype, hipStream_t st);
hipError_t launch_select_global(const VariantParams& p, hipStream_t st);
hipError_t launch_scores_only(const SelectParams& p, int dtype, hipStream_t st);
hipError_t launch_select_only(const SelectParams& p, hipStream_t st);

// Launchers (each validates nothing: the C ABI layer has already done so).
hipError_t launch_block_reps(const RepsParams& p, int dtype, int B, hipStream_t st);
hipError_t launch_score_select(const SelectParams& p, int dtype, hipStream_t st);
// retrieval analytics (analytics.hip)
hipError_t launch_masks_from_selection(const int32_t* sel_idx, const int32_t* sel_cnt, uint64_t* masks, int pairs,
                                       int k_blocks, int mask_words, hipStream_t st);
hipError_t launch_overlap_by_distance(const uint64_t* masks, const int32_t* pos, uint64_t* inter, int B, int Hkv,
                                      int gamma, int mask_words, int n_dist, hipStream_t st);
hipError_t launch_jaccard_adjacent(const uint64_t* masks_by_layer, uint64_t* inter_union, int n_layers,
                                   int64_t words_per_layer, hipStream_t st);
hipError_t launch_fill_zero(void* ptr, size_t bytes, hipStream_t st);

// Host-side planning shared by svf_workspace_bytes and the attention launcher.
struct AttnPlan {
  int32_t M, Mpad, n_splits;
  int32_t slice_rows;        // rows of a row group one workgroup merges: ceil(32 / min(n_splits, 16))
  bool mfma;                 // bf16, d = 128: matrix-core kernel; otherwise the vector-ALU kernel
  bool fused_select;         // anchor layers retrieve inside the attention kernel
  bool gather;               // the shape can use a gather list
  int32_t gather_groups;     // entries per (sequence, KV head): a whole number of 32-token tiles
  size_t off_o, off_m, off_l, off_tickets, off_gather, off_xkeys, off_epochs, bytes;
  size_t groups;             // (sequence, KV head, row group) triples: entries of tickets / epochs
};
AttnPlan plan_attn(const svf_shape_t& s, bool allow_mfma = true);

}  // namespace svf
