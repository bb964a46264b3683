/*
 * libsvf - sparse verification attention for speculative decoding on AMD MI355X (gfx950).
 *
 * C ABI of the verification-attention path of "Accelerate Speculative Decoding with
 * Sparse Computation in Verification" (Sec. 3.1 Sparse Attention, Sec. 3.2 Piecewise
 * Budget Control, Sec. 3.3 Inter-layer Retrieval Reuse).
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 *  - `const svf_shape_t*` is a HOST pointer.  Every other pointer is a DEVICE pointer
 *    owned by the caller; the library never allocates, frees or synchronises.
 *  - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the null
 *    stream) and the call returns immediately.
 *  - Return value: 0 on success, a negative SVF_ERR_* code otherwise.  All argument
 *    checks happen before any kernel launch; on error nothing has been enqueued.
 *  - Inputs must be finite.  NaN / Inf in q, K, V give unspecified results.
 *  - Tensor layouts (last index fastest):
 *      q, out          [B][gamma][Hq][d]          element type = shape.dtype
 *      k_draft,v_draft [B][gamma][Hkv][d]         element type = shape.dtype
 *      K, V            cache pool, element type = shape.dtype, addressed as
 *                        pool + page*kv_stride_page + slot*kv_stride_tok + h*kv_stride_head + c
 *                      (strides in elements, c in [0,d) contiguous).  With page_size > 0
 *                      token t of sequence b sits in page block_table[b][t / page_size],
 *                      slot t % page_size.  With page_size == 0 the cache is contiguous:
 *                      page = b, slot = t, block_table is ignored (may be NULL).
 *      block_table     int32 [B][max_pages_per_seq]
 *      seq_lens        int32 [B]   prefix length per sequence, drafts excluded, 1..max_seq_len
 *      reps            fp32  [B][Hkv][nb_max][d],  nb_max = ceil(max_seq_len / block_size)
 *      scores          fp32  [B][Hkv][nb_max]
 *      sel_idx         int32 [B][Hkv][k_blocks]   ascending block ids, padded with -1
 *      sel_cnt         int32 [B][Hkv]             = min(k_blocks, ceil(seq_len/block_size))
 *      draft_mask      uint64 [gamma] (or [B][gamma] when mask_per_batch): bit t of entry i
 *                      set = draft i attends draft t; bit i must be set.  NULL = linear
 *                      causal drafts (bits 0..i).
 *      lse             fp32  [B][gamma][Hq]       natural log of sum(exp(scaled logits))
 *  - Query head j belongs to KV head j / (Hq/Hkv).
 */
#ifndef SVF_H_
#define SVF_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { SVF_F32 = 0, SVF_BF16 = 1 };

enum {
  SVF_OK = 0,
  SVF_ERR_NULL = -1,      /* a required pointer is NULL                                    */
  SVF_ERR_SHAPE = -2,     /* B/gamma/Hq/Hkv/d/block_size/max_seq_len/strides out of range  */
  SVF_ERR_DTYPE = -3,     /* dtype not SVF_F32 / SVF_BF16                                  */
  SVF_ERR_PAGING = -4,    /* page_size and block_size not multiples of one another, or
                             max_pages_per_seq too small for max_seq_len                   */
  SVF_ERR_BUDGET = -5,    /* k_blocks < 1, n_sink + n_local > k_blocks, or more than 2^23
                             tokens kept per (sequence, KV head)                           */
  SVF_ERR_WORKSPACE = -6, /* workspace NULL, misaligned (256 B) or smaller than required   */
  SVF_ERR_HIP = -7        /* the HIP runtime refused a launch                              */
};

typedef struct svf_shape {
  int32_t B;                 /* sequences in the batch, >= 1                                 */
  int32_t gamma;             /* draft tokens (or draft-tree nodes) per sequence, 1..64       */
  int32_t Hq, Hkv;           /* query heads, KV heads; Hq % Hkv == 0                         */
  int32_t d;                 /* head dimension: 64 or 128                                    */
  int32_t dtype;             /* SVF_F32 or SVF_BF16                                          */
  int32_t block_size;        /* Bs: tokens per retrieval block (Sec. 3.1), >= 1              */
  int32_t page_size;         /* tokens per physical page; 0 = contiguous cache               */
  int32_t max_pages_per_seq; /* row length of block_table (unused when page_size == 0)       */
  int32_t max_seq_len;       /* largest prefix length any sequence may have                  */
  int64_t kv_stride_page;    /* elements between pages (contiguous: between sequences)       */
  int64_t kv_stride_tok;     /* elements between tokens of a page                            */
  int64_t kv_stride_head;    /* elements between KV heads of a token                         */
  int32_t k_blocks;          /* retrieval budget per (sequence, KV head), in blocks          */
  int32_t n_sink, n_local;   /* first / last blocks that are never evicted (inside k_blocks) */
  int32_t mask_per_batch;    /* 0: draft_mask is [gamma]; 1: [B][gamma]                      */
  float sm_scale;            /* softmax scale; <= 0 selects 1/sqrt(d)                        */
} svf_shape_t;

/* Library version (major*10000 + minor*100 + patch). */
int svf_version(void);

/* Static text for an SVF_ERR_* code. */
const char* svf_strerror(int code);

/*
 * Piecewise budget control, Sec. 3.2, Eq. 6, expressed per KV head and in blocks.
 * L <= L0: no eviction, returns ceil(L/block_size) and sets *dense = 1.
 * L  > L0: returns ceil(((L - L0) * rho + L0) / block_size) clamped to [1, ceil(L/block_size)],
 *          *dense = 0.  `dense` may be NULL.  Host-only arithmetic; returns a negative
 *          SVF_ERR_SHAPE for L < 1, L0 < 0, block_size < 1 or rho outside (0, 1).
 */
int32_t svf_budget_blocks(int64_t L, int64_t L0, double rho, int32_t block_size, int32_t* dense);

/*
 * Bytes of device workspace the calls below need for `shape` (always a multiple of 256;
 * 0 if the shape is invalid).  The workspace must be 256-byte aligned and must have been
 * cleared to zero once (svf_workspace_init) before its first use; the library leaves it
 * in a reusable state after every call.  Calls that share one workspace must be ordered
 * on one stream.  A workspace serves one shape: clear it again before using it with another.
 */
size_t svf_workspace_bytes(const svf_shape_t* shape);

/* Enqueue the one-time clearing of a workspace (a fill kernel; safe under graph capture). */
int svf_workspace_init(void* ws, size_t ws_bytes, void* stream);

/*
 * Tuning / test knob, carried by the workspace (the library keeps no state of its own).  The
 * workgroups that share one (sequence, KV head, row group) wait for each other in two places: on
 * anchor layers each scores a share of the blocks and waits for the others' keys, and every
 * workgroup merges a slice of the rows once the others' partial results have landed.  Both waits
 * are bounded by `polls` (default 64); a workgroup that runs out of patience scores all blocks
 * itself, respectively leaves its slice to the workgroup that arrives last.  The results are the
 * same bits whatever the number.  0 <= polls <= 4096 (0: never wait), -1 restores the default;
 * anything else SVF_ERR_SHAPE.  Enqueued on `stream` (a small fill kernel); svf_workspace_init
 * also restores the default.
 */
int svf_workspace_set_wait_polls(const svf_shape_t* shape, void* ws, size_t ws_bytes, int polls, void* stream);

/*
 * Block representatives (Sec. 3.1: the cache is partitioned per KV head into blocks of
 * block_size consecutive tokens, Eq. 4; the block term of Eq. 5 is the mean of its keys).
 *   reps[b][h][j][:] = mean over tokens t of block j of K[b][t][h][:],  fp32,
 * for blocks first_block <= j < first_block + n_blocks that exist in sequence b
 * (n_blocks = -1: all blocks).  The last block of a sequence averages the tokens it has.
 * Rows of blocks that do not exist are left untouched.
 */
int svf_block_reps(const svf_shape_t* shape, const void* K, const int32_t* block_table,
                   const int32_t* seq_lens, int32_t first_block, int32_t n_blocks,
                   float* reps, void* stream);

/*
 * Block scores and the shared block set (Sec. 3.1, Eq. 5 and the top-N rule; Sec. 2.2: the
 * first draft token retrieves for all draft tokens).
 *   q0[b][h][:]  = mean over the Hq/Hkv query heads of KV head h of q[b][0][.][:]
 *   s[b][h][j]   = q0[b][h] . reps[b][h][j]                       (fp32, unscaled)
 *   kept blocks  = first n_sink and last n_local blocks, then the highest scores until
 *                  min(k_blocks, nb_b) blocks are kept; equal scores: lowest block id first.
 * Writes sel_idx (ascending, -1 padded), sel_cnt and, if scores_or_null is given, s.
 * (Without the scores, shapes with a gather list take a single launch; the blocks are the same.)
 */
int svf_score_select(const svf_shape_t* shape, const void* q, const float* reps,
                     const int32_t* seq_lens, int32_t* sel_idx, int32_t* sel_cnt,
                     float* scores_or_null, void* ws, size_t ws_bytes, void* stream);

/*
 * Verification attention (Sec. 3.1 / 3.3: only the retrieved blocks participate): every
 * draft query (b, i, j) attends to all tokens of the blocks sel_idx[b][j / G][0..sel_cnt)
 * that lie below seq_lens[b], and to the drafts t allowed by its mask, under one softmax
 * with scale sm_scale; out = sum of softmax weights times values.  lse_or_null is optional.
 * A query row that sees no key at all (no selected token and a draft mask without its own bit)
 * gets out = 0 and lse = -inf.
 * Arithmetic of the bf16 path (d = 128): products of bf16 inputs accumulate in fp32; softmax
 * weights are rounded to bf16 before they multiply V; when the selected tokens are cut into
 * several splits (long budgets), each split's output, normalised by its own denominator, is
 * rounded to bf16 once before the splits are summed in fp32 in split order.  The result is the
 * same bits from call to call and does not depend on how the workgroups happen to be scheduled.
 * The fp32 path and other head dimensions keep everything in fp32.
 */
int svf_verify_attn(const svf_shape_t* shape, const void* q, const void* K, const void* V,
                    const int32_t* block_table, const int32_t* seq_lens,
                    const void* k_draft, const void* v_draft, const uint64_t* draft_mask_or_null,
                    const int32_t* sel_idx, const int32_t* sel_cnt,
                    void* out, float* lse_or_null, void* ws, size_t ws_bytes, void* stream);

/*
 * svf_verify_attn for callers that cannot allocate (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): the same result, bit for bit, with the workspace in a
 * static device array of svf_static_workspace_bytes() bytes (16 MiB) that every GPU the library
 * runs on holds until the process ends.  The call allocates and frees nothing and does not
 * synchronise; it enqueues one small fill kernel ahead of the attention kernels (the array keeps
 * the last call's contents, of whatever shape).  A shape whose svf_workspace_bytes exceeds the
 * array: SVF_ERR_WORKSPACE, nothing enqueued.  All calls on one GPU share that GPU's array:
 * calls that overlap in time on one GPU (different streams, different threads) race; order them.
 */
size_t svf_static_workspace_bytes(void);
int svf_verify_attn_static_ws(const svf_shape_t* shape, const void* q, const void* K, const void* V,
                              const int32_t* block_table, const int32_t* seq_lens,
                              const void* k_draft, const void* v_draft, const uint64_t* draft_mask_or_null,
                              const int32_t* sel_idx, const int32_t* sel_cnt,
                              void* out, float* lse_or_null, void* stream);

/*
 * One layer of one verification step with inter-layer retrieval reuse (Sec. 3.3, Eq. 9).
 * mode SVF_STEP_ANCHOR (anchor layer): svf_score_select into sel_idx / sel_cnt, then
 *   svf_verify_attn.  The call also leaves in `ws` a gather list: where in the cache pools the
 *   selected rows of this block_table / seq_lens / layout sit.
 * mode SVF_STEP_REUSE: svf_verify_attn with the sel_idx / sel_cnt the caller kept from the
 *   nearest preceding anchor layer (reps may then be NULL).  KV head h reuses KV head h's set.
 *   Nothing but the arguments is relied on.
 * mode SVF_STEP_REUSE_GATHER: the same result, faster: the kernel reads the anchor call's gather
 *   list instead of walking sel_idx and block_table again.  The caller promises that `ws`,
 *   sel_idx, sel_cnt, block_table, seq_lens and every field of `shape` are those of the last
 *   SVF_STEP_ANCHOR call on this `ws`, contents unchanged (K, V, q, the drafts and the outputs
 *   may differ: the layers of one verification step share their page table).  A broken promise
 *   gives attention over the anchor call's rows, never an access outside the pools it was built
 *   for.  Shapes that have no gather list (anything but bf16 with d = 128 and block and page
 *   sizes that are multiples of four, or more than 1024 kept blocks) take the SVF_STEP_REUSE path.
 * Any other mode: SVF_ERR_SHAPE.
 */
#define SVF_STEP_REUSE 0
#define SVF_STEP_ANCHOR 1
#define SVF_STEP_REUSE_GATHER 2
int svf_verify_step(const svf_shape_t* shape, int mode, const void* q, const float* reps,
                    const void* K, const void* V, const int32_t* block_table,
                    const int32_t* seq_lens, const void* k_draft, const void* v_draft,
                    const uint64_t* draft_mask_or_null, int32_t* sel_idx, int32_t* sel_cnt,
                    void* out, float* lse_or_null, void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * Retrieval analytics: the measurements the method's attention design rests on (Sec. 2.2 and
 * Fig. 2: draft tokens of one step retrieve similar blocks; Sec. 3.3, Eq. 7-8: adjacent layers
 * retrieve similar blocks, the least similar layers become anchor layers).  Block sets are bit
 * masks: block j of a (sequence, KV head) is bit j % 64 of word j / 64, svf_mask_words(shape)
 * uint64 words per mask, bits of blocks that do not exist are zero.  Counts come back as exact
 * integers; the caller forms the ratios.
 * ------------------------------------------------------------------------------------------ */

/* ceil(ceil(max_seq_len / block_size) / 64); 0 if the shape is invalid. */
int32_t svf_mask_words(const svf_shape_t* shape);

/* Bytes of device workspace svf_select_per_draft needs (multiple of 256; 0 if invalid). */
size_t svf_analytics_workspace_bytes(const svf_shape_t* shape);

/*
 * The blocks every draft token would retrieve with its own query (Sec. 2.2): the rule of
 * svf_score_select (Eq. 5 score, first n_sink / last n_local blocks kept, top-N, lowest id on
 * ties) applied to each of the gamma draft tokens' group-mean queries.  Draft 0's set is the one
 * svf_score_select returns, bit for bit.
 *   masks           uint64 [B][Hkv][gamma][svf_mask_words]   (device, out)
 *   scores_or_null  fp32   [B][gamma][Hkv][nb_max]           (device, out, optional)
 *   ws / ws_bytes   device scratch of svf_analytics_workspace_bytes (256-byte aligned)
 */
int svf_select_per_draft(const svf_shape_t* shape, const void* q, const float* reps,
                         const int32_t* seq_lens, uint64_t* masks, float* scores_or_null,
                         void* ws, size_t ws_bytes, void* stream);

/* masks [B][Hkv][svf_mask_words] (device, out) from the index lists svf_score_select writes. */
int svf_masks_from_selection(const svf_shape_t* shape, const int32_t* sel_idx,
                             const int32_t* sel_cnt, uint64_t* masks, void* stream);

/*
 * Overlap of the blocks retrieved by pairs of draft tokens, by positional distance (Sec. 2.2,
 * Fig. 2).  pos[i] (device int32 [gamma]) is draft i's position (its depth in the draft tree;
 * several drafts may share one).  For every sequence b and distance d < n_dist (1..64):
 *   inter[b][d] = sum over KV heads and pairs i < i' with |pos[i] - pos[i']| = d of |M_i & M_i'|
 * (device uint64 [B][n_dist], overwritten).  The caller divides by (kept blocks of b) x Hkv x
 * (pairs at distance d) to get the figure's ratio.  Needs svf_mask_words <= 64.
 */
int svf_overlap_by_distance(const svf_shape_t* shape, const uint64_t* masks, const int32_t* pos,
                            int32_t n_dist, uint64_t* inter, void* stream);

/*
 * Eq. 7 for one calibration sample: masks_by_layer is uint64 [n_layers][B][Hkv][svf_mask_words]
 * (device), layer l's retrieved blocks over all candidate blocks of the sample; inter_union is
 * uint64 [n_layers][2] (device, overwritten): |M_l & M_{l-1}| and |M_l | M_{l-1}|; layer 0 gets
 * (0, 0): its similarity is 0 by definition.
 */
int svf_jaccard_adjacent(const svf_shape_t* shape, const uint64_t* masks_by_layer, int32_t n_layers,
                         uint64_t* inter_union, void* stream);

/*
 * Eq. 8 (host): anchors[0..K) = the K layers with the largest 1 - J[l], ascending; equal values
 * go to the lower layer.  J is a host array of n_layers similarities (J[0] = 0 by definition, so
 * the first layer is always chosen).  SVF_ERR_NULL / SVF_ERR_SHAPE (K outside 1..n_layers, a J
 * outside [0, 1] or not a number).
 */
int svf_topk_anchors(const double* J, int32_t n_layers, int32_t K, int32_t* anchors);

/* ------------------------------------------------------------------------------------------
 * Retrieval variants: the same pipeline (block summaries -> block scores -> kept blocks ->
 * svf_verify_attn) with one of its rules exchanged.  Sec. 3.1 takes its block retrieval from
 * Quest, whose block summary is the per-channel minimum and maximum of the keys; Eq. 6 counts the
 * budget over all H KV heads of a sequence.  The default of every field is the rule of
 * svf_block_reps / svf_score_select, and with all defaults the two calls below ARE those.
 * ------------------------------------------------------------------------------------------ */
#define SVF_SUMMARY_MEAN 0    /* the mean key (block term of Eq. 5): summaries [B][Hkv][nb_max][d]      */
#define SVF_SUMMARY_MINMAX 1  /* per-channel minimum and maximum: summaries [B][Hkv][nb_max][2][d],
                                 minimum row first; score of a query head =
                                 sum over channels c of max(q_c * min_c, q_c * max_c), an upper bound
                                 of q . k over the keys of the block                                    */
#define SVF_GROUP_MEAN 0      /* score of a KV head = mean of its Hq/Hkv query heads' scores            */
#define SVF_GROUP_MAX 1       /* ... = their maximum                                                    */
#define SVF_BUDGET_PER_HEAD 0 /* every (sequence, KV head) keeps min(k_blocks, nb) blocks               */
#define SVF_BUDGET_GLOBAL 1   /* every sequence keeps min(n_total, Hkv * nb) (KV head, block) pairs,
                                 the highest scores over all its KV heads (Eq. 6 with its factor H);
                                 equal scores: lower KV head, then lower block.  n_sink / n_local
                                 blocks are kept in every KV head and count inside n_total.  sel_cnt
                                 then differs per KV head; shape.k_blocks is the row length of
                                 sel_idx and must be >= min(nb_max, n_total).                           */
typedef struct svf_retrieval {
  int32_t summary;        /* SVF_SUMMARY_*                                                        */
  int32_t summary_dtype;  /* element type of the summaries: SVF_F32, or SVF_BF16 (rounded to nearest
                             even from the fp32 value; half the bytes for the scores to read)     */
  int32_t group_rule;     /* SVF_GROUP_*                                                          */
  int32_t budget_rule;    /* SVF_BUDGET_*                                                         */
  int32_t n_total;        /* SVF_BUDGET_GLOBAL only: pairs kept per sequence, >= Hkv * (n_sink + n_local) */
} svf_retrieval_t;

/*
 * Block summaries of blocks first_block .. first_block + n_blocks (as svf_block_reps: -1 = all,
 * a partial last block summarises the tokens it has, rows of blocks that do not exist are left
 * untouched).  `retrieval` is a HOST pointer; `summaries` has the layout and element type it names.
 */
int svf_block_summaries(const svf_shape_t* shape, const svf_retrieval_t* retrieval, const void* K,
                        const int32_t* block_table, const int32_t* seq_lens, int32_t first_block,
                        int32_t n_blocks, void* summaries, void* stream);

/*
 * Scores of the first draft token's query heads against the summaries, combined per KV head
 * (group_rule), then the kept blocks (budget_rule), written as svf_score_select writes them
 * (sel_idx ascending per KV head, -1 padded; scores_or_null fp32 [B][Hkv][nb_max]).  The result
 * feeds svf_verify_attn with the same shape.  SVF_ERR_BUDGET: n_total or k_blocks too small for
 * the rule; SVF_ERR_SHAPE: an unknown rule.  `ws` is the workspace of svf_workspace_bytes(shape).
 */
int svf_retrieve(const svf_shape_t* shape, const svf_retrieval_t* retrieval, const void* q,
                 const void* summaries, const int32_t* seq_lens, int32_t* sel_idx, int32_t* sel_cnt,
                 float* scores_or_null, void* ws, size_t ws_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SVF_H_ */
