// Block scores and the shared top-N block set (Sec. 3.1, Eq. 5 and the selection rule;
// Sec. 2.2: the first draft token's query retrieves for every draft token).
//
// Two kernels.
//   scores:  wide, HBM-bound pass over the fp32 representatives.  A group of d/4 lanes owns
//            one block: float4 loads, fp32 dot with the group-mean first-draft query,
//            reduction inside the lane group.
//   select:  one workgroup per (sequence, KV head).  Scores become order-preserving 32-bit
//            keys (forced sink/local blocks get the maximum key); a 4-pass radix select over
//            LDS histograms (bins scanned with a wavefront prefix sum) finds the key of the
//            weakest kept block, and a final ascending
//            sweep keeps every block above it plus the lowest-indexed blocks equal to it,
//            using wavefront ballots for the ordered compaction.  Output is ascending.
#include <hip/hip_bf16.h>

#include "svf_device.h"

namespace svf {

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kKeysPerThread = 8;      // selection keys a thread keeps in registers
constexpr int kPasses = 4;              // blocks scored per lane group in the scores kernel

// grid: (ceil(nb_max / (kPasses * blocks per pass)), Hkv, B)
template <typename T, int D>
__global__ __launch_bounds__(kThreads) void block_scores_kernel(SelectParams p) {
  constexpr int LPB = kScoreLanes;           // lanes per block
  constexpr int NCH = D / (4 * LPB);         // 16-byte chunks per lane: sub, sub + 8, ...
  constexpr int BPW = kThreads / LPB;        // blocks per workgroup pass
  __shared__ __attribute__((aligned(16))) float q0[D];

  const int b = blockIdx.z, h = blockIdx.y;
  const int G = p.Hq / p.Hkv;
  const int sub = threadIdx.x % LPB;

  // All loads go out before anything waits, so that the query and the representatives share one
  // memory round trip.  First draft token's query: channel threadIdx.x mod D of the group's heads
  // (loaded by every thread, used by the first D); representative rows unconditionally (rows past
  // the sequence's last block exist in the buffer; their result is discarded).
  const T* qch = static_cast<const T*>(p.q) + ((int64_t)b * p.gamma * p.Hq + (int64_t)h * G) * D + threadIdx.x % D;
  const QueryHeads<T> qh = load_query_heads<T>(qch, G, D);
  float4 r[kPasses][NCH];
  int jj[kPasses];
#pragma unroll
  for (int u = 0; u < kPasses; ++u) {
    const int j = (blockIdx.x * kPasses + u) * BPW + threadIdx.x / LPB;
    jj[u] = j;
    const int jc = j < p.nb_max ? j : p.nb_max - 1;
    const float* row = p.reps + (((int64_t)b * p.Hkv + h) * p.nb_max + jc) * D + sub * 4;
#pragma unroll
    for (int i = 0; i < NCH; ++i) r[u][i] = *reinterpret_cast<const float4*>(row + i * 4 * LPB);
  }

  // averaged over the query heads of this KV head
  if (threadIdx.x < D) q0[threadIdx.x] = mean_query_channel<T>(qh, qch, G, D);
  const int L = clamped_len(p.seq_lens, b, p.max_seq_len);
  const int nb = (L + p.block_size - 1) / p.block_size;
  __syncthreads();

  float4 qv[NCH];
#pragma unroll
  for (int i = 0; i < NCH; ++i) qv[i] = *reinterpret_cast<const float4*>(q0 + sub * 4 + i * 4 * LPB);
#pragma unroll
  for (int u = 0; u < kPasses; ++u) {
    const float v = block_score<NCH>(r[u], qv);
    if (sub == 0 && jj[u] < p.nb_max)
      p.scores[((int64_t)b * p.Hkv + h) * p.nb_max + jj[u]] = jj[u] < nb ? v + 0.0f : 0.0f;
  }
}

// Scores of every draft token's query (Sec. 2.2: retrieval "based on their respective query
// values"), one pass over the representatives: the rows a thread holds are scored against the
// gamma mean queries in LDS, with the arithmetic of the kernel above (query 0 gives the same bits).
// grid: (ceil(nb_max / (kPasses * blocks per pass)) * ceil(gamma / kDraftsPerGroup), Hkv, B): a
// workgroup scores its rows against one group of drafts (the rows' other readers find them in L2);
// scores [B][gamma][Hkv][nb_max]
constexpr int kDraftsPerGroup = 8;
template <typename T, int D>
__global__ __launch_bounds__(kThreads) void block_scores_all_kernel(SelectParams p) {
  constexpr int LPB = kScoreLanes;
  constexpr int NCH = D / (4 * LPB);
  constexpr int BPW = kThreads / LPB;
  __shared__ __attribute__((aligned(16))) float qs[kDraftsPerGroup][D];

  const int b = blockIdx.z, h = blockIdx.y;
  const int n_chunks = (p.nb_max + kPasses * BPW - 1) / (kPasses * BPW);
  const int chunk = blockIdx.x % n_chunks;
  const int i0 = (blockIdx.x / n_chunks) * kDraftsPerGroup;      // first draft of this workgroup's group
  const int n_i = min(kDraftsPerGroup, p.gamma - i0);
  const int G = p.Hq / p.Hkv;
  const int sub = threadIdx.x % LPB;
  float4 r[kPasses][NCH];
  int jj[kPasses];
#pragma unroll
  for (int u = 0; u < kPasses; ++u) {
    const int j = (chunk * kPasses + u) * BPW + threadIdx.x / LPB;
    jj[u] = j;
    const int jc = j < p.nb_max ? j : p.nb_max - 1;
    const float* row = p.reps + (((int64_t)b * p.Hkv + h) * p.nb_max + jc) * D + sub * 4;
#pragma unroll
    for (int i = 0; i < NCH; ++i) r[u][i] = *reinterpret_cast<const float4*>(row + i * 4 * LPB);
  }
  for (int idx = threadIdx.x; idx < n_i * D; idx += kThreads) {
    const int i = idx / D, c = idx - i * D;
    const T* qch = static_cast<const T*>(p.q) + (((int64_t)b * p.gamma + i0 + i) * p.Hq + (int64_t)h * G) * D + c;
    qs[i][c] = mean_query_channel<T>(load_query_heads<T>(qch, G, D), qch, G, D);
  }
  const int L = clamped_len(p.seq_lens, b, p.max_seq_len);
  const int nb = (L + p.block_size - 1) / p.block_size;
  __syncthreads();
  for (int i = 0; i < n_i; ++i) {
    float4 qv[NCH];
#pragma unroll
    for (int c = 0; c < NCH; ++c) qv[c] = *reinterpret_cast<const float4*>(&qs[i][sub * 4 + c * 4 * LPB]);
#pragma unroll
    for (int u = 0; u < kPasses; ++u) {
      const float v = block_score<NCH>(r[u], qv);
      if (sub == 0 && jj[u] < p.nb_max)
        p.scores[(((int64_t)b * p.gamma + i0 + i) * p.Hkv + h) * p.nb_max + jj[u]] = jj[u] < nb ? v + 0.0f : 0.0f;
    }
  }
}

// grid: (Hkv, B * nq)
__global__ __launch_bounds__(kThreads) void select_kernel(SelectParams p) {
  __shared__ uint32_t hist[256];
  __shared__ uint32_t sh_prefix, sh_need;
  __shared__ uint32_t wave_eq[kWaves], wave_sel[kWaves];
  __shared__ uint32_t base_eq, base_sel;
  __shared__ int32_t sh_sel[kMaxGatherBlocks];     // kept block ids, for the gather list

  const int bq = blockIdx.y, h = blockIdx.x;             // bq = b * nq + query
  const int b = bq / p.nq;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int L = clamped_len(p.seq_lens, b, p.max_seq_len);
  const int nb = (L + p.block_size - 1) / p.block_size;
  const int cnt = min(p.k_blocks, nb);
  const float* sc = p.scores + ((int64_t)bq * p.Hkv + h) * p.nb_max;
  int32_t* out = p.sel_idx ? p.sel_idx + ((int64_t)bq * p.Hkv + h) * p.k_blocks : nullptr;
  // bit masks: a wavefront's ballot over 64 consecutive blocks is one word
  uint64_t* mask = p.masks ? p.masks + (((int64_t)b * p.Hkv + h) * p.nq + (bq - b * p.nq)) * p.mask_words : nullptr;

  auto key_of = [&](int j) -> uint32_t {
    if (j < p.n_sink || j >= nb - p.n_local) return 0xffffffffu;
    return score_key(sc[j]);
  };

  // keys of the first kKeysPerThread * 256 blocks stay in registers for all passes
  uint32_t kreg[kKeysPerThread];
#pragma unroll
  for (int i = 0; i < kKeysPerThread; ++i) {
    const int j = tid + i * kThreads;
    kreg[i] = j < nb ? key_of(j) : 0u;
  }

  // radix select: key of the cnt-th largest element
  if (tid == 0) { sh_prefix = 0; sh_need = (uint32_t)cnt; }
  for (int shift = 24; shift >= 0; shift -= 8) {
    hist[tid] = 0;
    __syncthreads();
    const uint32_t prefix = sh_prefix;
    const uint32_t hi_mask = shift == 24 ? 0u : (0xffffffffu << (shift + 8));
#pragma unroll
    for (int i = 0; i < kKeysPerThread; ++i)
      if (tid + i * kThreads < nb && (kreg[i] & hi_mask) == prefix) atomicAdd(&hist[(kreg[i] >> shift) & 0xff], 1u);
    for (int j = tid + kKeysPerThread * kThreads; j < nb; j += kThreads) {
      const uint32_t k = key_of(j);
      if ((k & hi_mask) == prefix) atomicAdd(&hist[(k >> shift) & 0xff], 1u);
    }
    __syncthreads();
    // Thread t looks at bin 255 - t, so an inclusive prefix sum over the threads counts the keys
    // in this bin and all higher ones; exactly one thread sees the running count cross `need`.
    {
      const uint32_t need = sh_need;
      const uint32_t hcount = hist[255 - tid];
      uint32_t incl = wave_inclusive_sum(hcount);
      if (lane == 63) wave_eq[wave] = incl;
      __syncthreads();
      for (int w = 0; w < wave; ++w) incl += wave_eq[w];
      const uint32_t above = incl - hcount;        // keys in strictly higher bins
      __syncthreads();                             // everyone has read sh_need / wave_eq
      if (incl >= need && above < need) {
        sh_need = need - above;                    // how many are still wanted from inside this bin
        sh_prefix = prefix | ((uint32_t)(255 - tid) << shift);
      }
    }
    __syncthreads();
  }
  const uint32_t tau = sh_prefix;           // key of the weakest kept block
  const uint32_t need_eq = sh_need;         // blocks equal to tau that are kept (lowest ids first)

  if (tid == 0) { base_eq = 0; base_sel = 0; }
  __syncthreads();
  for (int j0 = 0; j0 < nb; j0 += kThreads) {
    const int j = j0 + tid;
    const uint32_t k = j < nb ? key_of(j) : 0u;
    const bool is_eq = j < nb && k == tau;
    const bool is_gt = j < nb && k > tau;
    const uint64_t m_eq = __ballot(is_eq);
    if (lane == 0) wave_eq[wave] = (uint32_t)__popcll(m_eq);
    __syncthreads();
    uint32_t eq_rank = base_eq + (uint32_t)__popcll(m_eq & ((1ull << lane) - 1ull));
    for (int w = 0; w < wave; ++w) eq_rank += wave_eq[w];
    const bool keep = is_gt || (is_eq && eq_rank < need_eq);
    const uint64_t m_sel = __ballot(keep);
    if (lane == 0) wave_sel[wave] = (uint32_t)__popcll(m_sel);
    __syncthreads();
    uint32_t pos = base_sel + (uint32_t)__popcll(m_sel & ((1ull << lane) - 1ull));
    for (int w = 0; w < wave; ++w) pos += wave_sel[w];
    if (keep) {
      if (out) out[pos] = j;
      if (pos < (uint32_t)kMaxGatherBlocks) sh_sel[pos] = j;
    }
    if (mask && lane == 0 && (j0 >> 6) + wave < p.mask_words) mask[(j0 >> 6) + wave] = m_sel;
    __syncthreads();
    if (tid == 0) {
      uint32_t e = 0, s = 0;
      for (int w = 0; w < kWaves; ++w) { e += wave_eq[w]; s += wave_sel[w]; }
      base_eq += e;
      base_sel += s;
    }
    __syncthreads();
  }
  if (out)
    for (int i = cnt + tid; i < p.k_blocks; i += kThreads) out[i] = -1;
  if (tid == 0 && p.sel_cnt) p.sel_cnt[(int64_t)bq * p.Hkv + h] = cnt;
  // mask words past the last block's word group
  if (mask)
    for (int w = ((nb + kThreads - 1) / kThreads) * kWaves + tid; w < p.mask_words; w += kThreads) mask[w] = 0;

  // Gather list: where the K row of every fourth selected-token slot sits in the pool, and how
  // many of its four slots hold a real token.  (The last loop iteration ended with a barrier, so
  // sh_sel is complete; block and page sizes are multiples of four, so the four slots share a
  // block and a page.)
  if (p.gather) {
    uint64_t* gl = p.gather + ((int64_t)b * p.Hkv + h) * p.gather_groups;
    for (int e = tid; e < p.gather_groups; e += kThreads) {
      const int slot0 = 4 * e;
      const int bi = slot0 / p.block_size;
      uint64_t entry = 0;
      if (bi < cnt) {
        const int tok0 = sh_sel[bi] * p.block_size + (slot0 - bi * p.block_size);
        const int nv = min(max(L - tok0, 0), 4);
        if (nv > 0) {
          const int64_t off = (token_offset(p.kv, p.table, b, tok0) + (int64_t)h * p.kv.stride_head) * 2;
          entry = ((uint64_t)off & kGatherOffsetMask) | ((uint64_t)nv << kGatherCountShift);
        }
      }
      gl[e] = entry;
    }
  }
}

}  // namespace

hipError_t launch_score_select(const SelectParams& p, int dtype, hipStream_t st) {
  hipError_t e = launch_scores_only(p, dtype, st);
  if (e != hipSuccess) return e;
  return launch_select_only(p, st);
}

// The scores alone (p.nq = 1: the first draft token's; otherwise every draft token's).
hipError_t launch_scores_only(const SelectParams& p, int dtype, hipStream_t st) {
  const int bpw = kPasses * (kThreads / kScoreLanes);
  dim3 g1((p.nb_max + bpw - 1) / bpw, p.Hkv, p.B);
  if (p.nq > 1) {
    g1.x *= (unsigned)((p.gamma + kDraftsPerGroup - 1) / kDraftsPerGroup);
    if (dtype == SVF_F32) {
      if (p.d == 64) hipLaunchKernelGGL((block_scores_all_kernel<float, 64>), g1, dim3(kThreads), 0, st, p);
      else hipLaunchKernelGGL((block_scores_all_kernel<float, 128>), g1, dim3(kThreads), 0, st, p);
    } else {
      if (p.d == 64) hipLaunchKernelGGL((block_scores_all_kernel<__hip_bfloat16, 64>), g1, dim3(kThreads), 0, st, p);
      else hipLaunchKernelGGL((block_scores_all_kernel<__hip_bfloat16, 128>), g1, dim3(kThreads), 0, st, p);
    }
  } else if (dtype == SVF_F32) {
    if (p.d == 64) hipLaunchKernelGGL((block_scores_kernel<float, 64>), g1, dim3(kThreads), 0, st, p);
    else hipLaunchKernelGGL((block_scores_kernel<float, 128>), g1, dim3(kThreads), 0, st, p);
  } else {
    if (p.d == 64) hipLaunchKernelGGL((block_scores_kernel<__hip_bfloat16, 64>), g1, dim3(kThreads), 0, st, p);
    else hipLaunchKernelGGL((block_scores_kernel<__hip_bfloat16, 128>), g1, dim3(kThreads), 0, st, p);
  }
  return hipGetLastError();
}

// The selection alone, over scores that are already in p.scores.
hipError_t launch_select_only(const SelectParams& p, hipStream_t st) {
  hipLaunchKernelGGL(select_kernel, dim3(p.Hkv, p.B * p.nq), dim3(kThreads), 0, st, p);
  return hipGetLastError();
}

}  // namespace svf
