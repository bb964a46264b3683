// Retrieval variants: the block scores and the kept blocks with one rule of Sec. 3.1 exchanged.
//
//   scores:  the first draft token's score of every block PER QUERY HEAD, against the mean key
//            (Eq. 5) or against the per-channel minimum / maximum of the block's keys (Quest's
//            summary, which Sec. 3.1 starts from:  sum_c max(q_c min_c, q_c max_c) >= q . k for
//            every key of the block); the query heads of a KV head are combined by their mean or
//            their maximum.  Summaries are fp32 or bf16.  Same lane mapping as the main scores
//            kernel (eight lanes own a block, 16 channels each, fixed order of the arithmetic);
//            HBM-bound on the summaries, which are read once whatever the number of query heads.
//   select:  top-N over all (KV head, block) pairs of a sequence (Eq. 6 counts its budget over
//            the H KV heads): one workgroup per sequence, the radix select of the per-head kernel
//            over Hkv * nb keys, then an ordered sweep head by head that writes each head's kept
//            blocks ascending and its count.
#include <hip/hip_bf16.h>

#include "svf_device.h"

namespace svf {

namespace {

constexpr int kThreads = 256;
constexpr int kPasses = 4;             // blocks per lane group
constexpr int kHeadsPerRound = 8;      // query heads staged in LDS at a time

__device__ __forceinline__ float4 load4(const float* p) { return *reinterpret_cast<const float4*>(p); }
__device__ __forceinline__ float4 load4(const __hip_bfloat16* p) {
  const uint2 w = *reinterpret_cast<const uint2*>(p);
  return make_float4(__uint_as_float(w.x << 16), __uint_as_float(w.x & 0xffff0000u), __uint_as_float(w.y << 16),
                     __uint_as_float(w.y & 0xffff0000u));
}

// sum over this lane's channels of max(q * min, q * max), then over the lane group
template <int NCH>
__device__ __forceinline__ float bound_score(const float4 (&mn)[NCH], const float4 (&mx)[NCH], const float4 (&q)[NCH]) {
  float acc = 0.f;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    acc += fmaxf(q[i].x * mn[i].x, q[i].x * mx[i].x);
    acc += fmaxf(q[i].y * mn[i].y, q[i].y * mx[i].y);
    acc += fmaxf(q[i].z * mn[i].z, q[i].z * mx[i].z);
    acc += fmaxf(q[i].w * mn[i].w, q[i].w * mx[i].w);
  }
  return lane8_sum(acc);
}

// grid: (ceil(nb_max / (kPasses * blocks per pass)), Hkv, B)
template <typename QT, typename RT, int D, bool MINMAX, bool GMAX>
__global__ __launch_bounds__(kThreads) void variant_scores_kernel(VariantParams p) {
  constexpr int LPB = kScoreLanes;
  constexpr int NCH = D / (4 * LPB);
  constexpr int BPW = kThreads / LPB;
  constexpr int ROWS = MINMAX ? 2 : 1;
  __shared__ __attribute__((aligned(16))) float qs[kHeadsPerRound][D];

  const int b = blockIdx.z, h = blockIdx.y;
  const int G = p.Hq / p.Hkv;
  const int tid = threadIdx.x, sub = tid % LPB;
  float4 r[kPasses][ROWS][NCH];
  int jj[kPasses];
#pragma unroll
  for (int u = 0; u < kPasses; ++u) {
    const int j = (blockIdx.x * kPasses + u) * BPW + tid / LPB;
    jj[u] = j;
    const int jc = j < p.nb_max ? j : p.nb_max - 1;
    const RT* row = static_cast<const RT*>(p.summaries) + ((((int64_t)b * p.Hkv + h) * p.nb_max + jc) * ROWS) * D + sub * 4;
#pragma unroll
    for (int w = 0; w < ROWS; ++w)
#pragma unroll
      for (int i = 0; i < NCH; ++i) r[u][w][i] = load4(row + w * D + i * 4 * LPB);
  }
  const int L = clamped_len(p.seq_lens, b, p.max_seq_len);
  const int nb = (L + p.block_size - 1) / p.block_size;

  float acc[kPasses];
#pragma unroll
  for (int u = 0; u < kPasses; ++u) acc[u] = GMAX ? -__builtin_inff() : 0.f;
  const QT* q0 = static_cast<const QT*>(p.q) + ((int64_t)b * p.gamma * p.Hq + (int64_t)h * G) * D;
  for (int g0 = 0; g0 < G; g0 += kHeadsPerRound) {
    const int ng = min(kHeadsPerRound, G - g0);
    if (g0 > 0) __syncthreads();                          // the round before has been read
    for (int idx = tid; idx < ng * D; idx += kThreads) (&qs[0][0])[idx] = query_value(q0[(int64_t)g0 * D + idx]);
    __syncthreads();
    for (int g = 0; g < ng; ++g) {
      float4 qv[NCH];
#pragma unroll
      for (int i = 0; i < NCH; ++i) qv[i] = *reinterpret_cast<const float4*>(&qs[g][sub * 4 + i * 4 * LPB]);
#pragma unroll
      for (int u = 0; u < kPasses; ++u) {
        float s;
        if constexpr (MINMAX) s = bound_score<NCH>(r[u][0], r[u][1], qv);
        else s = block_score<NCH>(r[u][0], qv);
        acc[u] = GMAX ? fmaxf(acc[u], s) : acc[u] + s;
      }
    }
  }
#pragma unroll
  for (int u = 0; u < kPasses; ++u) {
    const float v = GMAX ? acc[u] : acc[u] / (float)G;
    if (sub == 0 && jj[u] < p.nb_max)
      p.scores[((int64_t)b * p.Hkv + h) * p.nb_max + jj[u]] = jj[u] < nb ? v + 0.0f : 0.0f;
  }
}

template <typename QT, typename RT, int D>
void launch_scores_for(const VariantParams& p, dim3 grid, hipStream_t st) {
  if (p.minmax) {
    if (p.group_max) hipLaunchKernelGGL((variant_scores_kernel<QT, RT, D, true, true>), grid, dim3(kThreads), 0, st, p);
    else hipLaunchKernelGGL((variant_scores_kernel<QT, RT, D, true, false>), grid, dim3(kThreads), 0, st, p);
  } else {
    if (p.group_max) hipLaunchKernelGGL((variant_scores_kernel<QT, RT, D, false, true>), grid, dim3(kThreads), 0, st, p);
    else hipLaunchKernelGGL((variant_scores_kernel<QT, RT, D, false, false>), grid, dim3(kThreads), 0, st, p);
  }
}
template <typename QT, typename RT>
void launch_scores_d(const VariantParams& p, dim3 grid, hipStream_t st) {
  if (p.d == 64) launch_scores_for<QT, RT, 64>(p, grid, st);
  else launch_scores_for<QT, RT, 128>(p, grid, st);
}

// ---- top-N over the (KV head, block) pairs of a sequence ---------------------------------------
constexpr int kGThreads = 1024;
constexpr int kGWaves = kGThreads / 64;
constexpr int kRegHeads = 8;

// grid: (B)
__global__ __launch_bounds__(kGThreads) void select_global_kernel(VariantParams p) {
  __shared__ uint32_t hist[256];
  __shared__ uint32_t sh_prefix, sh_need;
  __shared__ uint32_t wave_eq[kGWaves], wave_sel[kGWaves];
  __shared__ uint32_t base_eq, base_sel;

  const int b = blockIdx.x;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int L = clamped_len(p.seq_lens, b, p.max_seq_len);
  const int nb = (L + p.block_size - 1) / p.block_size;
  const int64_t total = (int64_t)p.Hkv * nb;
  const uint32_t keep_n = (uint32_t)(total < p.n_total ? total : p.n_total);
  const float* sc = p.scores + (int64_t)b * p.Hkv * p.nb_max;
  int32_t* out = p.sel_idx + (int64_t)b * p.Hkv * p.k_blocks;

  auto key_of = [&](int h, int j) -> uint32_t {
    if (j < p.n_sink || j >= nb - p.n_local) return 0xffffffffu;
    return score_key(sc[(int64_t)h * p.nb_max + j]);
  };

  // Up to kRegHeads KV heads of at most kGThreads blocks: thread t keeps the keys of block t of
  // every head in registers; larger problems read the scores again in every pass.
  const bool in_regs = p.Hkv <= kRegHeads && nb <= kGThreads;
  uint32_t kreg[kRegHeads];
#pragma unroll
  for (int h = 0; h < kRegHeads; ++h) kreg[h] = (in_regs && h < p.Hkv && tid < nb) ? key_of(h, tid) : 0u;

  // radix select: key of the keep_n-th largest pair
  if (tid == 0) { sh_prefix = 0; sh_need = keep_n; }
  for (int shift = 24; shift >= 0; shift -= 8) {
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    const uint32_t prefix = sh_prefix;
    const uint32_t need = sh_need;
    const uint32_t hi_mask = shift == 24 ? 0u : (0xffffffffu << (shift + 8));
    if (in_regs) {
#pragma unroll
      for (int h = 0; h < kRegHeads; ++h)
        if (h < p.Hkv && tid < nb && (kreg[h] & hi_mask) == prefix) atomicAdd(&hist[(kreg[h] >> shift) & 0xff], 1u);
    } else {
      for (int h = 0; h < p.Hkv; ++h)
        for (int j = tid; j < nb; j += kGThreads) {
          const uint32_t k = key_of(h, j);
          if ((k & hi_mask) == prefix) atomicAdd(&hist[(k >> shift) & 0xff], 1u);
        }
    }
    __syncthreads();
    // thread t < 256 looks at bin 255 - t: the inclusive prefix sum over those threads counts the
    // keys in this bin and all higher ones; exactly one thread sees the count cross `need`
    uint32_t hcount = 0, incl = 0;
    if (tid < 256) {                                     // whole wavefronts
      hcount = hist[255 - tid];
      incl = wave_inclusive_sum(hcount);
      if (lane == 63) wave_eq[wave] = incl;
    }
    __syncthreads();
    if (tid < 256) {
      for (int w = 0; w < wave; ++w) incl += wave_eq[w];
      const uint32_t above = incl - hcount;
      if (incl >= need && above < need) {
        sh_need = need - above;                          // (every thread read sh_need before the last barrier)
        sh_prefix = prefix | ((uint32_t)(255 - tid) << shift);
      }
    }
    __syncthreads();
  }
  const uint32_t tau = sh_prefix;            // key of the weakest kept pair
  const uint32_t need_eq = sh_need;          // pairs equal to tau that are kept (lowest head, then block, first)

  // ordered sweep, head by head: a head's kept blocks come out ascending, pairs equal to tau are
  // kept in (head, block) order until need_eq of them are
  if (tid == 0) base_eq = 0;
  auto sweep_head = [&](int h, auto key_at) {
    if (tid == 0) base_sel = 0;
    __syncthreads();
    for (int j0 = 0; j0 < nb; j0 += kGThreads) {
      const int j = j0 + tid;
      const uint32_t k = j < nb ? key_at(j) : 0u;
      const bool is_eq = keep_n > 0 && j < nb && k == tau;
      const bool is_gt = keep_n > 0 && j < nb && k > tau;
      const uint64_t m_eq = __ballot(is_eq);
      const uint64_t m_gt = __ballot(is_gt);
      if (lane == 0) { wave_eq[wave] = (uint32_t)__popcll(m_eq); wave_sel[wave] = (uint32_t)__popcll(m_gt); }
      __syncthreads();
      const uint64_t below = (1ull << lane) - 1ull;
      uint32_t eq_before = base_eq + (uint32_t)__popcll(m_eq & below), gt_before = (uint32_t)__popcll(m_gt & below);
      uint32_t eq_all = base_eq;
      for (int w = 0; w < kGWaves; ++w) {
        if (w < wave) { eq_before += wave_eq[w]; gt_before += wave_sel[w]; }
        eq_all += wave_eq[w];
      }
      // position = kept pairs in front: all larger ones, and the equal ones still inside need_eq
      const uint32_t eq_kept_before = min(eq_before, need_eq) - min(base_eq, need_eq);
      const bool keep = is_gt || (is_eq && eq_before < need_eq);
      const uint32_t pos = base_sel + gt_before + eq_kept_before;
      if (keep && pos < (uint32_t)p.k_blocks) out[(int64_t)h * p.k_blocks + pos] = j;
      __syncthreads();                                   // the per-wavefront counts have been read
      if (tid == 0) {
        uint32_t gt_all = 0;
        for (int w = 0; w < kGWaves; ++w) gt_all += wave_sel[w];
        base_sel += gt_all + (min(eq_all, need_eq) - min(base_eq, need_eq));
        base_eq = eq_all;
      }
      __syncthreads();
    }
    const int cnt = min((int)base_sel, p.k_blocks);
    for (int i = cnt + tid; i < p.k_blocks; i += kGThreads) out[(int64_t)h * p.k_blocks + i] = -1;
    if (tid == 0) p.sel_cnt[(int64_t)b * p.Hkv + h] = cnt;
    __syncthreads();                                     // base_sel has been read before the next head resets it
  };
  if (in_regs) {
#pragma unroll
    for (int h = 0; h < kRegHeads; ++h)
      if (h < p.Hkv) sweep_head(h, [&](int) { return kreg[h]; });
  } else {
    for (int h = 0; h < p.Hkv; ++h) sweep_head(h, [&](int j) { return key_of(h, j); });
  }
}

}  // namespace

hipError_t launch_variant_scores(const VariantParams& p, int dtype, hipStream_t st) {
  const int bpw = kPasses * (kThreads / kScoreLanes);
  dim3 grid((p.nb_max + bpw - 1) / bpw, p.Hkv, p.B);
  if (dtype == SVF_F32) {
    if (p.summary_bf16) launch_scores_d<float, __hip_bfloat16>(p, grid, st);
    else launch_scores_d<float, float>(p, grid, st);
  } else {
    if (p.summary_bf16) launch_scores_d<__hip_bfloat16, __hip_bfloat16>(p, grid, st);
    else launch_scores_d<__hip_bfloat16, float>(p, grid, st);
  }
  return hipGetLastError();
}

hipError_t launch_select_global(const VariantParams& p, hipStream_t st) {
  hipLaunchKernelGGL(select_global_kernel, dim3(p.B), dim3(kGThreads), 0, st, p);
  return hipGetLastError();
}

}  // namespace svf
