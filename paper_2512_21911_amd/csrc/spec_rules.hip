// Expert skipping of the sparse mixture of experts (Sec. 3.5, Eq. 15-16) and acceptance /
// resampling of the draft tokens (Sec. 2.1, Eq. 2-3): small, latency-bound kernels.
//
//   moe kernels   32 lanes per token, lane j holds the weight of the token's j-th expert.  A
//                 lane's rank (weights below it, equal weights by position) comes from k shuffles;
//                 the weights are put in rank order in LDS and every lane adds its prefix
//                 sequentially in ascending order (the order the sums are defined in).
//   median        one workgroup per skip size: 4-pass radix select over the tokens' ratios
//                 (positive floats order like their bit patterns), twice when T is even.
//   accept        one workgroup per sequence: the gamma acceptance tests in one wavefront, then,
//                 if a position was rejected, the residual mass of every chunk of 256 consecutive
//                 tokens (a wavefront reads a chunk as one contiguous kilobyte per distribution),
//                 a scan of the chunk sums, and a walk of the one chunk the target falls in.
#include <hip/hip_runtime.h>

#include "svf.h"
#include "svf_rules.h"

namespace {

constexpr int kMoeThreads = 256;
constexpr int kTokPerBlock = kMoeThreads / 32;

// Rank of lane j's weight among the token's k weights and the token's sorted prefix sums.
// Returns this lane's rank; prefix (sum of the weights of rank <= lane) and total through refs.
__device__ __forceinline__ int rank_and_prefix(float w, int j, int k, float* sorted, float& prefix, float& total) {
  int rank = 0;
  const int base = (threadIdx.x & 63) & ~31;             // first lane of this token in the wavefront
  for (int l = 0; l < k; ++l) {
    const float o = __shfl(w, base + l, 64);
    rank += (o < w || (o == w && l < j)) ? 1 : 0;
  }
  if (j < k) sorted[rank] = w;
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  float s = 0.f, tot = 0.f;
  for (int l = 0; l < k; ++l) {
    tot += sorted[l];
    if (l == j) s = tot;
  }
  prefix = s;
  total = tot;
  return rank;
}

// grid: ceil(T / 8); block: 256
__global__ __launch_bounds__(kMoeThreads) void moe_skip_kernel(const float* __restrict__ w, int T, int k, int m,
                                                               const float* __restrict__ beta, int32_t* n_skip,
                                                               uint32_t* keep_mask) {
  __shared__ float sorted[kTokPerBlock][32];
  const int j = threadIdx.x & 31, tl = threadIdx.x >> 5;
  const int t = blockIdx.x * kTokPerBlock + tl;
  const bool live = t < T;
  const float wj = (live && j < k) ? w[(int64_t)t * k + j] : 0.f;
  float prefix, total;
  const int rank = rank_and_prefix(wj, j, k, sorted[tl], prefix, total);
  // lane j looks at skip size i = j + 1
  const bool ok = live && j < m && prefix / total < beta[j];
  const uint64_t b = __ballot(ok);
  const uint32_t mine = (uint32_t)(b >> ((threadIdx.x & 32) ? 32 : 0));
  const int skip = mine ? 32 - __builtin_clz(mine) : 0;
  const uint64_t kb = __ballot(live && j < k && rank >= skip);
  if (live && j == 0) {
    n_skip[t] = skip;
    keep_mask[t] = (uint32_t)(kb >> ((threadIdx.x & 32) ? 32 : 0));
  }
}

// ratios[i-1][t] = r_i of token t; grid: ceil(T / 8)
__global__ __launch_bounds__(kMoeThreads) void moe_ratios_kernel(const float* __restrict__ w, int T, int k,
                                                                 float* ratios) {
  __shared__ float sorted[kTokPerBlock][32];
  const int j = threadIdx.x & 31, tl = threadIdx.x >> 5;
  const int t = blockIdx.x * kTokPerBlock + tl;
  const bool live = t < T;
  const float wj = (live && j < k) ? w[(int64_t)t * k + j] : 0.f;
  float prefix, total;
  rank_and_prefix(wj, j, k, sorted[tl], prefix, total);
  if (live && j < k - 1) ratios[(int64_t)j * T + t] = prefix / total;
}

// The value of 0-based rank `rank` (ascending) among vals[0 .. T): radix select on the bit patterns
// (the values are positive).  Every thread returns the value.
__device__ float select_rank(const float* __restrict__ vals, int T, uint32_t rank, uint32_t* hist, uint32_t* sh) {
  const int tid = threadIdx.x;
  uint32_t prefix = 0, need = rank;                       // `need` smaller keys with this prefix come first
  for (int shift = 24; shift >= 0; shift -= 8) {
    hist[tid] = 0;
    __syncthreads();
    const uint32_t hi_mask = shift == 24 ? 0u : (0xffffffffu << (shift + 8));
    for (int i = tid; i < T; i += 256) {
      const uint32_t key = __float_as_uint(vals[i]);
      if ((key & hi_mask) == prefix) atomicAdd(&hist[(key >> shift) & 0xff], 1u);
    }
    __syncthreads();
    if (tid == 0) {
      uint32_t below = 0;
      int bin = 0;
      for (; bin < 256; ++bin) {
        if (below + hist[bin] > need) break;
        below += hist[bin];
      }
      sh[0] = prefix | ((uint32_t)bin << shift);
      sh[1] = need - below;
    }
    __syncthreads();
    prefix = sh[0];
    need = sh[1];
    __syncthreads();
  }
  return __uint_as_float(prefix);
}

// grid: (k - 1); block: 256
__global__ __launch_bounds__(256) void moe_median_kernel(const float* __restrict__ ratios, int T, float* beta) {
  __shared__ uint32_t hist[256];
  __shared__ uint32_t sh[2];
  const float* col = ratios + (int64_t)blockIdx.x * T;
  const float hi = select_rank(col, T, (uint32_t)(T / 2), hist, sh);
  float med = hi;
  if ((T & 1) == 0) med = 0.5f * (select_rank(col, T, (uint32_t)(T / 2 - 1), hist, sh) + hi);
  if (threadIdx.x == 0) beta[blockIdx.x] = med;
}

// ---- acceptance / resampling -------------------------------------------------------------------
constexpr int kAccThreads = 1024;
constexpr int kAccWaves = kAccThreads / 64;
constexpr int kChunk = 256;                               // tokens per chunk: four per lane
constexpr int kMaxChunks = 2 * kAccThreads;               // two chunk sums per thread in the scan

// Inclusive prefix sum over the 64 lanes with cross-lane operand moves only (no trip through LDS
// per step): shifts by 1, 2, 4, 8 inside each row of 16 lanes (lanes without a source add zero),
// then the last lane of row 0 / row 2 into rows 1 / 3, then the last lane of row 1 into rows 2, 3.
template <int CTRL, int ROW_MASK, bool BOUND>
__device__ __forceinline__ float lane_move(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, ROW_MASK, 0xf, BOUND));
}
__device__ __forceinline__ float wave_inclusive_sum_f(float v, int /*lane*/) {
  v += lane_move<0x111, 0xf, true>(v);    // row_shr:1
  v += lane_move<0x112, 0xf, true>(v);    // row_shr:2
  v += lane_move<0x114, 0xf, true>(v);    // row_shr:4
  v += lane_move<0x118, 0xf, true>(v);    // row_shr:8
  v += lane_move<0x142, 0xa, false>(v);   // row_bcast:15 -> rows 1, 3
  v += lane_move<0x143, 0xc, false>(v);   // row_bcast:31 -> rows 2, 3
  return v;
}

// Residual mass (Eq. 3) of tokens v .. v + 3 of the rejected position; tokens past V count nothing.
__device__ __forceinline__ float4 residual4(const float* __restrict__ pt, const float* __restrict__ pd, int v, int V,
                                            bool aligned, bool from_target) {
  float4 a = make_float4(0.f, 0.f, 0.f, 0.f), d = a;
  if (aligned && v + 3 < V) {
    a = *reinterpret_cast<const float4*>(pt + v);
    d = *reinterpret_cast<const float4*>(pd + v);
  } else {
    if (v < V) { a.x = pt[v]; d.x = pd[v]; }
    if (v + 1 < V) { a.y = pt[v + 1]; d.y = pd[v + 1]; }
    if (v + 2 < V) { a.z = pt[v + 2]; d.z = pd[v + 2]; }
    if (v + 3 < V) { a.w = pt[v + 3]; d.w = pd[v + 3]; }
  }
  if (from_target) return a;
  return make_float4(fmaxf(0.f, a.x - d.x), fmaxf(0.f, a.y - d.y), fmaxf(0.f, a.z - d.z), fmaxf(0.f, a.w - d.w));
}

// grid: (B); block: 1024.  The vocabulary is cut into chunks of 256 consecutive tokens (a lane holds
// four, so a wavefront reads a chunk as one contiguous kilobyte per distribution); wavefront w sums
// the chunks of its contiguous share, the chunk sums are scanned by the workgroup, and the chunk the
// target mass falls in is walked by one wavefront.  The intervals [lower, upper) are built so that
// one's upper bound is the next one's lower bound bit for bit: exactly one chunk and one lane match.
__global__ __launch_bounds__(kAccThreads) void accept_kernel(const float* __restrict__ p_target,
                                                             const float* __restrict__ p_draft,
                                                             const int32_t* __restrict__ draft_tokens,
                                                             const float* __restrict__ u_accept,
                                                             const float* __restrict__ u_resample, int gamma, int V,
                                                             int32_t* n_accepted, int32_t* resampled) {
  __shared__ float csum[kMaxChunks];
  __shared__ float wave_sum[kAccWaves];
  __shared__ int sh_n, sh_pick, sh_chunk;
  __shared__ float sh_total, sh_base;
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t seq = (int64_t)b * gamma;
  if (wave == 0) {
    bool rejected = false;
    if (lane < gamma) {
      const int x = min(max(draft_tokens[seq + lane], 0), V - 1);
      const float pt = p_target[(seq + lane) * V + x], pd = p_draft[(seq + lane) * V + x];
      const float alpha = pd > 0.f ? fminf(1.0f, pt / pd) : 1.0f;                 // Eq. 2
      rejected = !(u_accept[seq + lane] < alpha);
    }
    const uint64_t rj = __ballot(rejected);
    if (lane == 0) sh_n = rj ? __builtin_ctzll(rj) : gamma;
  }
  __syncthreads();
  const int n = sh_n;
  if (n == gamma) {
    if (tid == 0) { n_accepted[b] = n; resampled[b] = -1; }
    return;
  }
  const float* pt = p_target + (seq + n) * V;
  const float* pd = p_draft + (seq + n) * V;
  const bool aligned = (V & 3) == 0;
  const int n_chunks = (V + kChunk - 1) / kChunk;
  const int cpw = (n_chunks + kAccWaves - 1) / kAccWaves;
  const int c_begin = wave * cpw, c_end = min(c_begin + cpw, n_chunks);
  bool from_target = false;
  float total = 0.f;
  for (int round = 0; round < 2; ++round) {
    if (tid == 0) { sh_chunk = n_chunks - 1; sh_base = 0.f; sh_pick = V - 1; }
    for (int i = tid; i < kMaxChunks; i += kAccThreads) csum[i] = 0.f;
    __syncthreads();
    // chunk sums, eight chunks' loads in flight per wavefront
    for (int c0 = c_begin; c0 < c_end; c0 += 8) {
      float4 r[8];
#pragma unroll
      for (int u = 0; u < 8; ++u)
        r[u] = residual4(pt, pd, min(c0 + u, c_end - 1) * kChunk + 4 * lane, V, aligned, from_target);
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const float incl = wave_inclusive_sum_f(((r[u].x + r[u].y) + r[u].z) + r[u].w, lane);
        if (lane == 63 && c0 + u < c_end) csum[c0 + u] = incl;
      }
    }
    __syncthreads();
    // scan of the chunk sums: thread t takes chunks 2t and 2t + 1
    const float s0 = csum[2 * tid], s1 = csum[2 * tid + 1];
    const float incl = wave_inclusive_sum_f(s0 + s1, lane);
    if (lane == 63) wave_sum[wave] = incl;
    __syncthreads();
    float before = 0.f;
    for (int w2 = 0; w2 < wave; ++w2) before += wave_sum[w2];
    const float prev = __shfl_up(incl, 1, 64);
    const float upper = before + incl;
    const float lower = lane == 0 ? before : before + prev;
    if (tid == kAccThreads - 1) sh_total = upper;
    __syncthreads();
    total = sh_total;
    if (total > 0.f || from_target) {
      const float target = u_resample[b] * total;
      if (lower <= target && target < upper) {
        const bool second = !(target < lower + s0);
        sh_chunk = min(2 * tid + (second ? 1 : 0), n_chunks - 1);
        sh_base = second ? lower + s0 : lower;
      }
      break;
    }
    from_target = true;                                   // the distributions coincide: resample from p_theta
    __syncthreads();
  }
  __syncthreads();
  if (wave == 0) {
    const float target = u_resample[b] * total;
    const int v = sh_chunk * kChunk + 4 * lane;
    const float base = sh_base;
    // (if rounding leaves the target just outside every lane's interval: the chunk's last token)
    if (lane == 0) sh_pick = min((sh_chunk + 1) * kChunk, V) - 1;
    const float4 r = residual4(pt, pd, v, V, aligned, from_target);
    const float incl = wave_inclusive_sum_f(((r.x + r.y) + r.z) + r.w, lane);
    const float prev = __shfl_up(incl, 1, 64);
    const float upper = base + incl;
    float c = lane == 0 ? base : base + prev;
    if (c <= target && target < upper) {
      int pick = v + 3;
      c += r.x;
      if (c > target) pick = v;
      else if ((c += r.y) > target) pick = v + 1;
      else if ((c += r.z) > target) pick = v + 2;
      sh_pick = min(pick, V - 1);
    }
  }
  __syncthreads();
  if (tid == 0) { n_accepted[b] = n; resampled[b] = sh_pick; }
}

size_t align256(size_t x) { return (x + 255) / 256 * 256; }

}  // namespace

extern "C" {

int svf_moe_skip(const float* w, int32_t T, int32_t k, int32_t m, const float* beta, int32_t* n_skip,
                 uint32_t* keep_mask, void* stream) {
  if (!w || !beta || !n_skip || !keep_mask) return SVF_ERR_NULL;
  if (T < 1 || k < 2 || k > 32) return SVF_ERR_SHAPE;
  if (m < 1 || m >= k) return SVF_ERR_BUDGET;
  hipLaunchKernelGGL(moe_skip_kernel, dim3((T + kTokPerBlock - 1) / kTokPerBlock), dim3(kMoeThreads), 0,
                     static_cast<hipStream_t>(stream), w, T, k, m, beta, n_skip, keep_mask);
  return hipGetLastError() == hipSuccess ? SVF_OK : SVF_ERR_HIP;
}

size_t svf_moe_calibrate_workspace_bytes(int32_t T, int32_t k) {
  if (T < 1 || k < 2 || k > 32) return 0;
  return align256((size_t)(k - 1) * T * sizeof(float));
}

int svf_moe_calibrate(const float* w_cal, int32_t T, int32_t k, float* beta, void* ws, size_t ws_bytes,
                      void* stream) {
  if (!w_cal || !beta) return SVF_ERR_NULL;
  if (T < 1 || k < 2 || k > 32) return SVF_ERR_SHAPE;
  if (!ws || reinterpret_cast<uintptr_t>(ws) % 256 || ws_bytes < svf_moe_calibrate_workspace_bytes(T, k))
    return SVF_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  float* ratios = static_cast<float*>(ws);
  hipLaunchKernelGGL(moe_ratios_kernel, dim3((T + kTokPerBlock - 1) / kTokPerBlock), dim3(kMoeThreads), 0, st, w_cal,
                     T, k, ratios);
  if (hipGetLastError() != hipSuccess) return SVF_ERR_HIP;
  hipLaunchKernelGGL(moe_median_kernel, dim3(k - 1), dim3(256), 0, st, ratios, T, beta);
  return hipGetLastError() == hipSuccess ? SVF_OK : SVF_ERR_HIP;
}

int svf_accept_resample(const float* p_target, const float* p_draft, const int32_t* draft_tokens,
                        const float* u_accept, const float* u_resample, int32_t B, int32_t gamma, int32_t V,
                        int32_t* n_accepted, int32_t* resampled, void* stream) {
  if (!p_target || !p_draft || !draft_tokens || !u_accept || !u_resample || !n_accepted || !resampled)
    return SVF_ERR_NULL;
  if (B < 1 || gamma < 1 || gamma > 64 || V < 1 || V > kMaxChunks * kChunk) return SVF_ERR_SHAPE;
  hipLaunchKernelGGL(accept_kernel, dim3(B), dim3(kAccThreads), 0, static_cast<hipStream_t>(stream), p_target, p_draft,
                     draft_tokens, u_accept, u_resample, gamma, V, n_accepted, resampled);
  return hipGetLastError() == hipSuccess ? SVF_OK : SVF_ERR_HIP;
}

}  // extern "C"
