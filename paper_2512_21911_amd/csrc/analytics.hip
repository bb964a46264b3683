// Retrieval analytics on block bit masks (block j = bit j % 64 of word j / 64):
//   overlap of the blocks retrieved by different draft tokens, by positional distance
//     (Sec. 2.2, Fig. 2: intersection of the two tokens' blocks over the number of blocks);
//   Jaccard similarity of adjacent layers' masks (Sec. 3.3, Eq. 7), the input of the anchor-layer
//     choice (Eq. 8, done on the host);
//   masks from the index lists the retrieval produces.
// All results are exact integer counts (intersections, unions); the ratios are formed by the
// caller, so the outcome does not depend on the order of the additions.
#include "svf_device.h"

namespace svf {

namespace {

constexpr int kThreads = 256;
constexpr int kMaxDrafts = 64;
constexpr int kMaxMaskWords = 64;     // masks of up to 4096 blocks are staged in LDS
constexpr int kMaxDist = 64;

// grid: pairs (sequence, KV head); one thread per kept block
__global__ __launch_bounds__(kThreads) void masks_from_selection_kernel(const int32_t* __restrict__ sel_idx,
                                                                         const int32_t* __restrict__ sel_cnt,
                                                                         uint64_t* __restrict__ masks, int k_blocks,
                                                                         int mask_words) {
  extern __shared__ unsigned long long words[];
  const int pair = blockIdx.x;
  for (int w = threadIdx.x; w < mask_words; w += kThreads) words[w] = 0ull;
  __syncthreads();
  const int cnt = min(max(sel_cnt[pair], 0), k_blocks);
  for (int i = threadIdx.x; i < cnt; i += kThreads) {
    const int j = sel_idx[(int64_t)pair * k_blocks + i];
    if (j >= 0 && (j >> 6) < mask_words) atomicOr(&words[j >> 6], 1ull << (j & 63));
  }
  __syncthreads();
  for (int w = threadIdx.x; w < mask_words; w += kThreads) masks[(int64_t)pair * mask_words + w] = words[w];
}

// grid: (Hkv, B).  masks [B][Hkv][gamma][W]; inter [B][n_dist] must be zero on entry.
__global__ __launch_bounds__(kThreads) void overlap_kernel(const uint64_t* __restrict__ masks,
                                                            const int32_t* __restrict__ pos,
                                                            unsigned long long* __restrict__ inter, int gamma,
                                                            int mask_words, int n_dist) {
  __shared__ uint64_t m[kMaxDrafts * kMaxMaskWords];
  __shared__ int32_t ps[kMaxDrafts];
  __shared__ unsigned long long bins[kMaxDist];
  const int h = blockIdx.x, b = blockIdx.y, Hkv = gridDim.x;
  const uint64_t* src = masks + ((int64_t)b * Hkv + h) * gamma * mask_words;
  for (int i = threadIdx.x; i < gamma * mask_words; i += kThreads) m[i] = src[i];
  for (int i = threadIdx.x; i < gamma; i += kThreads) ps[i] = pos[i];
  for (int i = threadIdx.x; i < n_dist; i += kThreads) bins[i] = 0ull;
  __syncthreads();
  const int n_pairs = gamma * (gamma - 1) / 2;
  for (int p = threadIdx.x; p < n_pairs; p += kThreads) {
    // p-th pair (i, i2), i < i2, in row-major order
    int i = 0, rem = p;
    while (rem >= gamma - 1 - i) {
      rem -= gamma - 1 - i;
      ++i;
    }
    const int i2 = i + 1 + rem;
    const int dist = abs(ps[i] - ps[i2]);
    if (dist >= n_dist) continue;
    unsigned long long c = 0;
    for (int w = 0; w < mask_words; ++w) c += (unsigned long long)__popcll(m[i * mask_words + w] & m[i2 * mask_words + w]);
    atomicAdd(&bins[dist], c);
  }
  __syncthreads();
  for (int i = threadIdx.x; i < n_dist; i += kThreads)
    if (bins[i]) atomicAdd(&inter[(int64_t)b * n_dist + i], bins[i]);
}

// grid: n_layers.  masks_by_layer [L][words_per_layer]; inter_union [L][2]; layer 0: (0, 0).
__global__ __launch_bounds__(kThreads) void jaccard_kernel(const uint64_t* __restrict__ masks_by_layer,
                                                            unsigned long long* __restrict__ inter_union,
                                                            int64_t words_per_layer) {
  __shared__ unsigned long long red[2][kThreads / 64];
  const int l = blockIdx.x;
  unsigned long long ci = 0, cu = 0;
  if (l > 0) {
    const uint64_t* a = masks_by_layer + (int64_t)l * words_per_layer;
    const uint64_t* c = a - words_per_layer;
    for (int64_t w = threadIdx.x; w < words_per_layer; w += kThreads) {
      ci += (unsigned long long)__popcll(a[w] & c[w]);
      cu += (unsigned long long)__popcll(a[w] | c[w]);
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    ci += __shfl_xor(ci, o, 64);
    cu += __shfl_xor(cu, o, 64);
  }
  if ((threadIdx.x & 63) == 0) {
    red[0][threadIdx.x >> 6] = ci;
    red[1][threadIdx.x >> 6] = cu;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    unsigned long long si = 0, su = 0;
    for (int w = 0; w < kThreads / 64; ++w) {
      si += red[0][w];
      su += red[1][w];
    }
    inter_union[2 * l] = si;
    inter_union[2 * l + 1] = su;
  }
}

__global__ void zero_u64_kernel(unsigned long long* p, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0ull;
}

}  // namespace

hipError_t launch_masks_from_selection(const int32_t* sel_idx, const int32_t* sel_cnt, uint64_t* masks, int pairs,
                                       int k_blocks, int mask_words, hipStream_t st) {
  hipLaunchKernelGGL(masks_from_selection_kernel, dim3(pairs), dim3(kThreads), (size_t)mask_words * 8, st, sel_idx,
                     sel_cnt, masks, k_blocks, mask_words);
  return hipGetLastError();
}

hipError_t launch_overlap_by_distance(const uint64_t* masks, const int32_t* pos, uint64_t* inter, int B, int Hkv,
                                      int gamma, int mask_words, int n_dist, hipStream_t st) {
  const int64_t n = (int64_t)B * n_dist;
  hipLaunchKernelGGL(zero_u64_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st,
                     reinterpret_cast<unsigned long long*>(inter), n);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(overlap_kernel, dim3(Hkv, B), dim3(kThreads), 0, st, masks, pos,
                     reinterpret_cast<unsigned long long*>(inter), gamma, mask_words, n_dist);
  return hipGetLastError();
}

hipError_t launch_jaccard_adjacent(const uint64_t* masks_by_layer, uint64_t* inter_union, int n_layers,
                                   int64_t words_per_layer, hipStream_t st) {
  hipLaunchKernelGGL(jaccard_kernel, dim3(n_layers), dim3(kThreads), 0, st, masks_by_layer,
                     reinterpret_cast<unsigned long long*>(inter_union), words_per_layer);
  return hipGetLastError();
}

}  // namespace svf
