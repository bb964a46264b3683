// Verification attention, vector-ALU kernel (Sec. 3.1 / 3.3: the draft queries attend to the
// retrieved blocks of their KV head and, through the draft mask, to each other).
//
// Used for fp32 inputs and for head dimensions the matrix-core kernel does not cover.
// Split-K over the selected tokens: workgroup (split, kv head, sequence x row group) walks
// its share of 32-token tiles (prefix tiles first, then the draft tile(s)), staging K and V
// through LDS as fp32; thread (r, sub) owns query row r of the row group and the channels
// sub, sub+8, ...  The 8 lanes of a row compute its 32 logits, keep the running maximum and
// denominator in registers (online softmax in the log2 domain) and accumulate its output.
// Each split writes an unnormalised partial (o, m, l); a second kernel merges the splits
// with the log-sum-exp rule and writes out / lse.
#include <hip/hip_bf16.h>

#include "svf_device.h"

namespace svf {

namespace {

constexpr int kThreads = 256;
constexpr int kRows = 32;      // query rows per workgroup
constexpr int kTile = 32;      // tokens per tile
constexpr int kSub = 8;        // lanes per query row

template <typename T>
__device__ __forceinline__ float to_float(T x);
template <>
__device__ __forceinline__ float to_float<float>(float x) { return x; }
template <>
__device__ __forceinline__ float to_float<__hip_bfloat16>(__hip_bfloat16 x) { return __bfloat162float(x); }

// grid: (n_splits, Hkv, B * row_groups)
template <typename T, int D>
__global__ __launch_bounds__(kThreads) void verify_attn_valu_kernel(AttnParams p, int row_groups) {
  constexpr int KP = D + 1;                   // padded K row (floats) to spread LDS banks
  __shared__ float sQ[kRows * D];
  __shared__ float sK[kTile * KP];
  __shared__ float sV[kTile * D];
  __shared__ float sP[kRows * (kTile + 1)];
  __shared__ int sTok[kTile];                 // >= 0: prefix token, -1: invalid, -2 - t: draft t

  const int split = blockIdx.x, h = blockIdx.y;
  const int b = blockIdx.z / row_groups, rg = blockIdx.z - b * row_groups;
  const int tid = threadIdx.x;
  const int r = tid / kSub, sub = tid % kSub;
  const int row = rg * kRows + r;             // row inside the (b, h) pair: draft * G + group head
  const bool row_ok = row < p.M;
  const int di = row_ok ? row / p.G : 0;      // draft index of this row
  const int hq = h * p.G + (row_ok ? row % p.G : 0);

  const int L = clamped_len(p.seq_lens, b, p.max_seq_len);
  const int cnt = min(max(p.sel_cnt[(int64_t)b * p.Hkv + h], 0), p.k_blocks);
  const int32_t* sel = p.sel_idx + ((int64_t)b * p.Hkv + h) * p.k_blocks;
  const int n_prefix = cnt * p.block_size;    // token slots of the selected blocks
  const int tiles_p = (n_prefix + kTile - 1) / kTile;
  const int tiles_d = (p.gamma + kTile - 1) / kTile;
  const int tiles = tiles_p + tiles_d;
  const int per = (tiles + p.n_splits - 1) / p.n_splits;
  const int tile0 = split * per;
  const int tile1 = min(tiles, tile0 + per);

  uint64_t mask = 0;
  if (row_ok) {
    if (p.draft_mask) mask = p.draft_mask[p.mask_per_batch ? (int64_t)b * p.gamma + di : di];
    else mask = di >= 63 ? ~0ull : ((2ull << di) - 1ull);
  }

  // stage this row group's queries as fp32
  for (int e = tid; e < kRows * D; e += kThreads) {
    const int rr = e / D, c = e - rr * D;
    const int grow = rg * kRows + rr;
    float v = 0.f;
    if (grow < p.M) {
      const int i = grow / p.G, j = h * p.G + grow % p.G;
      v = to_float<T>(static_cast<const T*>(p.q)[(((int64_t)b * p.gamma + i) * p.Hq + j) * D + c]);
    }
    sQ[e] = v;
  }

  float m_run = -INFINITY, l_run = 0.f;
  float acc[D / kSub];
#pragma unroll
  for (int i = 0; i < D / kSub; ++i) acc[i] = 0.f;

  for (int tile = tile0; tile < tile1; ++tile) {
    __syncthreads();                          // previous tile fully consumed (and sQ visible)
    // which token sits in each of the tile's 32 slots
    if (tid < kTile) {
      int code = -1;
      if (tile < tiles_p) {
        const int slot = tile * kTile + tid;
        if (slot < n_prefix) {
          const int bi = slot / p.block_size;
          const int blk = sel[bi];
          const int t = blk * p.block_size + (slot - bi * p.block_size);
          if (blk >= 0 && t < L) code = t;
        }
      } else {
        const int t = (tile - tiles_p) * kTile + tid;
        if (t < p.gamma) code = -2 - t;
      }
      sTok[tid] = code;
    }
    __syncthreads();
    // cooperative load: 8 threads per token, D/8 channels each
    {
      const int tt = tid / 8, part = tid % 8;
      const int code = sTok[tt];
      constexpr int CH = D / 8;
      const T* ksrc = nullptr;
      const T* vsrc = nullptr;
      if (code >= 0) {
        const int64_t off = token_offset(p.kv, p.table, b, code) + (int64_t)h * p.kv.stride_head + part * CH;
        ksrc = static_cast<const T*>(p.K) + off;
        vsrc = static_cast<const T*>(p.V) + off;
      } else if (code <= -2) {
        const int64_t off = (((int64_t)b * p.gamma + (-2 - code)) * p.Hkv + h) * D + part * CH;
        ksrc = static_cast<const T*>(p.k_draft) + off;
        vsrc = static_cast<const T*>(p.v_draft) + off;
      }
#pragma unroll
      for (int c = 0; c < CH; ++c) {
        sK[tt * KP + part * CH + c] = ksrc ? to_float<T>(ksrc[c]) : 0.f;
        sV[tt * D + part * CH + c] = vsrc ? to_float<T>(vsrc[c]) : 0.f;
      }
    }
    __syncthreads();

    // logits of row r against tokens sub, sub + 8, sub + 16, sub + 24
    float s[kTile / kSub];
    float m_tile = -INFINITY;
#pragma unroll
    for (int u = 0; u < kTile / kSub; ++u) {
      const int t = sub + kSub * u;
      const int code = sTok[t];
      float dot = 0.f;
#pragma unroll 8
      for (int c = 0; c < D; ++c) dot += sQ[r * D + c] * sK[t * KP + c];
      bool vis = code >= 0;
      if (code <= -2) vis = (mask >> (-2 - code)) & 1ull;
      s[u] = vis && row_ok ? dot * p.scale_log2 : -INFINITY;
      m_tile = fmaxf(m_tile, s[u]);
    }
#pragma unroll
    for (int o = 1; o < kSub; o <<= 1) m_tile = fmaxf(m_tile, __shfl_xor(m_tile, o, 64));
    const float m_new = fmaxf(m_run, m_tile);
    const float m_use = m_new == -INFINITY ? 0.f : m_new;
    const float alpha = exp2f(m_run - m_use);          // m_run = -inf gives 0
    float l_tile = 0.f;
#pragma unroll
    for (int u = 0; u < kTile / kSub; ++u) {
      const float pe = exp2f(s[u] - m_use);
      l_tile += pe;
      sP[r * (kTile + 1) + sub + kSub * u] = pe;
    }
#pragma unroll
    for (int o = 1; o < kSub; o <<= 1) l_tile += __shfl_xor(l_tile, o, 64);
    l_run = l_run * alpha + l_tile;
    m_run = m_new;
    __syncthreads();                          // sP complete (rows are wave-local, but keep it simple)

#pragma unroll
    for (int i = 0; i < D / kSub; ++i) acc[i] *= alpha;
    for (int t = 0; t < kTile; ++t) {
      const float pe = sP[r * (kTile + 1) + t];
#pragma unroll
      for (int i = 0; i < D / kSub; ++i) acc[i] += pe * sV[t * D + sub + kSub * i];
    }
  }

  // partial result of this split
  const int64_t pr = (((int64_t)b * p.Hkv + h) * p.n_splits + split) * p.Mpad + row;
  if (row < p.Mpad) {
#pragma unroll
    for (int i = 0; i < D / kSub; ++i) p.part_o[pr * D + sub + kSub * i] = acc[i];
    if (sub == 0) {
      p.part_m[pr] = m_run;
      p.part_l[pr] = l_run;
    }
  }
}

template <typename T>
__device__ __forceinline__ void store_out(T* dst, float v);
template <>
__device__ __forceinline__ void store_out<float>(float* dst, float v) { *dst = v; }
template <>
__device__ __forceinline__ void store_out<__hip_bfloat16>(__hip_bfloat16* dst, float v) {
  *dst = __float2bfloat16(v);   // round to nearest even
}

// grid: (M, Hkv, B); block: D threads.  Merges the per-split partials of one query row.
template <typename T>
__global__ void merge_splits_kernel(AttnParams p) {
  const int row = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int c = threadIdx.x;
  const int D = p.d;
  const int64_t base = ((int64_t)b * p.Hkv + h) * p.n_splits;
  float m = -INFINITY;
  for (int s = 0; s < p.n_splits; ++s) m = fmaxf(m, p.part_m[(base + s) * p.Mpad + row]);
  float l = 0.f, o = 0.f;
  for (int s = 0; s < p.n_splits; ++s) {
    const int64_t pr = (base + s) * p.Mpad + row;
    const float ms = p.part_m[pr];
    if (ms == -INFINITY) continue;
    const float w = exp2f(ms - m);
    l += w * p.part_l[pr];
    o += w * p.part_o[pr * D + c];
  }
  const int i = row / p.G, j = h * p.G + row % p.G;
  const int64_t orow = ((int64_t)b * p.gamma + i) * p.Hq + j;
  // a row that saw no key at all (no kept block, a draft mask without its own bit): zero, lse = -inf
  store_out<T>(static_cast<T*>(p.out) + orow * D + c, l > 0.f ? o / l : 0.f);
  if (p.lse && c == 0) p.lse[orow] = (m + log2f(l)) * 0.6931471805599453f;
}

}  // namespace

hipError_t launch_merge_splits(const AttnParams& p, int dtype, hipStream_t st) {
  dim3 grid(p.M, p.Hkv, p.B);
  if (dtype == SVF_F32) hipLaunchKernelGGL(merge_splits_kernel<float>, grid, dim3(p.d), 0, st, p);
  else hipLaunchKernelGGL(merge_splits_kernel<__hip_bfloat16>, grid, dim3(p.d), 0, st, p);
  return hipGetLastError();
}

hipError_t launch_verify_attn_valu(const AttnParams& p, int dtype, hipStream_t st) {
  const int row_groups = p.Mpad / kRows;
  dim3 grid(p.n_splits, p.Hkv, p.B * row_groups);
  if (dtype == SVF_F32) {
    if (p.d == 64) hipLaunchKernelGGL((verify_attn_valu_kernel<float, 64>), grid, dim3(kThreads), 0, st, p, row_groups);
    else hipLaunchKernelGGL((verify_attn_valu_kernel<float, 128>), grid, dim3(kThreads), 0, st, p, row_groups);
  } else {
    if (p.d == 64) hipLaunchKernelGGL((verify_attn_valu_kernel<__hip_bfloat16, 64>), grid, dim3(kThreads), 0, st, p, row_groups);
    else hipLaunchKernelGGL((verify_attn_valu_kernel<__hip_bfloat16, 128>), grid, dim3(kThreads), 0, st, p, row_groups);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return launch_merge_splits(p, dtype, st);
}

}  // namespace svf
