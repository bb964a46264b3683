// Block representatives: the mean key of every retrieval block (Sec. 3.1; block term of Eq. 5),
// or, as a variant, the per-channel minimum and maximum of its keys (the block summary of Quest,
// which Sec. 3.1 names as its starting point); fp32 or bf16 output.
//
// HBM-bound streaming reduction: K is read exactly once with 16-byte loads, fp32 accumulation
// in a fixed (logical-token) order, fp32 representatives written once.  One workgroup per
// (sequence, block); a thread owns one 16-byte column chunk of one KV head and walks the
// block's tokens with a stride of TOK_PAR tokens, TOK_PAR thread groups cover the tokens in
// parallel and are combined through LDS in a fixed order, so the result does not depend on
// the physical page order.
#include <hip/hip_bf16.h>

#include "svf_device.h"

namespace svf {

namespace {

constexpr int kThreads = 256;

template <typename T>
struct Vec16;
template <>
struct Vec16<float> {
  static constexpr int N = 4;
  __device__ static void load(const float* p, float (&v)[4]) {
    const float4 x = *reinterpret_cast<const float4*>(p);
    v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w;
  }
};
template <>
struct Vec16<__hip_bfloat16> {
  static constexpr int N = 8;
  __device__ static void load(const __hip_bfloat16* p, float (&v)[8]) {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 x = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));   // read once
    const uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[2 * i] = __uint_as_float(w[i] << 16);
      v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
};

// Four consecutive values to the output's element type.
__device__ __forceinline__ void store4(float* o, float a, float b, float c, float d) {
  *reinterpret_cast<float4*>(o) = make_float4(a, b, c, d);
}
__device__ __forceinline__ void store4(__hip_bfloat16* o, float a, float b, float c, float d) {
  const __hip_bfloat16 h[4] = {__float2bfloat16(a), __float2bfloat16(b), __float2bfloat16(c), __float2bfloat16(d)};
  uint2 w;
  w.x = (uint32_t)__builtin_bit_cast(unsigned short, h[0]) | ((uint32_t)__builtin_bit_cast(unsigned short, h[1]) << 16);
  w.y = (uint32_t)__builtin_bit_cast(unsigned short, h[2]) | ((uint32_t)__builtin_bit_cast(unsigned short, h[3]) << 16);
  *reinterpret_cast<uint2*>(o) = w;
}

// grid: (blocks in range, B, column groups); block: kThreads.  MINMAX: acc holds the running
// minimum and acc2 the running maximum instead of the sum; OT: element type written.
template <typename T, bool MINMAX, typename OT>
__global__ __launch_bounds__(kThreads) void block_reps_kernel(RepsParams p, int cols, int cpb, int tok_par) {
  constexpr int N = Vec16<T>::N;
  __shared__ float red[kThreads * N * (MINMAX ? 2 : 1)];

  const int b = blockIdx.y;
  const int j = p.first_block + blockIdx.x;
  const int L = clamped_len(p.seq_lens, b, p.max_seq_len);
  const int t0 = j * p.block_size;
  if (t0 >= L) return;                                  // block does not exist in this sequence
  const int n_tok = min(p.block_size, L - t0);

  const int tid = threadIdx.x;
  const int tl = tid / cpb;                             // token lane
  const int col = blockIdx.z * cpb + (tid - tl * cpb);  // 16-byte column chunk over (head, channel)
  const bool active = tl < tok_par && col < cols;
  const int chunks_per_head = p.d / N;
  const int h = col / chunks_per_head;
  const int c = (col - h * chunks_per_head) * N;

  float acc[N], acc2[MINMAX ? N : 1];
#pragma unroll
  for (int i = 0; i < N; ++i) {
    acc[i] = MINMAX ? __builtin_inff() : 0.f;
    if (MINMAX) acc2[i] = -__builtin_inff();
  }
  auto take = [&](const float (&v)[N]) {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      if (MINMAX) {
        acc[i] = fminf(acc[i], v[i]);
        acc2[i] = fmaxf(acc2[i], v[i]);
      } else {
        acc[i] += v[i];
      }
    }
  };

  if (active) {
    const T* K = static_cast<const T*>(p.K) + (int64_t)h * p.kv.stride_head + c;
    int t = tl;
    // four independent loads in flight per iteration
    for (; t + 3 * tok_par < n_tok; t += 4 * tok_par) {
      float v[4][N];
#pragma unroll
      for (int u = 0; u < 4; ++u)
        Vec16<T>::load(K + token_offset(p.kv, p.table, b, t0 + t + u * tok_par), v[u]);
#pragma unroll
      for (int u = 0; u < 4; ++u) take(v[u]);
    }
    for (; t < n_tok; t += tok_par) {
      float v[N];
      Vec16<T>::load(K + token_offset(p.kv, p.table, b, t0 + t), v);
      take(v);
    }
  }

  if (tok_par > 1) {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      red[tid * N + i] = acc[i];
      if (MINMAX) red[(kThreads + tid) * N + i] = acc2[i];
    }
    __syncthreads();
    if (active && tl == 0) {
      for (int u = 1; u < tok_par; ++u)
#pragma unroll
        for (int i = 0; i < N; ++i) {
          if (MINMAX) {
            acc[i] = fminf(acc[i], red[(u * cpb + tid) * N + i]);
            acc2[i] = fmaxf(acc2[i], red[(kThreads + u * cpb + tid) * N + i]);
          } else {
            acc[i] += red[(u * cpb + tid) * N + i];
          }
        }
    }
  }
  if (active && tl == 0) {
    const float inv = MINMAX ? 1.0f : 1.0f / (float)n_tok;
    OT* r = static_cast<OT*>(p.reps) + ((((int64_t)b * p.Hkv + h) * p.nb_max + j) * (MINMAX ? 2 : 1)) * p.d + c;
#pragma unroll
    for (int i = 0; i < N; i += 4) {
      store4(r + i, acc[i] * inv, acc[i + 1] * inv, acc[i + 2] * inv, acc[i + 3] * inv);
      if (MINMAX) store4(r + p.d + i, acc2[i], acc2[i + 1], acc2[i + 2], acc2[i + 3]);
    }
  }
}

template <typename T>
void launch_for(const RepsParams& p, dim3 grid, int cols, int cpb, int tok_par, hipStream_t st) {
  if (p.minmax) {
    if (p.out_bf16) hipLaunchKernelGGL((block_reps_kernel<T, true, __hip_bfloat16>), grid, dim3(kThreads), 0, st, p, cols, cpb, tok_par);
    else hipLaunchKernelGGL((block_reps_kernel<T, true, float>), grid, dim3(kThreads), 0, st, p, cols, cpb, tok_par);
  } else {
    if (p.out_bf16) hipLaunchKernelGGL((block_reps_kernel<T, false, __hip_bfloat16>), grid, dim3(kThreads), 0, st, p, cols, cpb, tok_par);
    else hipLaunchKernelGGL((block_reps_kernel<T, false, float>), grid, dim3(kThreads), 0, st, p, cols, cpb, tok_par);
  }
}

}  // namespace

hipError_t launch_block_reps(const RepsParams& p, int dtype, int B, hipStream_t st) {
  if (p.n_blocks <= 0) return hipSuccess;
  const int N = dtype == SVF_F32 ? 4 : 8;
  const int cols = p.Hkv * p.d / N;
  const int cpb = cols < kThreads ? cols : kThreads;
  const int tok_par = kThreads / cpb;
  dim3 grid(p.n_blocks, B, (cols + cpb - 1) / cpb);
  if (dtype == SVF_F32) launch_for<float>(p, grid, cols, cpb, tok_par, st);
  else launch_for<__hip_bfloat16>(p, grid, cols, cpb, tok_par, st);
  return hipGetLastError();
}

}  // namespace svf
