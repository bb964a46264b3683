// Sparse feed-forward verification (Sec. 3.4, Eq. 10-14) for the M draft tokens of a step.
//
// Weight-bandwidth-bound: M <= 64 tokens against three [d_ff][d_model] bf16 matrices.  The
// matrix cores do the arithmetic (32x32x16 bf16, tokens padded to 32 or 64 columns; they idle
// most of the time), the work is organising the reads: every weight row is read at most once,
// in long contiguous runs, and the rows of W_up / W_down of hidden channels that are inactive
// for all M tokens are not read at all.
//
//   gate/up kernels one workgroup of four wavefronts per tile of hidden channels; the wavefronts
//                   split the model dimension in chunks of 128.  A chunk of the tile (32 rows x
//                   256 bytes per matrix) goes straight from global memory to the wavefront's
//                   own LDS stage (two stages, the next chunk is in flight while this one is
//                   multiplied), the matching piece of x comes through registers.
//                   Joint walk (default): the gate and the up matrix together, then
//                   h = act(W_gate x + b_gate), the active bits |h| >= tau per (channel, token),
//                   and h * up, masked per token, out as bf16 [tokens][d_ff]; x is fetched once
//                   for both matrices and nothing waits between them, but every row of W_up is
//                   read.  Gate first: the gate walk, the active bits, then the same walk over
//                   W_up where a row that no token needs is replaced by a row that is read anyway.
//   down kernel     y^T = W_down^T-rows times h_up: one workgroup of eight wavefronts per
//                   (128 output columns, slice of the hidden channels).  The weight rows are
//                   contiguous along the output dimension while the matrix core wants its
//                   operand contiguous along the reduction; each lane therefore loads four
//                   output columns of eight channels and byte-permutes them into operands
//                   (row i of sub-product nt = output column 4 i + nt).  Rows of channels
//                   nobody needs are skipped.  Wavefront results are added in wavefront order
//                   through LDS (one barrier); the slices' partial sums are added, with b_down, by a third
//                   small kernel (fixed order: the result does not depend on scheduling).
#include <hip/hip_bf16.h>
#include <hip/hip_runtime.h>

#include "svf_ffn_device.h"

namespace svf {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float floatx2;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
typedef __attribute__((__vector_size__(2 * sizeof(uint32_t)))) uint32_t u32x2;

#define FFN_GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void*)(p))
#define FFN_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))

constexpr int kTileRows = 32;                          // hidden channels per gate/up workgroup
constexpr int kChunkK = 128;                           // model dimensions per chunk
constexpr int kRowBytes = kChunkK * 2;                 // 256
constexpr int kChunkBytes = kTileRows * kRowBytes;     // 8 KB
constexpr int kGuWaves = 4;
constexpr int kGuThreads = kGuWaves * 64;
constexpr int kStages = 2;

// s_waitcnt with only the vector-memory counter constrained
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (0x7 << 4) | (0xF << 8));
  asm volatile("" ::: "memory");
}
// LDS read issued by hand (a compiler-issued one would first wait for every direct-to-LDS load
// in flight); valid once lds_wait has been given the registers
__device__ __forceinline__ u32x4 lds_read16(uint32_t addr) {
  u32x4 v;
  asm volatile("ds_read_b128 %0, %1" : "=v"(v) : "v"(addr) : "memory");
  return v;
}
__device__ __forceinline__ void lds_wait(u32x4 (&r)[8]) {
  asm volatile("s_waitcnt lgkmcnt(0)"
               : "+v"(r[0]), "+v"(r[1]), "+v"(r[2]), "+v"(r[3]), "+v"(r[4]), "+v"(r[5]), "+v"(r[6]), "+v"(r[7])
               :
               : "memory");
}
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  const floatx2 f = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));   // round to nearest even
}

__device__ __forceinline__ float activate(float z, int act) {
  if (act == SVF_ACT_SILU) return z / (1.0f + __expf(-z));
  return 0.5f * z * (1.0f + erff(z * 0.70710678118654752f));
}

// One walk of a wavefront over its chunks of a 32-row tile of NMAT matrices at once (the same
// rows of each): acc[mat][t] += W_mat_tile(chunk) x^T(chunk).
//   w_rows[mat]: address of row 0 of the tile in matrix mat; row_of(r): which tile row to read
//   for row r (a row nobody needs is redirected, its products are thrown away); stage: the
//   wavefront's two LDS stages of NMAT chunks each.
//   The workgroup's n_waves wavefronts take the chunks wave, wave + n_waves, ...
template <int NT, int NMAT, typename RowOf>
__device__ __forceinline__ void walk_tile(const FfnParams& p, const char* const (&w_rows)[NMAT], RowOf row_of,
                                          const char* x, unsigned char* stage, int wave, int n_waves, int lane,
                                          floatx16 (&acc)[NMAT][NT]) {
  constexpr int kStageBytes = NMAT * kChunkBytes;
  const int l32 = lane & 31, g = lane >> 5;
  const int n_chunks = p.d_model / kChunkK;
  const int64_t row_bytes = (int64_t)p.d_model * 2;
  // direct-to-LDS loads: instruction n brings rows 4n .. 4n+3, 16 lanes per row; the 16-byte
  // piece at position c of row r holds piece c ^ (r mod 16) of the chunk (bank spreading)
  const int lrow = lane >> 4, lcol = lane & 15;
  int64_t src_off[8];
#pragma unroll
  for (int n = 0; n < 8; ++n) {
    const int r = 4 * n + lrow;
    src_off[n] = (int64_t)row_of(r) * row_bytes + ((lcol ^ (r & 15)) << 4);
  }
  // x rows of this lane's token(s): eight 16-byte pieces per chunk (k-step ks, lane half g)
  const char* xrow[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) xrow[t] = x + (int64_t)min(l32 + 32 * t, p.M - 1) * row_bytes + g * 16;

  auto issue = [&](int kc, unsigned char* dst) {
#pragma unroll
    for (int mat = 0; mat < NMAT; ++mat)
#pragma unroll
      for (int n = 0; n < 8; ++n)
        __builtin_amdgcn_global_load_lds(FFN_GLOBAL_PTR(w_rows[mat] + src_off[n] + (int64_t)kc * kRowBytes),
                                         FFN_LDS_PTR(dst + mat * kChunkBytes + n * 1024), 16, 0, 2);
  };
  u32x4 xr[NT][8];
  auto load_x = [&](int kc) {
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int ks = 0; ks < 8; ++ks)
        xr[t][ks] = *reinterpret_cast<const u32x4*>(xrow[t] + (int64_t)kc * kRowBytes + ks * 32);
  };
  auto compute = [&](const unsigned char* src) {
    const uint32_t kx = (uint32_t)((g ^ (l32 & 15)) << 4);
#pragma unroll
    for (int mat = 0; mat < NMAT; ++mat) {
      const uint32_t base = (uint32_t)(uintptr_t)FFN_LDS_PTR(src + mat * kChunkBytes) + l32 * kRowBytes;
      u32x4 wf[8];
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) wf[ks] = lds_read16(base + (kx ^ (uint32_t)(ks << 5)));
      lds_wait(wf);
#pragma unroll
      for (int ks = 0; ks < 8; ++ks)
#pragma unroll
        for (int t = 0; t < NT; ++t)
          acc[mat][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, wf[ks]),
                                                                __builtin_bit_cast(bf16x8, xr[t][ks]), acc[mat][t], 0,
                                                                0, 0);
    }
  };

  // The weight chunk after this one is on its way into the other
  // stage while this one is multiplied; the x pieces of the next chunk are loaded right after
  // the multiply (one register set), long before that chunk's weights can have arrived.  Loads
  // retire in order, so "all but the 8 NMAT just issued" is one fixed wait count.
  int kc = wave;
  if (kc >= n_chunks) return;
  issue(kc, stage);
  load_x(kc);
  int cur = 0;
  while (true) {
    const int kn = kc + n_waves;
    if (kn >= n_chunks) {
      wait_vmcnt<0>();
      compute(stage + cur * kStageBytes);
      break;
    }
    issue(kn, stage + (cur ^ 1) * kStageBytes);
    wait_vmcnt<8 * NMAT>();
    compute(stage + cur * kStageBytes);
    load_x(kn);
    kc = kn;
    cur ^= 1;
  }
}

// grid: (d_ff / 32); block: 256
template <int NT>
__global__ __launch_bounds__(kGuThreads) void ffn_gate_up_kernel(FfnParams p) {
  constexpr int RS = 32 * NT + 1;                        // row stride of the [channel][token] tiles in LDS
  __shared__ __attribute__((aligned(1024))) unsigned char smem[kGuWaves * kStages * kChunkBytes];
  __shared__ float s_h[kTileRows * RS];
  __shared__ uint64_t s_act[kTileRows];
  static_assert(kTileRows * RS * 4 <= kStages * kChunkBytes, "a wavefront's partial tile fits its own stages");

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int l32 = lane & 31, g = lane >> 5;
  const int c0 = blockIdx.x * kTileRows;
  unsigned char* stage = smem + wave * (kStages * kChunkBytes);
  float* red = reinterpret_cast<float*>(stage);         // this wavefront's partial [channel][token]
  const char* x = static_cast<const char*>(p.x);
  const int64_t row_bytes = (int64_t)p.d_model * 2;

  auto put_partial = [&](const floatx16 (&acc)[NT]) {
    // value v of a lane is channel 8 (v / 4) + 4 g + v % 4, token l32 (+ 32 t)
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int v = 0; v < 16; ++v) red[(8 * (v >> 2) + 4 * g + (v & 3)) * RS + l32 + 32 * t] = acc[t][v];
  };
  auto sum_partials = [&](int c, int m) {
    float s = 0.f;
#pragma unroll
    for (int w = 0; w < kGuWaves; ++w)
      s += reinterpret_cast<const float*>(smem + w * (kStages * kChunkBytes))[c * RS + m];
    return s;
  };

  // ---- gate: h = act(W_gate x + b_gate), active bits (Eq. 10, 12) ----
  floatx16 acc[1][NT];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[0][t][v] = 0.f;
  {
    const char* const rows[1] = {static_cast<const char*>(p.w_gate) + (int64_t)c0 * row_bytes};
    walk_tile<NT, 1>(p, rows, [](int r) { return r; }, x, stage, wave, kGuWaves, lane, acc);
  }
  put_partial(acc[0]);
  __syncthreads();
  {
    // thread: channel tid / 8, tokens (tid % 8) * 4 NT ... + 4 NT
    const int c = tid >> 3, m0 = (tid & 7) * 4 * NT;
    const float bg = p.b_gate ? p.b_gate[c0 + c] : 0.f;
    uint64_t bits = 0;
#pragma unroll
    for (int i = 0; i < 4 * NT; ++i) {
      const int m = m0 + i;
      const float h = activate(sum_partials(c, m) + bg, p.act);
      s_h[c * RS + m] = h;
      if (m < p.M && !(fabsf(h) < p.tau)) bits |= 1ull << m;
    }
    // the eight threads of a channel are neighbours in a wavefront
#pragma unroll
    for (int o = 1; o < 8; o <<= 1) {
      const uint32_t lo = __shfl_xor((uint32_t)bits, o, 64), hi = __shfl_xor((uint32_t)(bits >> 32), o, 64);
      bits |= (uint64_t)lo | ((uint64_t)hi << 32);
    }
    if ((tid & 7) == 0) {
      s_act[c] = bits;
      p.rowany[c0 + c] = bits != 0 ? 1 : 0;
      if (p.active) p.active[c0 + c] = bits;
    }
  }
  __syncthreads();                                        // partials read, s_h / s_act written

  // ---- up: only rows some token needs are read; h * up per token (Eq. 13) ----
  const uint64_t my_bits = s_act[l32];
  const uint32_t rowmask = (uint32_t)__ballot(my_bits != 0 && lane < 32);
  bf16x8 zero8;
#pragma unroll
  for (int i = 0; i < 8; ++i) zero8[i] = 0;
  // thread: token tid / 4, channels (tid % 4) * 8 ... + 8 (16 bytes of h_up)
  const int om = tid >> 2, oc = (tid & 3) * 8;
  char* out = static_cast<char*>(p.h_up) + ((int64_t)om * p.d_ff + c0 + oc) * 2;
  if (rowmask == 0) {                                     // uniform: nothing of this tile is used
    if (om < 32 * NT) *reinterpret_cast<bf16x8*>(out) = zero8;
    return;
  }
  const int first = __builtin_ctz(rowmask);
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[0][t][v] = 0.f;
  {
    const char* const rows[1] = {static_cast<const char*>(p.w_up) + (int64_t)c0 * row_bytes};
    walk_tile<NT, 1>(p, rows, [=](int r) { return ((rowmask >> r) & 1u) ? r : first; }, x, stage, wave, kGuWaves, lane,
                     acc);
  }
  put_partial(acc[0]);
  __syncthreads();
  if (om < 32 * NT) {
    u32x4 w;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      float hu[2];
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        const int c = oc + 2 * j + e;
        const float up = sum_partials(c, om) + (p.b_up ? p.b_up[c0 + c] : 0.f);
        hu[e] = ((s_act[c] >> om) & 1ull) ? s_h[c * RS + om] * up : 0.f;
      }
      w[j] = pack_bf16(hu[0], hu[1]);
    }
    *reinterpret_cast<u32x4*>(out) = w;
  }
}

// The same result with the gate and the up matrix walked together: x is fetched once per chunk for
// both, and the workgroup's memory pipeline does not run dry between a gate and an up walk; the
// price is that every row of W_up is read, needed or not.
//   TILES channel tiles per workgroup share the x pieces as well (TILES = 2 for more than 32
//   tokens, where fetching x costs as much as fetching the weights), WAVES wavefronts split the
//   model dimension; TILES * WAVES = 4, 128 KB of stages, one workgroup per compute unit.  So
//   the tile height p.tile_rows <= 32 is chosen such that the workgroups fill whole rounds; the
//   rows of the 32-row matrix-core tile past it repeat its last row, and a tile that would
//   reach past d_ff is moved back to end there (the channels it shares with its neighbour are
//   computed twice, to the same bits).
// grid: (ceil(ceil(d_ff / tile_rows) / TILES)); block: 64 WAVES
template <int NT, int TILES, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void ffn_gate_up_fused_kernel(FfnParams p) {
  constexpr int RS = 32 * NT + 1;
  constexpr int NMAT = 2 * TILES;                        // gate tiles, then up tiles
  constexpr int kWaveBytes = kStages * NMAT * kChunkBytes;
  constexpr int kThreads = WAVES * 64;
  __shared__ __attribute__((aligned(1024))) unsigned char smem[WAVES * kWaveBytes];
  static_assert(NMAT * kTileRows * RS * 4 <= kWaveBytes, "a wavefront's partial tiles fit its own stages");

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int l32 = lane & 31, g = lane >> 5;
  const int R = p.tile_rows;
  int c0[TILES];
#pragma unroll
  for (int s = 0; s < TILES; ++s) c0[s] = min((blockIdx.x * TILES + s) * R, p.d_ff - R);
  unsigned char* stage = smem + wave * kWaveBytes;
  const int64_t row_bytes = (int64_t)p.d_model * 2;

  floatx16 acc[NMAT][NT];
#pragma unroll
  for (int mat = 0; mat < NMAT; ++mat)
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[mat][t][v] = 0.f;
  {
    const char* rows[NMAT];
#pragma unroll
    for (int s = 0; s < TILES; ++s) {
      rows[s] = static_cast<const char*>(p.w_gate) + (int64_t)c0[s] * row_bytes;
      rows[TILES + s] = static_cast<const char*>(p.w_up) + (int64_t)c0[s] * row_bytes;
    }
    const char* const(&crows)[NMAT] = rows;
    walk_tile<NT, NMAT>(p, crows, [=](int r) { return min(r, R - 1); }, static_cast<const char*>(p.x), stage, wave,
                        WAVES, lane, acc);
  }
  // partial tiles [matrix][channel][token] into this wavefront's own stages
  float* red = reinterpret_cast<float*>(stage);
#pragma unroll
  for (int mat = 0; mat < NMAT; ++mat)
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int v = 0; v < 16; ++v)
        red[(mat * kTileRows + 8 * (v >> 2) + 4 * g + (v & 3)) * RS + l32 + 32 * t] = acc[mat][t][v];
  __syncthreads();
  // thread: tile row tid / 8 (+ 8 WAVES per round), tokens (tid % 8) * 4 NT ... + 4 NT
  const int m0 = (tid & 7) * 4 * NT;
  for (int cc = tid >> 3; cc < TILES * kTileRows; cc += kThreads / 8) {
    const int s = cc / kTileRows, c = cc - s * kTileRows;
    if (c >= R) continue;                                 // (the eight threads of a row go together)
    const int ch = c0[s] + c;
    const float bg = p.b_gate ? p.b_gate[ch] : 0.f;
    const float bu = p.b_up ? p.b_up[ch] : 0.f;
    uint64_t bits = 0;
#pragma unroll
    for (int i = 0; i < 4 * NT; ++i) {
      const int m = m0 + i;
      float zg = 0.f, zu = 0.f;
#pragma unroll
      for (int w = 0; w < WAVES; ++w) {
        const float* r = reinterpret_cast<const float*>(smem + w * kWaveBytes);
        zg += r[(s * kTileRows + c) * RS + m];
        zu += r[((TILES + s) * kTileRows + c) * RS + m];
      }
      const float h = activate(zg + bg, p.act);
      const bool on = m < p.M && !(fabsf(h) < p.tau);
      if (on) bits |= 1ull << m;
      const float hu = on ? h * (zu + bu) : 0.f;
      reinterpret_cast<__hip_bfloat16*>(p.h_up)[(int64_t)m * p.d_ff + ch] = __float2bfloat16(hu);
    }
#pragma unroll
    for (int o = 1; o < 8; o <<= 1) {
      const uint32_t lo = __shfl_xor((uint32_t)bits, o, 64), hi = __shfl_xor((uint32_t)(bits >> 32), o, 64);
      bits |= (uint64_t)lo | ((uint64_t)hi << 32);
    }
    if ((tid & 7) == 0) {
      p.rowany[ch] = bits != 0 ? 1 : 0;
      if (p.active) p.active[ch] = bits;
    }
  }
}

// ---- down projection ---------------------------------------------------------------------------
constexpr int kDnWaves = 8;
constexpr int kDnThreads = kDnWaves * 64;
constexpr int kDnCols = 128;                             // output columns per workgroup
constexpr int kDepth = 2;                                // k-steps of 16 channels loaded ahead

template <int NT>
struct DownLoads {
  u32x2 w[8];                                            // four output columns of eight channels
  u32x4 h[NT];                                           // h_up of this lane's token(s) for its eight channels
  uint32_t bits;                                         // which of the step's 16 channels are needed
};

// grid: (d_model / 128, k_splits); block: 512
template <int NT>
__global__ __launch_bounds__(kDnThreads) void ffn_down_kernel(FfnParams p) {
  constexpr int kRedStride = kDnCols + 4;                // floats per token row: keeps rows off each other's banks
  __shared__ __attribute__((aligned(16))) float s_red[kDnWaves][32 * kRedStride];        // [wavefront][token][column]

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int l32 = lane & 31, g = lane >> 5;
  const int n0 = blockIdx.x * kDnCols;
  const int n_steps = p.d_ff / 16;
  const int stride = kDnWaves * p.k_splits;
  const int first = blockIdx.y * kDnWaves + wave;
  const int64_t row_bytes = (int64_t)p.d_model * 2;
  const char* wd = static_cast<const char*>(p.w_down_t) + (int64_t)(n0 + 4 * l32) * 2;
  const char* hu = static_cast<const char*>(p.h_up);

  floatx16 acc[NT][4];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int nt = 0; nt < 4; ++nt)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[t][nt][v] = 0.f;

  // k-slot e of lane half g in step s is channel 16 s + 8 g + e
  auto load_step = [&](int s, DownLoads<NT>& d) {
    d.bits = 0;
    if (s < n_steps) {                                                            // uniform
      const u32x4 any = *reinterpret_cast<const u32x4*>(p.rowany + 16 * s);     // one byte per channel
#pragma unroll
      for (int i = 0; i < 16; ++i) d.bits |= ((any[i >> 2] >> (8 * (i & 3))) & 0xffu) ? (1u << i) : 0u;
    }
    const uint32_t mine = (d.bits >> (8 * g)) & 0xffu;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      u32x2 v = {0u, 0u};
      if ((mine >> e) & 1u)
        v = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(wd + (int64_t)(16 * s + 8 * g + e) * row_bytes));
      d.w[e] = v;
    }
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      u32x4 v = {0u, 0u, 0u, 0u};
      if (d.bits != 0) v = *reinterpret_cast<const u32x4*>(hu + ((int64_t)(l32 + 32 * t) * p.d_ff + 16 * s + 8 * g) * 2);
      d.h[t] = v;
    }
  };
  auto compute_step = [&](const DownLoads<NT>& d) {
    if (d.bits == 0) return;                              // uniform: no channel of the step is needed
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) {
      u32x4 w;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint32_t a = nt < 2 ? d.w[2 * j][0] : d.w[2 * j][1];
        const uint32_t b = nt < 2 ? d.w[2 * j + 1][0] : d.w[2 * j + 1][1];
        w[j] = __builtin_amdgcn_perm(b, a, (nt & 1) ? 0x07060302u : 0x05040100u);
      }
#pragma unroll
      for (int t = 0; t < NT; ++t)
        acc[t][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, w),
                                                             __builtin_bit_cast(bf16x8, d.h[t]), acc[t][nt], 0, 0, 0);
    }
  };

  // software pipeline, kDepth steps ahead (register sets rotate by full unrolling)
  DownLoads<NT> ring[kDepth + 1];
#pragma unroll
  for (int i = 0; i < kDepth; ++i) load_step(first + i * stride, ring[i]);
  for (int s = first; s < n_steps; s += (kDepth + 1) * stride) {
#pragma unroll
    for (int i = 0; i <= kDepth; ++i) {
      load_step(s + (i + kDepth) * stride, ring[(i + kDepth) % (kDepth + 1)]);
      compute_step(ring[i]);
    }
  }

  // Every wavefront parks the rows of the real tokens (32 token columns at a time) in LDS; after
  // one barrier the 512 threads add the eight wavefronts' values in wavefront order and write
  // the slice's partial sums as whole rows.
  // value v of a lane: output column n0 + 4 (8 (v / 4) + 4 g + v % 4) + nt, token l32 (+ 32 t)
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    if (t > 0) __syncthreads();                           // the round before has been read
    if (l32 + 32 * t < p.M) {
      float* row = &s_red[wave][l32 * kRedStride];
#pragma unroll
      for (int v = 0; v < 16; ++v)
        *reinterpret_cast<float4*>(row + 4 * (8 * (v >> 2) + 4 * g + (v & 3))) =
            make_float4(acc[t][0][v], acc[t][1][v], acc[t][2][v], acc[t][3][v]);
    }
    __syncthreads();
    const int rows = min(p.M - 32 * t, 32);
    for (int i = tid; i < rows * (kDnCols / 4); i += kDnThreads) {
      const int m = i / (kDnCols / 4), c4 = i - m * (kDnCols / 4);
      float4 sum = *reinterpret_cast<const float4*>(&s_red[0][m * kRedStride + 4 * c4]);
#pragma unroll
      for (int w = 1; w < kDnWaves; ++w) {
        const float4 o = *reinterpret_cast<const float4*>(&s_red[w][m * kRedStride + 4 * c4]);
        sum.x += o.x; sum.y += o.y; sum.z += o.z; sum.w += o.w;
      }
      *reinterpret_cast<float4*>(p.partial + ((int64_t)blockIdx.y * p.M + 32 * t + m) * p.d_model + n0 + 4 * c4) = sum;
    }
  }
}

// y = bf16(sum over slices of partial + b_down); grid: ceil(M * d_model / (4 * 256))
__global__ __launch_bounds__(256) void ffn_reduce_kernel(FfnParams p) {
  const int64_t i4 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
  const int64_t total = (int64_t)p.M * p.d_model;
  if (i4 >= total) return;
  const int n = (int)(i4 % p.d_model);
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  // eight slices requested before the first is added (one after the other, every slice costs a
  // trip to memory); added in slice order
  for (int k0 = 0; k0 < p.k_splits; k0 += 8) {
    float4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u)
      v[u] = *reinterpret_cast<const float4*>(p.partial + (int64_t)min(k0 + u, p.k_splits - 1) * total + i4);
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (k0 + u < p.k_splits) { s.x += v[u].x; s.y += v[u].y; s.z += v[u].z; s.w += v[u].w; }
  }
  if (p.b_down) {
    const float4 b = *reinterpret_cast<const float4*>(p.b_down + n);
    s.x += b.x; s.y += b.y; s.z += b.z; s.w += b.w;
  }
  u32x2 o = {pack_bf16(s.x, s.y), pack_bf16(s.z, s.w)};
  *reinterpret_cast<u32x2*>(static_cast<char*>(p.y) + i4 * 2) = o;
}

}  // namespace

// Channels per tile of the fused walk: one workgroup per compute unit runs at a time, so the
// cost is (rounds of 256 workgroups) x (rows per tile); the largest multiple of four that
// minimises it.
int ffn_fused_tile_rows(int d_ff, int M) {
  const int per_wg = M <= 32 ? 1 : 2;                     // channel tiles per workgroup
  int best = kTileRows;
  int64_t best_cost = -1;
  for (int r = kTileRows; r >= 16; r -= 4) {
    const int64_t wgs = ((d_ff + r - 1) / r + per_wg - 1) / per_wg;
    const int64_t cost = ((wgs + 255) / 256) * r;
    if (best_cost < 0 || cost < best_cost) { best_cost = cost; best = r; }
  }
  return best;
}

int ffn_k_splits(int d_model, int d_ff) {
  const int n_tiles = d_model / kDnCols;
  int ks = 256 / (n_tiles > 0 ? n_tiles : 1);                                     // one workgroup per compute unit
  const int max_ks = d_ff / (16 * kDnWaves) > 0 ? d_ff / (16 * kDnWaves) : 1;   // at least one step per wavefront
  if (ks > max_ks) ks = max_ks;
  return ks < 1 ? 1 : ks;
}

hipError_t launch_sparse_ffn(const FfnParams& p, hipStream_t st) {
  const dim3 gu(p.d_ff / kTileRows);
  if (p.fused_walk) {
    const int tiles = (p.d_ff + p.tile_rows - 1) / p.tile_rows;
    if (p.M <= 32) hipLaunchKernelGGL((ffn_gate_up_fused_kernel<1, 1, 4>), dim3(tiles), dim3(256), 0, st, p);
    else hipLaunchKernelGGL((ffn_gate_up_fused_kernel<2, 2, 2>), dim3((tiles + 1) / 2), dim3(128), 0, st, p);
  } else {
    if (p.M <= 32) hipLaunchKernelGGL(ffn_gate_up_kernel<1>, gu, dim3(kGuThreads), 0, st, p);
    else hipLaunchKernelGGL(ffn_gate_up_kernel<2>, gu, dim3(kGuThreads), 0, st, p);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  dim3 gd(p.d_model / kDnCols, p.k_splits);
  if (p.M <= 32) hipLaunchKernelGGL(ffn_down_kernel<1>, gd, dim3(kDnThreads), 0, st, p);
  else hipLaunchKernelGGL(ffn_down_kernel<2>, gd, dim3(kDnThreads), 0, st, p);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int64_t quads = ((int64_t)p.M * p.d_model + 3) / 4;
  hipLaunchKernelGGL(ffn_reduce_kernel, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, st, p);
  return hipGetLastError();
}

}  // namespace svf
