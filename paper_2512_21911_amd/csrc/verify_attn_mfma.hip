// Verification attention, matrix-core kernel: bf16 inputs, head dimension 128 (Sec. 3.1 / 3.3:
// the draft queries attend to the retrieved blocks of their KV head and, through the draft
// mask, to each other).
//
// Shape of the work.  For one (sequence, KV head) the gamma x G query rows that share the KV
// head are packed into M = gamma * G rows (row = draft * G + head-in-group) so that every
// selected key/value is read from HBM once and used by all of them.  The selected tokens
// (plus the draft tokens) are cut into 32-token tiles; tile t belongs to wavefront t mod NW,
// NW = 4 * n_splits wavefronts per pair (4 per workgroup).  The launch is sized so that a
// wavefront owns at most kMaxTiles tiles, i.e. every byte the kernel will ever read is
// requested within the first microsecond: the kernel is a single HBM burst followed by a
// merge, which is what a 34 MB problem on an 8 TB/s part needs.
//
// Data path.  A wavefront resolves the addresses of all its tiles first (selected block id ->
// page table -> row offset), then streams K and V rows straight into LDS with 16-byte
// direct-to-LDS loads (no registers in between; two 16 KB stages per wavefront, private to it,
// so no workgroup barrier is needed in the main loop).  The 16-byte chunks of a row are placed
// at an XOR-swizzled position (chosen on the global-address side, since the LDS side of such
// a load is fixed by the lane id) which makes the fragment reads below bank-conflict free.
//
// Math.  Both products run on the matrix cores in transposed form so that a query row lives
// in a fixed lane (lane mod 32) from the first MFMA to the final store:
//   S^T[token][row] = K[token][:] . Q[row][:]       A = K tile (LDS, ds_read_b128), B = Q (registers)
//   O^T[dim][row]  += V^T[dim][token] P^T[token][row]   A = V tile (LDS, 8-byte reads + byte
//                                                    permutes = transpose), B = P (registers)
// The row maximum / denominator therefore need one cross-lane step (lanes l and l+32) per tile
// and the rescale of O is a per-lane scalar.  Softmax runs in the log2 domain in fp32; P is
// rounded to bf16 for the second product, accumulators are fp32.
//
// Merge.  The four wavefronts of a workgroup combine through LDS (log-sum-exp rule); with more
// than one split per pair the workgroup writes an unnormalised fp32 partial and the last
// workgroup to arrive for that pair (atomic ticket) merges all splits and writes out / lse,
// so the whole call is a single launch.
#include <hip/hip_bf16.h>

#include "svf_device.h"

namespace svf {

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = 4;
constexpr int kTile = 32;            // tokens per tile
constexpr int kD = 128;              // head dimension
constexpr int kRowBytes = kD * 2;    // one bf16 K/V row
constexpr int kTileBytes = kTile * kRowBytes;          // 8 KB: K (or V) part of a stage
constexpr int kMaxTiles = 4;         // tiles a wavefront may own
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;

#define SVF_GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void*)(p))
#define SVF_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))

// s_waitcnt with only the vector-memory counter constrained (gfx9 encoding:
// vmcnt = bits [3:0] and [15:14], expcnt [6:4], lgkmcnt [11:8]).
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (0x7 << 4) | (0xF << 8));
  asm volatile("" ::: "memory");
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  // round to nearest even
  uint32_t a = __float_as_uint(lo), b = __float_as_uint(hi);
  a += 0x7fffu + ((a >> 16) & 1u);
  b += 0x7fffu + ((b >> 16) & 1u);
  return (a >> 16) | (b & 0xffff0000u);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// LDS: two stages of one K tile and one V tile per wavefront.  The four arrays are separate
// objects on purpose: the compiler then knows which outstanding direct-to-LDS loads a given
// LDS read can depend on, and waits for those only.  After the main loop array w is reused as
// wavefront w's fp32 output buffer for the in-workgroup merge.
constexpr int kArrayBytes = kWaves * kTileBytes;      // 32 KB
static_assert(kArrayBytes >= 64 * kD * 4, "one array holds a wavefront's 64 x 128 fp32 output");

// grid: (n_splits, Hkv, B * row_groups); block: 256
template <int RT>
__global__ __launch_bounds__(kThreads) void verify_attn_mfma_kernel(AttnParams p, int row_groups) {
  __shared__ __attribute__((aligned(1024))) unsigned char sK0[kArrayBytes];
  __shared__ __attribute__((aligned(1024))) unsigned char sV0[kArrayBytes];
  __shared__ __attribute__((aligned(1024))) unsigned char sK1[kArrayBytes];
  __shared__ __attribute__((aligned(1024))) unsigned char sV1[kArrayBytes];
  __shared__ float sm_m[kWaves][64];
  __shared__ float sm_l[kWaves][64];

  const int split = blockIdx.x, h = blockIdx.y;
  const int b = blockIdx.z / row_groups, rg = blockIdx.z - b * row_groups;
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int l32 = lane & 31, g = lane >> 5;
  const int pair = b * p.Hkv + h;
  constexpr int ROWS = 32 * RT;
  const int row0 = rg * ROWS;

  const int L = clamped_len(p.seq_lens, b, p.max_seq_len);
  const int cnt = min(max(p.sel_cnt[pair], 0), p.k_blocks);
  const int32_t* __restrict__ sel = p.sel_idx + (int64_t)pair * p.k_blocks;
  const int n_prefix = cnt * p.block_size;
  const int tiles_d = (p.gamma + kTile - 1) / kTile;           // draft tiles come first
  const int tiles = tiles_d + (n_prefix + kTile - 1) / kTile;
  const int NW = kWaves * p.n_splits;
  const int gw = split * kWaves + wave;

  const __hip_bfloat16* Kc = static_cast<const __hip_bfloat16*>(p.K);
  const __hip_bfloat16* Vc = static_cast<const __hip_bfloat16*>(p.V);
  const __hip_bfloat16* Kd = static_cast<const __hip_bfloat16*>(p.k_draft);
  const __hip_bfloat16* Vd = static_cast<const __hip_bfloat16*>(p.v_draft);

  // ---- resolve the addresses of all tiles this wavefront owns --------------------------------
  // Written without branches around the loads so that the (up to four) block-id loads go out
  // together, then the page-table loads: two memory round trips instead of eight.
  // Rows are 16-byte aligned, so bit 0 of an element offset is free to say "relative to the
  // draft arrays" (set) or "relative to the cache pools" (clear).
  const int64_t safe_off = (((int64_t)b * p.gamma * p.Hkv + h) * kD) | 1;   // draft 0: always readable
  int n_my = 0;
  bool t_draft[kMaxTiles], t_ok[kMaxTiles];
  int t_blk[kMaxTiles], t_in[kMaxTiles];
#pragma unroll
  for (int u = 0; u < kMaxTiles; ++u) {
    const int t = gw + u * NW;
    if (t < tiles) n_my = u + 1;
    t_draft[u] = t < tiles_d;
    const int slot = (t - tiles_d) * kTile + l32;
    t_ok[u] = t < tiles && !t_draft[u] && slot < n_prefix;
    const int sl = t_ok[u] ? slot : 0;
    const int bi = p.block_shift >= 0 ? sl >> p.block_shift : sl / p.block_size;
    t_in[u] = sl - bi * p.block_size;
    t_blk[u] = sel[bi];                                  // bi < k_blocks always
  }
  int t_phys[kMaxTiles], t_slot[kMaxTiles];
#pragma unroll
  for (int u = 0; u < kMaxTiles; ++u) {
    int tok = t_blk[u] * p.block_size + t_in[u];
    t_ok[u] = t_ok[u] && t_blk[u] >= 0 && tok < L;
    tok = t_ok[u] ? tok : 0;
    if (p.kv.page_size == 0) {
      t_phys[u] = b;
      t_slot[u] = tok;
    } else {
      const int pg = p.kv.page_shift >= 0 ? tok >> p.kv.page_shift : tok / p.kv.page_size;
      t_slot[u] = tok - pg * p.kv.page_size;
      t_phys[u] = p.table[(int64_t)b * p.kv.max_pages + pg];   // pg = 0 for invalid slots
    }
  }
  int64_t t_off[kMaxTiles];
  uint32_t t_valid[kMaxTiles];
#pragma unroll
  for (int u = 0; u < kMaxTiles; ++u) {
    const int t = gw + u * NW;
    int64_t off = safe_off;
    bool ok = t_ok[u];
    if (ok) off = (int64_t)t_phys[u] * p.kv.stride_page + (int64_t)t_slot[u] * p.kv.stride_tok +
                  (int64_t)h * p.kv.stride_head;
    if (t_draft[u]) {
      const int di = t * kTile + l32;
      ok = di < p.gamma;
      if (ok) off = ((((int64_t)b * p.gamma + di) * p.Hkv + h) * kD) | 1;
    }
    // invalid slots read the (finite, always mapped) first draft row and are masked out below
    t_off[u] = off;
    t_valid[u] = (uint32_t)__ballot(ok);
  }

  // ---- queries of this lane's rows as B operands, and the rows' draft masks -------------------
  bf16x8 qf[RT][8];
  uint64_t rmask[RT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    const int row = row0 + rt * 32 + l32;
    const bool ok = row < p.M;
    const int i = ok ? row / p.G : 0;
    const int j = h * p.G + (ok ? row - i * p.G : 0);
    const __hip_bfloat16* qrow =
        static_cast<const __hip_bfloat16*>(p.q) + (((int64_t)b * p.gamma + i) * p.Hq + j) * kD + g * 8;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qf[rt][ks] = *reinterpret_cast<const bf16x8*>(qrow + ks * 16);
    uint64_t m = 0;
    if (ok) {
      if (p.draft_mask) m = p.draft_mask[p.mask_per_batch ? (int64_t)b * p.gamma + i : i];
      else m = i >= 63 ? ~0ull : ((2ull << i) - 1ull);
    }
    rmask[rt] = m;
  }

  // chunk swizzle: 16-byte chunk c of the row in tile slot s sits at position c ^ (s & 15)
  auto issue_tile = [&](int64_t my_off, unsigned char* kdst, unsigned char* vdst) {
    const int pos = lane & 15;
#pragma unroll
    for (int n = 0; n < 8; ++n) {
      const int s = 4 * n + (lane >> 4);                 // slot of this lane in load n
      const int64_t off = __shfl(my_off, s, 64);
      const int c = pos ^ (s & 15);
      const bool from_draft = off & 1;
      const int64_t o = (off & ~(int64_t)1) + c * 8;
      const __hip_bfloat16* ksrc = (from_draft ? Kd : Kc) + o;
      const __hip_bfloat16* vsrc = (from_draft ? Vd : Vc) + o;
      __builtin_amdgcn_global_load_lds(SVF_GLOBAL_PTR(ksrc), SVF_LDS_PTR(kdst + n * 1024), 16, 0, 0);
      __builtin_amdgcn_global_load_lds(SVF_GLOBAL_PTR(vsrc), SVF_LDS_PTR(vdst + n * 1024), 16, 0, 0);
    }
  };
  unsigned char* const myK0 = sK0 + wave * kTileBytes;
  unsigned char* const myV0 = sV0 + wave * kTileBytes;
  unsigned char* const myK1 = sK1 + wave * kTileBytes;
  unsigned char* const myV1 = sV1 + wave * kTileBytes;

  // ---- main loop ---------------------------------------------------------------------------
  float m_run[RT], l_run[RT];
  floatx16 oacc[RT][4];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    m_run[rt] = -INFINITY;
    l_run[rt] = 0.f;
#pragma unroll
    for (int nt = 0; nt < 4; ++nt)
#pragma unroll
      for (int v = 0; v < 16; ++v) oacc[rt][nt][v] = 0.f;
  }

  if (n_my > 0) issue_tile(t_off[0], myK0, myV0);
  if (n_my > 1) issue_tile(t_off[1], myK1, myV1);

#pragma unroll
  for (int u = 0; u < kMaxTiles; ++u) {
    if (u < n_my) {
      // the 16 loads of tile u are followed by at most the 16 loads of tile u + 1
      if (u + 1 < n_my) wait_vmcnt<16>(); else wait_vmcnt<0>();
      const unsigned char* kt = (u & 1) ? myK1 : myK0;
      const unsigned char* vt = (u & 1) ? myV1 : myV0;

      // S^T = K Q^T : token = l32 (A rows), row = l32 (B cols)
      floatx16 sacc[RT];
#pragma unroll
      for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int v = 0; v < 16; ++v) sacc[rt][v] = 0.f;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const int c = 2 * ks + g;
        const bf16x8 kf = *reinterpret_cast<const bf16x8*>(kt + l32 * kRowBytes + ((c ^ (l32 & 15)) << 4));
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
          sacc[rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[rt][ks], sacc[rt], 0, 0, 0);
      }

      // online softmax; value v of a lane is token 8*(v/4) + 4*g + v%4 of the tile
      const int draft_base = (gw + u * NW) * kTile;       // first draft index of a draft tile
      bf16x8 pf[RT][2];
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) {
        uint32_t allowed = t_valid[u];
        if (t_draft[u]) allowed &= (uint32_t)(rmask[rt] >> (draft_base & 63));
        float sc[16];
        float mx = -INFINITY;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int tok = 8 * (v >> 2) + 4 * g + (v & 3);
          const bool vis = (allowed >> tok) & 1u;
          sc[v] = vis ? sacc[rt][v] * p.scale_log2 : -INFINITY;
          mx = fmaxf(mx, sc[v]);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m_run[rt], mx);
        const float m_use = m_new == -INFINITY ? 0.f : m_new;
        const float alpha = fast_exp2(m_run[rt] - m_use);
        float ls = 0.f;
        float pe[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          pe[v] = fast_exp2(sc[v] - m_use);
          ls += pe[v];
        }
        l_run[rt] = l_run[rt] * alpha + ls;
        m_run[rt] = m_new;
#pragma unroll
        for (int nt = 0; nt < 4; ++nt)
#pragma unroll
          for (int v = 0; v < 16; ++v) oacc[rt][nt][v] *= alpha;
#pragma unroll
        for (int ks2 = 0; ks2 < 2; ++ks2) {
          u32x4 w;
#pragma unroll
          for (int j = 0; j < 4; ++j) w[j] = pack_bf16(pe[8 * ks2 + 2 * j], pe[8 * ks2 + 2 * j + 1]);
          pf[rt][ks2] = __builtin_bit_cast(bf16x8, w);
        }
      }

      // O^T += V^T P^T : A row i = l32 carries dims 4*i + nt, k-slot e of group g is token
      // 16*ks2 + 8*(e/4) + 4*g + e%4
#pragma unroll
      for (int ks2 = 0; ks2 < 2; ++ks2) {
        uint2 x[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int tok = 16 * ks2 + 8 * (e >> 2) + 4 * g + (e & 3);
          const int c = l32 >> 1;
          x[e] = *reinterpret_cast<const uint2*>(vt + tok * kRowBytes + ((c ^ (tok & 15)) << 4) + ((l32 & 1) << 3));
        }
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) {
          u32x4 w;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const uint32_t a = nt < 2 ? x[2 * j].x : x[2 * j].y;
            const uint32_t c2 = nt < 2 ? x[2 * j + 1].x : x[2 * j + 1].y;
            w[j] = __builtin_amdgcn_perm(c2, a, (nt & 1) ? 0x07060302u : 0x05040100u);
          }
          const bf16x8 vf = __builtin_bit_cast(bf16x8, w);
#pragma unroll
          for (int rt = 0; rt < RT; ++rt)
            oacc[rt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[rt][ks2], oacc[rt][nt], 0, 0, 0);
        }
      }

      // refill this stage with the tile after next
      if (u + 2 < kMaxTiles && u + 2 < n_my) {
        if (u & 1) issue_tile(t_off[u + 2 < kMaxTiles ? u + 2 : 0], myK1, myV1);
        else issue_tile(t_off[u + 2 < kMaxTiles ? u + 2 : 0], myK0, myV0);
      }
    }
  }

  // ---- combine the four wavefronts through LDS ---------------------------------------------
  // Wavefront w parks its rescaled fp32 output in array w as [ROWS][32 float4]; float4 chunk c4
  // of row r sits at position c4 ^ (r & 31), which keeps both the row-per-lane writes and the
  // chunk-per-lane reads off each other's banks.
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) l_run[rt] += __shfl_xor(l_run[rt], 32, 64);
  if (g == 0) {
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      sm_m[wave][rt * 32 + l32] = m_run[rt];
      sm_l[wave][rt * 32 + l32] = l_run[rt];
    }
  }
  __syncthreads();                       // every wavefront is done with its K/V stages
  float4* const obuf[kWaves] = {reinterpret_cast<float4*>(sK0), reinterpret_cast<float4*>(sV0),
                                reinterpret_cast<float4*>(sK1), reinterpret_cast<float4*>(sV1)};
  {
    float4* mine = wave == 0 ? obuf[0] : wave == 1 ? obuf[1] : wave == 2 ? obuf[2] : obuf[3];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      const int r = rt * 32 + l32;
      float mw = -INFINITY;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) mw = fmaxf(mw, sm_m[w][r]);
      const float f = m_run[rt] == -INFINITY ? 0.f : fast_exp2(m_run[rt] - mw);
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int i = 8 * (v >> 2) + 4 * g + (v & 3);      // dims 4*i .. 4*i+3
        mine[r * 32 + (i ^ l32)] =
            make_float4(oacc[rt][0][v] * f, oacc[rt][1][v] * f, oacc[rt][2][v] * f, oacc[rt][3][v] * f);
      }
    }
  }
  __syncthreads();

  // 256 threads: thread -> (row, float4 chunk); ROWS * 32 float4 in total
  const int64_t part_row0 = ((int64_t)pair * p.n_splits + split) * p.Mpad + row0;
  for (int e = tid; e < ROWS * (kD / 4); e += kThreads) {
    const int r = e >> 5, c4 = e & 31;
    float mw = -INFINITY;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) mw = fmaxf(mw, sm_m[w][r]);
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    float lw = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const float4 t = obuf[w][r * 32 + (c4 ^ (r & 31))];
      acc.x += t.x; acc.y += t.y; acc.z += t.z; acc.w += t.w;
      const float mwv = sm_m[w][r];
      lw += mwv == -INFINITY ? 0.f : sm_l[w][r] * fast_exp2(mwv - mw);
    }
    if (row0 + r < p.Mpad) {
      *reinterpret_cast<float4*>(p.part_o + (part_row0 + r) * kD + 4 * c4) = acc;
      if (c4 == 0) {
        p.part_m[part_row0 + r] = mw;
        p.part_l[part_row0 + r] = lw;
      }
    }
  }
}

}  // namespace

hipError_t launch_merge_splits(const AttnParams& p, int dtype, hipStream_t st);

bool mfma_supported(const svf_shape_t& s) { return s.dtype == SVF_BF16 && s.d == 128; }

// Splits per (sequence, KV head, row group): enough workgroups to cover the 256 compute units,
// never more than kMaxTiles tiles per wavefront, never less than one tile per wavefront.
int mfma_splits(const svf_shape_t& s) {
  const int M = s.gamma * (s.Hq / s.Hkv);
  const int rows = M <= 32 ? 32 : 64;
  const int64_t groups = (int64_t)s.B * s.Hkv * ((M + rows - 1) / rows);
  const int64_t tiles = ((int64_t)s.k_blocks * s.block_size + kTile - 1) / kTile + (s.gamma + kTile - 1) / kTile;
  int64_t lo = (tiles + kWaves * kMaxTiles - 1) / (kWaves * kMaxTiles);
  int64_t hi = (tiles + kWaves - 1) / kWaves;
  int64_t want = (256 + groups - 1) / groups;
  if (want < lo) want = lo;
  if (want > hi) want = hi;
  return (int)want;
}

hipError_t launch_verify_attn_mfma(const AttnParams& p, hipStream_t st) {
  const int rows = p.M <= 32 ? 32 : 64;
  const int row_groups = (p.M + rows - 1) / rows;
  dim3 grid(p.n_splits, p.Hkv, p.B * row_groups);
  hipError_t e;
  if (rows == 32)
    hipLaunchKernelGGL(verify_attn_mfma_kernel<1>, grid, dim3(kThreads), 0, st, p, row_groups);
  else
    hipLaunchKernelGGL(verify_attn_mfma_kernel<2>, grid, dim3(kThreads), 0, st, p, row_groups);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  return launch_merge_splits(p, SVF_BF16, st);
}

}  // namespace svf
