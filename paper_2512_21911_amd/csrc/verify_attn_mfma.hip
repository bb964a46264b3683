// Verification attention, matrix-core kernel: bf16 inputs, head dimension 128 (Sec. 3.1 / 3.3:
// the draft queries attend to the retrieved blocks of their KV head and, through the draft
// mask, to each other).
//
// Shape of the work.  For one (sequence, KV head) the gamma x G query rows that share the KV
// head are packed into M = gamma * G rows (row = draft * G + head-in-group), 32 rows per
// workgroup, so that every selected key/value is read from HBM once and used by all of them
// (with more than 32 rows the row groups of a pair run on one XCD and share its L2).  The selected tokens
// (plus the draft tokens) are cut into 32-token tiles; tile t belongs to wavefront t mod NW,
// NW = 4 * n_splits wavefronts per pair (4 per workgroup).  The launch is sized so that a
// wavefront owns at most kMaxTiles tiles, i.e. every byte the kernel will ever read is
// requested as early as the memory system accepts it: the kernel is one HBM burst followed by
// a merge, which is what a 34 MB problem on an 8 TB/s part needs.
//
// Data path.  A wavefront resolves the addresses of all its tiles first (selected block id ->
// page table -> row offset), then streams K and V rows straight into LDS with 16-byte
// direct-to-LDS loads (no registers in between; two 16 KB stages per wavefront, private to it,
// so the main loop needs no workgroup barrier).  The 16-byte chunks of a row are placed at an
// XOR-swizzled position (chosen on the global-address side, since the LDS side of such a load
// is fixed by the lane id) which keeps the fragment reads below off each other's banks.
// The LDS reads of the main loop are issued by hand (inline ds_read + explicit waits): the
// compiler would otherwise wait for every outstanding direct-to-LDS load before any LDS read
// and serialise the two stages.
//
// Math.  Both products run on the matrix cores in transposed form so that a query row lives
// in a fixed lane (lane mod 32) from the first MFMA to the final store:
//   S^T[token][row] = K[token][:] . Q[row][:]           A = K tile (LDS, 16-byte reads), B = Q (registers)
//   O^T[dim][row]  += V^T[dim][token] P^T[token][row]   A = V tile (LDS, 8-byte reads + byte
//                                                       permutes = transpose), B = P (registers)
// The row maximum / denominator therefore need one cross-lane step (lanes l and l+32) per tile
// and the rescale of O is a per-lane scalar, applied only when the maximum moved by more than
// kRescaleGap (the stale maximum is kept otherwise; the final division makes this exact).
// Softmax runs in the log2 domain in fp32; P is rounded to bf16 (hardware RNE) for the second
// product; accumulators are fp32.
//
// Merge.  The four wavefronts of a workgroup combine through LDS (log-sum-exp rule).  With one
// split per pair the workgroup writes out / lse itself.  Otherwise it writes an unnormalised
// fp32 partial, and the last workgroup to arrive for that pair (atomic ticket, release /
// acquire fences at device scope) merges all splits: the whole call is a single launch.
// Workgroup ids are mapped so that all splits of a pair share id mod 8, which on this part
// places them on one XCD, i.e. the partials normally never leave that XCD's L2.
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
constexpr int kStageBytes = 2 * kTileBytes;            // K then V
constexpr int kWaveLds = 2 * kStageBytes;              // two stages per wavefront: 32 KB
constexpr int kMaxTiles = 4;         // tiles a wavefront may own
constexpr int kXcds = 8;
constexpr float kRescaleGap = 8.0f;  // log2 units the running maximum may lag behind

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float floatx2;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
typedef __attribute__((__vector_size__(2 * sizeof(uint32_t)))) uint32_t u32x2;

#define SVF_GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void*)(p))
#define SVF_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))

// s_waitcnt with only the vector-memory counter constrained (gfx9 encoding:
// vmcnt = bits [3:0] and [15:14], expcnt [6:4], lgkmcnt [11:8]).
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (0x7 << 4) | (0xF << 8));
  asm volatile("" ::: "memory");
}

// Hand-issued LDS reads.  The value is not valid until lds_wait8() has been given the register.
template <int OFF>
__device__ __forceinline__ u32x4 lds_read16(uint32_t addr) {
  u32x4 v;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF) : "memory");
  return v;
}
template <int OFF>
__device__ __forceinline__ u32x2 lds_read8(uint32_t addr) {
  u32x2 v;
  asm volatile("ds_read_b64 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF) : "memory");
  return v;
}
// Waits for all LDS reads; the registers pass through the statement so that no use of them can
// be scheduled above the wait.
template <typename T>
__device__ __forceinline__ void lds_wait8(T (&r)[8]) {
  asm volatile("s_waitcnt lgkmcnt(0)"
               : "+v"(r[0]), "+v"(r[1]), "+v"(r[2]), "+v"(r[3]), "+v"(r[4]), "+v"(r[5]), "+v"(r[6]), "+v"(r[7])
               :
               : "memory");
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  const floatx2 f = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));   // round to nearest even
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Stores of data exchanged between workgroups.  A relaxed atomic store at device scope compiles
// to a write-through store, so making it visible across the chip's L2 slices needs no bulk
// write-back, only a wait for the store's acknowledgement.
__device__ __forceinline__ void store_coherent16(void* p, u32x4 bits) {
  // the 16-byte form of the same device-scope write-through store
  asm volatile("global_store_dwordx4 %0, %1, off sc1" : : "v"(p), "v"(bits) : "memory");
}
__device__ __forceinline__ void store_coherent2(float* p, float a, float b) {
  const uint64_t bits = (uint64_t)__float_as_uint(a) | ((uint64_t)__float_as_uint(b) << 32);
  __hip_atomic_store(reinterpret_cast<uint64_t*>(p), bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// One 32-token tile against RT row tiles.  krel / vrel: this lane's byte offsets of its K
// fragments (8 k-steps) and V rows (8 k-slots) inside a stage; stage: LDS address of the stage.
template <int RT, bool FIRST>
__device__ __forceinline__ void process_tile(uint32_t stage, const uint32_t (&krel)[8], const uint32_t (&vrel)[8],
                                             const bf16x8 (&qf)[RT][8], const uint32_t (&allowed)[RT],
                                             bool all_visible, float scale_log2, int g,
                                             float (&m_run)[RT], float (&l_run)[RT], floatx16 (&oacc)[RT][4]) {
  // K fragments, then the first half of the V rows (they land while the S MFMAs run)
  u32x4 kf[8];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) kf[ks] = lds_read16<0>(stage + krel[ks]);
  lds_wait8(kf);
  u32x2 x0[8], x1[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) x0[e] = lds_read8<kTileBytes>(stage + vrel[e]);

  // S^T = K Q^T : token = lane mod 32 (A rows), query row = lane mod 32 (B columns)
  floatx16 sacc[RT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
#pragma unroll
    for (int v = 0; v < 16; ++v) sacc[rt][v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
      sacc[rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kf[ks]), qf[rt][ks],
                                                         sacc[rt], 0, 0, 0);
  }

  // online softmax; value v of a lane is token 8*(v/4) + 4*g + v%4 of the tile
  bf16x8 pf[RT][2];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    // invisible tokens drop out by setting their raw score to -inf (the scale is positive)
    if (!all_visible) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int tok = 8 * (v >> 2) + 4 * g + (v & 3);
        if (!((allowed[rt] >> tok) & 1u)) sacc[rt][v] = -INFINITY;
      }
    }
    float mx = sacc[rt][0];
#pragma unroll
    for (int v = 1; v < 16; ++v) mx = fmaxf(mx, sacc[rt][v]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * scale_log2;
    // keep the old reference while the maximum has not run away from it
    float m_ref = m_run[rt];
    if (FIRST) {
      m_ref = mx;
    } else {
      const bool move = mx > m_ref + kRescaleGap;
      if (__any(move)) {
        const float m_new = move ? mx : m_ref;
        const float alpha = m_new == m_ref ? 1.0f : fast_exp2(m_ref - m_new);   // -inf - finite -> 0
        l_run[rt] *= alpha;
#pragma unroll
        for (int nt = 0; nt < 4; ++nt)
#pragma unroll
          for (int v = 0; v < 16; ++v) oacc[rt][nt][v] *= alpha;
        m_ref = m_new;
      }
    }
    m_run[rt] = m_ref;
    const float m_use = m_ref == -INFINITY ? 0.f : m_ref;
    float ls = 0.f;
    float pe[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      pe[v] = fast_exp2(__builtin_fmaf(sacc[rt][v], scale_log2, -m_use));
      ls += pe[v];
    }
    l_run[rt] += ls;
#pragma unroll
    for (int ks2 = 0; ks2 < 2; ++ks2) {
      u32x4 w;
#pragma unroll
      for (int j = 0; j < 4; ++j) w[j] = pack_bf16(pe[8 * ks2 + 2 * j], pe[8 * ks2 + 2 * j + 1]);
      pf[rt][ks2] = __builtin_bit_cast(bf16x8, w);
    }
  }

  // O^T += V^T P^T : A row i = lane mod 32 carries dims 4*i + nt; k-slot e of lane group g is
  // token 16*ks2 + 8*(e/4) + 4*g + e%4.  x[e] holds dims 4*i .. 4*i+3 of that token.
  lds_wait8(x0);
#pragma unroll
  for (int e = 0; e < 8; ++e) x1[e] = lds_read8<kTileBytes + 16 * kRowBytes>(stage + vrel[e]);
#pragma unroll
  for (int ks2 = 0; ks2 < 2; ++ks2) {
    if (ks2 == 1) lds_wait8(x1);
    const u32x2(&x)[8] = ks2 == 0 ? x0 : x1;
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) {
      u32x4 w;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint32_t a = nt < 2 ? x[2 * j][0] : x[2 * j][1];
        const uint32_t c2 = nt < 2 ? x[2 * j + 1][0] : x[2 * j + 1][1];
        w[j] = __builtin_amdgcn_perm(c2, a, (nt & 1) ? 0x07060302u : 0x05040100u);
      }
      const bf16x8 vf = __builtin_bit_cast(bf16x8, w);
#pragma unroll
      for (int rt = 0; rt < RT; ++rt)
        oacc[rt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[rt][ks2], oacc[rt][nt], 0, 0, 0);
    }
  }
}

// Partials exchanged between the workgroups of a group: per row (m, l) in fp32 and the
// normalised output o / l in bf16 (its magnitude is bounded by the values' and bf16 is the
// precision of the inputs and of the final output; accumulation stays fp32 on both sides).
// 8-byte load of four such channels (or of an (m, l) pair).  LOCAL: the data is known to sit
// in, or behind, this XCD's L2, so only the per-CU cache has to be bypassed, which is what a
// relaxed atomic load at workgroup scope compiles to; otherwise a plain load (after an acquire).
template <bool LOCAL>
__device__ __forceinline__ uint64_t load_partial8(const void* p) {
  if (LOCAL)
    return __hip_atomic_load(reinterpret_cast<const uint64_t*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  return *reinterpret_cast<const uint64_t*>(p);
}
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// Final merge of a group's split partials by its last workgroup (256 threads): eight threads
// per row, 16 channels each.  All splits, the workgroup's own included, are read back in split
// order, so the result does not depend on which workgroup happened to arrive last; the loads of
// kMergeBatch splits are all in flight before the first is used.
template <bool LOCAL>
__device__ __forceinline__ void merge_splits(const AttnParams& p, int64_t g_row, int64_t orow, bool row_ok, int cg) {
  constexpr int kMergeBatch = 8;
  const uint16_t* part_o = reinterpret_cast<const uint16_t*>(p.part_o);
  float acc[16];
#pragma unroll
  for (int c = 0; c < 16; ++c) acc[c] = 0.f;
  float m_acc = -INFINITY, l_acc = 0.f;
  for (int s0 = 0; s0 < p.n_splits; s0 += kMergeBatch) {
    float pm[kMergeBatch], pl[kMergeBatch];
    uint32_t t[kMergeBatch][8];
#pragma unroll
    for (int u = 0; u < kMergeBatch; ++u) {
      // entries past the last split (index clamped) get weight 0 below
      const int64_t pr = g_row + (int64_t)min(s0 + u, p.n_splits - 1) * p.Mpad;
      const uint64_t ml = load_partial8<LOCAL>(p.part_ml + 2 * pr);
      pm[u] = __uint_as_float((uint32_t)ml);
      pl[u] = __uint_as_float((uint32_t)(ml >> 32));
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const uint64_t w = load_partial8<LOCAL>(part_o + pr * kD + cg * 16 + 4 * c);
        t[u][2 * c] = (uint32_t)w;
        t[u][2 * c + 1] = (uint32_t)(w >> 32);
      }
    }
    float mb = m_acc;
#pragma unroll
    for (int u = 0; u < kMergeBatch; ++u) {
      if (s0 + u >= p.n_splits) pm[u] = -INFINITY;
      mb = fmaxf(mb, pm[u]);
    }
    const float fa = m_acc == -INFINITY ? 0.f : fast_exp2(m_acc - mb);
    l_acc *= fa;
#pragma unroll
    for (int c = 0; c < 16; ++c) acc[c] *= fa;
#pragma unroll
    for (int u = 0; u < kMergeBatch; ++u) {
      // weight of split s: exp2(m_s - m) * l_s, applied to its normalised output
      const float w = pm[u] != -INFINITY ? fast_exp2(pm[u] - mb) * pl[u] : 0.f;
      l_acc += w;
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        acc[2 * c] += w * bf16_lo(t[u][c]);
        acc[2 * c + 1] += w * bf16_hi(t[u][c]);
      }
    }
    m_acc = mb;
  }
  if (row_ok) {
    const float inv = 1.0f / l_acc;
    u32x4 o0, o1;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      o0[c] = pack_bf16(acc[2 * c] * inv, acc[2 * c + 1] * inv);
      o1[c] = pack_bf16(acc[8 + 2 * c] * inv, acc[8 + 2 * c + 1] * inv);
    }
    u32x4* dst = reinterpret_cast<u32x4*>(static_cast<__hip_bfloat16*>(p.out) + orow * kD + cg * 16);
    dst[0] = o0;
    dst[1] = o1;
    if (p.lse && cg == 0) p.lse[orow] = (m_acc + log2f(l_acc)) * 0.6931471805599453f;
  }
}

// grid: 1-D, kXcds * ceil(groups / kXcds) * n_splits workgroups, groups = B * Hkv * row_groups
template <int RT>
__global__ __launch_bounds__(kThreads) void verify_attn_mfma_kernel(AttnParams p, int row_groups, int groups) {
  // two stages per wavefront, plus one extra stage for the first draft tile so that the
  // wavefront owning it (wavefront 0 of split 0) still has all its loads in flight at once
  __shared__ __attribute__((aligned(1024))) unsigned char smem[kWaves * kWaveLds + kStageBytes];
  __shared__ float sm_m[kWaves][64];
  __shared__ float sm_l[kWaves][64];
  __shared__ int sm_last;

  // workgroup id -> (group, split): all splits of a group share id mod kXcds
  const int xcd = blockIdx.x % kXcds, slot = blockIdx.x / kXcds;
  const int group = xcd + kXcds * (slot / p.n_splits);
  const int split = slot % p.n_splits;
  if (group >= groups) return;
  // row groups of one pair are `pairs` apart, i.e. on the same XCD whenever pairs is a multiple
  // of eight: the second reader of a pair's K/V then finds them in that XCD's L2
  const int pairs = groups / row_groups;
  const int rg = group / pairs, pair = group - rg * pairs;
  const int b = pair / p.Hkv, h = pair - b * p.Hkv;

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int l32 = lane & 31, g = lane >> 5;
  constexpr int ROWS = 32 * RT;
  const int row0 = rg * ROWS;
  const int NW = kWaves * p.n_splits;
  const int gw = split * kWaves + wave;
  const int tiles_d = (p.gamma + kTile - 1) / kTile;           // draft tiles come first

  const __hip_bfloat16* Kc = static_cast<const __hip_bfloat16*>(p.K);
  const __hip_bfloat16* Vc = static_cast<const __hip_bfloat16*>(p.V);
  const __hip_bfloat16* Kd = static_cast<const __hip_bfloat16*>(p.k_draft);
  const __hip_bfloat16* Vd = static_cast<const __hip_bfloat16*>(p.v_draft);
  const int32_t* __restrict__ sel = p.sel_idx + (int64_t)pair * p.k_blocks;

  // ---- queries of this lane's rows as B operands, and the rows' draft masks -------------------
  // Issued before anything else: vector loads complete in order, so a wait for these must not
  // have the K/V stream in front of it.
  bf16x8 qf[RT][8];
  uint64_t rmask[RT];
  int rdraft[RT];                // draft index of the row, -1 for padding rows
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
    // unconditional load (row 0's entry for padding rows); combined with the causal default
    // only after the stream has been started, so that nothing waits on it here
    const uint64_t* mp = p.draft_mask ? p.draft_mask + (p.mask_per_batch ? (int64_t)b * p.gamma + i : i) : nullptr;
    rmask[rt] = mp ? *mp : 0;
    rdraft[rt] = ok ? i : -1;
  }

  // ---- resolve the addresses of all tiles this wavefront owns --------------------------------
  // Written without branches around the loads so that the (up to four) block-id loads go out
  // together and at once (they do not wait for sel_cnt / seq_lens), then the page-table loads:
  // two memory round trips in front of the K/V stream.
  int t_in[kMaxTiles], t_blk[kMaxTiles];
#pragma unroll
  for (int u = 0; u < kMaxTiles; ++u) {
    const int t = gw + u * NW;
    int slot_p = (t - tiles_d) * kTile + l32;
    slot_p = slot_p < 0 ? 0 : slot_p;
    int bi = p.block_shift >= 0 ? slot_p >> p.block_shift : slot_p / p.block_size;
    t_in[u] = slot_p - bi * p.block_size;
    bi = bi < p.k_blocks ? bi : p.k_blocks - 1;
    t_blk[u] = sel[bi];
  }
  const int L = clamped_len(p.seq_lens, b, p.max_seq_len);
  const int cnt = min(max(p.sel_cnt[pair], 0), p.k_blocks);
  const int n_prefix = cnt * p.block_size;
  const int tiles = tiles_d + (n_prefix + kTile - 1) / kTile;

  int n_my = 0;
  bool t_draft[kMaxTiles], t_ok[kMaxTiles];
  int t_phys[kMaxTiles], t_slot[kMaxTiles];
#pragma unroll
  for (int u = 0; u < kMaxTiles; ++u) {
    const int t = gw + u * NW;
    if (t < tiles) n_my = u + 1;
    t_draft[u] = t < tiles_d;
    const int slot_p = (t - tiles_d) * kTile + l32;
    int tok = t_blk[u] * p.block_size + t_in[u];
    t_ok[u] = t < tiles && !t_draft[u] && slot_p < n_prefix && t_blk[u] >= 0 && tok < L;
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
  // Rows are 16-byte aligned, so bit 0 of an element offset is free to say "relative to the
  // draft arrays" (set) or "relative to the cache pools" (clear).
  const int64_t safe_off = (((int64_t)b * p.gamma * p.Hkv + h) * kD) | 1;   // draft 0: always readable
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

  // chunk swizzle: 16-byte chunk c of the row in tile slot s sits at position c ^ (s & 15)
  unsigned char* const my_lds = smem + wave * kWaveLds;
  // Load n of a tile covers slots 4n .. 4n+3 (16 lanes per slot); a lane fetches the byte address
  // of "its" slot's K row (bit 0: the row is a draft row) from the lane that resolved it.  The
  // shuffles of a tile are issued together, ahead of its loads, so that their LDS round trips
  // overlap instead of sitting between the loads.
  const int64_t kbase_c = (int64_t)(uintptr_t)Kc, kbase_d = (int64_t)(uintptr_t)Kd;
  const int64_t dv_c = (int64_t)(uintptr_t)Vc - kbase_c, dv_d = (int64_t)(uintptr_t)Vd - kbase_d;
  // element offset (bit 0 = draft) -> byte address of the K row, bit 0 kept; masks, not selects
  auto row_addr = [&](int64_t off) -> int64_t {
    const int64_t is_d = -(off & 1);
    return kbase_c + ((kbase_d - kbase_c) & is_d) + ((off & ~(int64_t)1) << 1) + (off & 1);
  };
  auto gather_tile = [&](int64_t my_addr, int64_t (&a)[8]) {
#pragma unroll
    for (int n = 0; n < 8; ++n) a[n] = __shfl(my_addr, 4 * n + (lane >> 4), 64);
  };
  auto issue_tile = [&](const int64_t (&a)[8], unsigned char* kdst) {
    unsigned char* vdst = kdst + kTileBytes;
    const int pos = lane & 15;
#pragma unroll
    for (int n = 0; n < 8; ++n) {
      const int s = 4 * n + (lane >> 4);                 // slot of this lane in load n
      const int c = pos ^ (s & 15);
      const int64_t ka = (a[n] & ~(int64_t)1) + c * 16;
      const int64_t va = ka + dv_c + ((dv_d - dv_c) & -(a[n] & 1));
      __builtin_amdgcn_global_load_lds(SVF_GLOBAL_PTR(ka), SVF_LDS_PTR(kdst + n * 1024), 16, 0, 0);
      __builtin_amdgcn_global_load_lds(SVF_GLOBAL_PTR(va), SVF_LDS_PTR(vdst + n * 1024), 16, 0, 0);
    }
  };
  // Everything loaded so far (queries, block ids, page table entries) is needed before the
  // stream starts anyway; draining the counter here keeps later register reuse from being
  // mistaken for a hazard against the stream.
  wait_vmcnt<0>();
  // Tile u of a wavefront sits in stage u & 1; the owner of draft tile 0 keeps that tile in
  // the extra stage and its other tiles in stages (u - 1) & 1.
  const bool own_x = gw == 0;
  unsigned char* const x_lds = smem + kWaves * kWaveLds;
  auto stage_ptr = [&](int u) -> unsigned char* {
    if (own_x) return u == 0 ? x_lds : my_lds + ((u - 1) & 1) * kStageBytes;
    return my_lds + (u & 1) * kStageBytes;
  };
  int n_issued = 0;
  {
    int64_t a0[8], a1[8], a2[8];
    gather_tile(row_addr(t_off[0]), a0);
    gather_tile(row_addr(t_off[1]), a1);
    if (own_x) gather_tile(row_addr(t_off[2]), a2);
    if (n_my > 0) { issue_tile(a0, stage_ptr(0)); n_issued = 1; }
    if (n_my > 1) { issue_tile(a1, stage_ptr(1)); n_issued = 2; }
    if (own_x && n_my > 2) { issue_tile(a2, stage_ptr(2)); n_issued = 3; }
  }

  // this lane's read offsets inside a stage
  uint32_t krel[8], vrel[8];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) krel[ks] = l32 * kRowBytes + (((2 * ks + g) ^ (l32 & 15)) << 4);
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int tok = 8 * (e >> 2) + 4 * g + (e & 3);
    vrel[e] = tok * kRowBytes + (((l32 >> 1) ^ (tok & 15)) << 4) + ((l32 & 1) << 3);
  }

#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    const int i = rdraft[rt];
    if (i < 0) rmask[rt] = 0;
    else if (!p.draft_mask) rmask[rt] = i >= 63 ? ~0ull : ((2ull << i) - 1ull);   // linear causal drafts
  }

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

#pragma unroll
  for (int u = 0; u < kMaxTiles; ++u) {
    if (u < n_my) {
      // Tiles are issued in order, 16 loads each, so tile u has arrived once at most
      // 16 * (tiles issued after it) loads are outstanding.
      const int after = n_issued - (u + 1);
      if (after >= 2) wait_vmcnt<32>(); else if (after == 1) wait_vmcnt<16>(); else wait_vmcnt<0>();
      uint32_t allowed[RT];
      const bool all_visible = !t_draft[u] && t_valid[u] == 0xffffffffu;
      const int draft_base = (gw + u * NW) * kTile;       // first draft index of a draft tile
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) {
        allowed[rt] = t_valid[u];
        if (t_draft[u]) allowed[rt] &= (uint32_t)(rmask[rt] >> (draft_base & 63));
      }
      const uint32_t stage = (uint32_t)(uintptr_t)SVF_LDS_PTR(stage_ptr(u));
      if (u == 0)
        process_tile<RT, true>(stage, krel, vrel, qf, allowed, all_visible, p.scale_log2, g, m_run, l_run, oacc);
      else
        process_tile<RT, false>(stage, krel, vrel, qf, allowed, all_visible, p.scale_log2, g, m_run, l_run, oacc);
      // refill the stage just consumed with the tile two further on (its LDS reads have completed);
      // the extra stage is never reused
      if (u + 2 < kMaxTiles && u + 2 < n_my && !(own_x && u == 0)) {
        int64_t a[8];
        gather_tile(row_addr(t_off[u + 2 < kMaxTiles ? u + 2 : 0]), a);
        issue_tile(a, stage_ptr(u));
        n_issued = u + 3;
      }
    }
  }

  // ---- combine the four wavefronts through LDS ---------------------------------------------
  // Wavefront w parks its rescaled fp32 output in its own 32 KB as [ROWS][32 float4]; float4
  // chunk c4 of row r sits at position c4 ^ (r & 31), which keeps both the row-per-lane writes
  // and the chunk-per-lane reads off each other's banks.
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
  {
    float4* mine = reinterpret_cast<float4*>(my_lds);
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      const int r = rt * 32 + l32;
      float mw = -INFINITY;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) mw = fmaxf(mw, sm_m[w][r]);
      const float f = m_run[rt] == -INFINITY ? 0.f : fast_exp2(m_run[rt] - mw);
      if (g == 0) sm_l[wave][r] = l_run[rt] * f;           // denominators leave here already rescaled
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int i = 8 * (v >> 2) + 4 * g + (v & 3);      // dims 4*i .. 4*i+3
        mine[r * 32 + (i ^ l32)] =
            make_float4(oacc[rt][0][v] * f, oacc[rt][1][v] * f, oacc[rt][2][v] * f, oacc[rt][3][v] * f);
      }
    }
  }
  __syncthreads();

  // 256 threads: eight per row, 16 channels (four float4 chunks) each; RT passes of 32 rows
  const bool single = p.n_splits == 1;
  const int cg = tid & 7;
  float racc[RT][16];
  int64_t rorow[RT];
  bool rok[RT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    const int r = rt * 32 + (tid >> 3);
    float mw = -INFINITY, lw = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      mw = fmaxf(mw, sm_m[w][r]);
      lw += sm_l[w][r];
    }
#pragma unroll
    for (int c = 0; c < 16; ++c) racc[rt][c] = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w)
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const float4 t = reinterpret_cast<const float4*>(smem + w * kWaveLds)[r * 32 + ((cg * 4 + c) ^ (r & 31))];
        racc[rt][4 * c] += t.x; racc[rt][4 * c + 1] += t.y; racc[rt][4 * c + 2] += t.z; racc[rt][4 * c + 3] += t.w;
      }
    const int row = row0 + r;
    rok[rt] = row < p.M;
    const int i = rok[rt] ? row / p.G : 0, j = h * p.G + (rok[rt] ? row % p.G : 0);
    rorow[rt] = ((int64_t)b * p.gamma + i) * p.Hq + j;
    if (single) {
      if (rok[rt]) {
        const float inv = 1.0f / lw;
        u32x4 o0, o1;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          o0[c] = pack_bf16(racc[rt][2 * c] * inv, racc[rt][2 * c + 1] * inv);
          o1[c] = pack_bf16(racc[rt][8 + 2 * c] * inv, racc[rt][8 + 2 * c + 1] * inv);
        }
        u32x4* dst = reinterpret_cast<u32x4*>(static_cast<__hip_bfloat16*>(p.out) + rorow[rt] * kD + cg * 16);
        dst[0] = o0;
        dst[1] = o1;
        if (p.lse && cg == 0) p.lse[rorow[rt]] = (mw + log2f(lw)) * 0.6931471805599453f;
      }
    } else if (row < p.Mpad) {
      // this split's partial: normalised output in bf16, (m, l) in fp32, written through
      const int64_t pr = ((int64_t)pair * p.n_splits + split) * p.Mpad + row;
      const float inv = lw > 0.f ? 1.0f / lw : 0.f;
      u32x4 o0, o1;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        o0[c] = pack_bf16(racc[rt][2 * c] * inv, racc[rt][2 * c + 1] * inv);
        o1[c] = pack_bf16(racc[rt][8 + 2 * c] * inv, racc[rt][8 + 2 * c + 1] * inv);
      }
      uint16_t* po = reinterpret_cast<uint16_t*>(p.part_o) + pr * kD + cg * 16;
      store_coherent16(po, o0);
      store_coherent16(po + 8, o1);
      if (cg == 0) store_coherent2(p.part_ml + 2 * pr, mw, lw);
    }
  }
  if (single) return;

  // ---- last workgroup of the group merges the splits ------------------------------------------
  // The partials were written through to device-coherent memory; once those stores have been
  // acknowledged (vmcnt = 0) the ticket may be taken.  No bulk cache write-back.
  // The ticket is one 64-bit counter: bits [15:0] count arrivals, and eight 6-bit fields above
  // count arrivals per XCD, so that the last workgroup learns whether every partial of its
  // group was written through the L2 it is about to read from.
  wait_vmcnt<0>();
  __syncthreads();
  if (tid == 0) {
    uint32_t xcc;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
    const int field = 16 + 6 * (int)(xcc & 7u);
    const uint64_t prev = __hip_atomic_fetch_add(&p.tickets[group], 1ull | (1ull << field), __ATOMIC_RELAXED,
                                                 __HIP_MEMORY_SCOPE_AGENT);
    const bool last = (prev & 0xffffull) == (uint64_t)(p.n_splits - 1);
    const bool same_xcd = p.n_splits <= 63 && ((prev >> field) & 63ull) == (uint64_t)(p.n_splits - 1);
    // leave the counter ready for the next call
    if (last) __hip_atomic_store(&p.tickets[group], 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    sm_last = last ? (same_xcd ? 2 : 1) : 0;
  }
  __syncthreads();
  const int last_kind = sm_last;
  if (last_kind == 0) return;
  // Remote writers: acquire at device scope, which drops whatever this XCD's caches still hold
  // of the partial buffers (they are reused by every call); ordinary loads then fetch the
  // written-through data.  Local writers only (the normal case): this XCD's L2 is their common
  // coherence point, loads that bypass the per-CU cache are enough.
  if (last_kind == 1) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    const int64_t g_row = (int64_t)pair * p.n_splits * p.Mpad + row0 + rt * 32 + (tid >> 3);
    if (last_kind == 2) merge_splits<true>(p, g_row, rorow[rt], rok[rt], cg);
    else merge_splits<false>(p, g_row, rorow[rt], rok[rt], cg);
  }
}

}  // namespace

bool mfma_supported(const svf_shape_t& s) { return s.dtype == SVF_BF16 && s.d == 128; }

// Splits per (sequence, KV head, row group): enough workgroups to cover the 256 compute units,
// never more than kMaxTiles tiles per wavefront, never less than one tile per wavefront.
int mfma_splits(const svf_shape_t& s) {
  const int M = s.gamma * (s.Hq / s.Hkv);
  const int rows = 32;
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
  const int rows = 32;
  const int row_groups = (p.M + rows - 1) / rows;
  const int groups = p.B * p.Hkv * row_groups;
  const unsigned grid = (unsigned)(kXcds * ((groups + kXcds - 1) / kXcds) * p.n_splits);
  hipLaunchKernelGGL(verify_attn_mfma_kernel<1>, dim3(grid), dim3(kThreads), 0, st, p, row_groups, groups);
  return hipGetLastError();
}

}  // namespace svf
