// Verification attention, matrix-core kernel: bf16 inputs, head dimension 128 (Sec. 3.1 / 3.3:
// the draft queries attend to the retrieved blocks of their KV head and, through the draft
// mask, to each other).
//
// What bounds this kernel.  One layer's selected K+V is a few tens of MB: at 8 TB/s the stream
// itself lasts ~5 us, so everything serial around it counts.  A wavefront issues one
// instruction every four cycles (~0.6 G instructions/s), whatever the instruction; a
// thousand-instruction prologue costs 1.7 us.  Hence: eight wavefronts per workgroup (two per
// SIMD, so that two instruction streams interleave), one 32-token tile per wavefront in the
// common case, and as few instructions as possible in front of the K/V loads: the addresses of
// a tile are resolved by eight lanes in parallel (one per group of four consecutive tokens,
// which share a block and a page), moved to scalar registers, and every load is "scalar base +
// per-lane 32-bit offset" with the per-lane offsets computed once.  Load instructions count as
// well as bytes: a compute unit hands the memory pipeline one per ~20 cycles, so what a
// workgroup requests before its tiles is kept to few instructions.
//
// Shape of the work.  For one (sequence, KV head) the gamma x G query rows that share the KV
// head are packed into M = gamma * G rows (row = draft * G + head-in-group), 32 rows per
// workgroup, so that every selected key/value is read from HBM once and used by all of them
// (with more than 32 rows the row groups of a pair run on one XCD and share its L2).  The
// selected tokens plus the draft tokens are cut into 32-token tiles; tile t belongs to
// wavefront t mod NW, NW = 8 * n_splits wavefronts per (pair, row group).
//
// Data path.  K and V rows go straight into LDS with 16-byte direct-to-LDS loads (no registers
// in between), one 16 KB stage per wavefront, private to it: no workgroup barrier in the main
// loop.  The wavefront that owns draft tile 0 keeps it in a ninth stage, so that its prefix
// tile streams at the same time.  In launches where no wavefront has a second cache tile every
// wavefront still fetches a tile, but wavefronts 4 .. 7 leave theirs to wavefronts 0 .. 3 (one
// barrier), which halves what has to be combined afterwards.  The 16-byte chunks of a row sit at an XOR-swizzled position
// (chosen on the global-address side; the LDS side of such a load is fixed by the lane id),
// which keeps the fragment reads off each other's banks.  The LDS reads of the main loop are
// issued by hand (inline ds_read + explicit waits): the compiler would otherwise wait for every
// outstanding direct-to-LDS load before any LDS read.
//
// Math.  Both products run on the matrix cores in transposed form so that a query row lives
// in a fixed lane (lane mod 32) from the first MFMA to the final store:
//   S^T[token][row] = K[token][:] . Q[row][:]           A = K tile (LDS, 16-byte reads), B = Q (registers)
//   O^T[dim][row]  += V^T[dim][token] P^T[token][row]   A = V tile (LDS, transposing 8-byte reads),
//                                                       B = P (registers)
// Softmax runs in the log2 domain in fp32 with one cross-lane step per tile (lanes l, l+32);
// the rescale of O is a per-lane scalar, applied only when the maximum moved by more than
// kRescaleGap.  P is rounded to bf16 (hardware RNE) for the second product; accumulators fp32.
//
// Merge.  The computing wavefronts combine through LDS (log-sum-exp rule).  With one split the
// workgroup writes out / lse itself.  Otherwise every workgroup of a (pair, row group) stores a
// partial (normalised output in bf16, (m, l) in fp32 inside a 16-byte record that carries the
// call's tag twice) and then merges a slice of the rows itself: two of its wavefronts wait (a
// bounded number of polls) until every record of the other splits' rows of that slice shows the
// tag, fetch those partials (forming the weights while they are on their way), and sum in split
// order, taking the own split from LDS.  No workgroup
// waits for all others and none is the designated merger; a slice whose wait ran out is marked
// in the group's arrival word and merged by whichever workgroup arrives last.  The tag is the
// group's call counter plus one, kept in the workspace and advanced by the workgroup that
// arrives last, so the kernel needs no clearing between calls.
//
// Scope of the exchange.  Workgroup ids are mapped so that all splits of a group share id mod 8,
// which the dispatcher places on one XCD; each workgroup also adds its XCD number to a
// per-group counter, and only if every arrival so far came from the XCD it runs on does it
// store its partial with plain stores (acknowledged by that XCD's L2, where the readers' L1-
// bypassing loads are served).  Otherwise partials and records are written through to memory.
#include <hip/hip_bf16.h>

#include "svf_device.h"

namespace svf {

namespace {

constexpr int kThreads = 512;
constexpr int kWaves = 8;
constexpr int kTile = 32;            // tokens per tile
constexpr int kD = 128;              // head dimension
constexpr int kRowBytes = kD * 2;    // one bf16 K/V row
constexpr int kTileBytes = kTile * kRowBytes;          // 8 KB: K (or V) part of a stage
constexpr int kStageBytes = 2 * kTileBytes;            // K then V
constexpr int kMaxTiles = 4;         // tiles a wavefront may own (processed one after the other)
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
// Transposing LDS read (ds_read_b64_tr_b16), issued by hand.  Within every group of 16 lanes, lane
// i receives as element j (of four 16-bit elements) element i % 4 of the 8 bytes that lane
// 4 * j + i / 4 of the group addresses.  So if lane L addresses channels c0 + 4 * (L % 4) .. + 3 of
// the row of token t0 + L / 4, lane i ends up with channel c0 + i of tokens t0 .. t0 + 3: four
// k-slots of a matrix-core A operand whose row is a channel, with no register shuffling.
template <int OFF>
__device__ __forceinline__ u32x2 lds_read8_tr(uint32_t addr) {
  u32x2 v;
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF) : "memory");
  return v;
}
// The eight transposing reads of one k-step of the second product.  Piece e = 2 nt + h is chunk
// 4 nt + vc of the token rows vtok + 8 h (+ 16 KS2), at the swizzled position (4 nt + vc) ^ token.
// With L = vc ^ (vtok & 3) (bits 0, 1), g = bit 2 of vtok and h = bit 3 of the token that is
//   16 L + 64 ((nt & 1) ^ g) + 128 ((nt >> 1) ^ h),
// and 64 ((nt & 1) ^ g) = 64 (nt & 1) + 64 g for even nt, 64 (nt & 1) - 64 g for odd nt: two
// per-lane addresses (even / odd nt) and an immediate per piece, instead of an XOR and an addition
// per piece in every tile.
template <int E, int KS2>
__device__ __forceinline__ u32x2 lds_read_vt_piece(uint32_t even, uint32_t odd) {
  constexpr int nt = E >> 1, h = E & 1;
  return lds_read8_tr<64 * (nt & 1) + 128 * ((nt >> 1) ^ h) + h * 8 * kRowBytes + KS2 * 16 * kRowBytes>((nt & 1) ? odd : even);
}
template <int KS2>
__device__ __forceinline__ void lds_read_vt(u32x2 (&x)[8], uint32_t even, uint32_t odd) {
  x[0] = lds_read_vt_piece<0, KS2>(even, odd);
  x[1] = lds_read_vt_piece<1, KS2>(even, odd);
  x[2] = lds_read_vt_piece<2, KS2>(even, odd);
  x[3] = lds_read_vt_piece<3, KS2>(even, odd);
  x[4] = lds_read_vt_piece<4, KS2>(even, odd);
  x[5] = lds_read_vt_piece<5, KS2>(even, odd);
  x[6] = lds_read_vt_piece<6, KS2>(even, odd);
  x[7] = lds_read_vt_piece<7, KS2>(even, odd);
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

template <typename T>
__device__ __forceinline__ void lds_wait2(T (&r)[2]) {
  asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(r[0]), "+v"(r[1]) : : "memory");
}
// LDS store issued by hand (a compiler-issued one would first wait for every direct-to-LDS load in flight)
__device__ __forceinline__ void lds_write4(uint32_t addr, uint32_t value) {
  asm volatile("ds_write_b32 %0, %1" : : "v"(addr), "v"(value) : "memory");
}

template <typename T>
__device__ __forceinline__ void lds_wait4(T (&r)[4]) {
  asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(r[0]), "+v"(r[1]), "+v"(r[2]), "+v"(r[3]) : : "memory");
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  const floatx2 f = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));   // round to nearest even
}
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Maximum / sum of the values that lanes l and l ^ 32 hold (a query row's two half-rows): the
// halves of the wavefront are exchanged by one cross-lane instruction, v_permlane32_swap, which
// hands back (lower half twice, upper half twice); a shuffle would go through LDS and, with its
// wait, drain the LDS reads in flight around it.
__device__ __forceinline__ float halves_max(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float halves_sum(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Stores of data exchanged between workgroups: device-scope write-through stores, so making
// them visible across the chip's L2 slices needs no bulk write-back, only a wait for the
// stores' acknowledgement.
// (A store of more than eight bytes still reads its data registers in the cycle after it issues:
// the wait state keeps whatever the compiler schedules next from overwriting them.  The compiler
// inserts it by itself for its own stores, not behind an inline one.)
__device__ __forceinline__ void store_coherent16(void* p, u32x4 bits) {
  asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" : : "v"(p), "v"(bits) : "memory");
}
// The same store left in the L2 (written back when the kernel ends): enough, and acknowledged much
// sooner, when every reader is known to sit behind the same L2.
__device__ __forceinline__ void store_l2_16(void* p, u32x4 bits) {
  asm volatile("global_store_dwordx4 %0, %1, off\n\ts_nop 1" : : "v"(p), "v"(bits) : "memory");
}
__device__ __forceinline__ uint32_t xcc_id() {
  uint32_t xcc;
  asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
  return xcc & 7u;
}
__device__ __forceinline__ void store_coherent2(float* p, float a, float b) {
  const uint64_t bits = (uint64_t)__float_as_uint(a) | ((uint64_t)__float_as_uint(b) << 32);
  __hip_atomic_store(reinterpret_cast<uint64_t*>(p), bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void store_coherent8(void* p, u32x2 bits) {
  const uint64_t w = (uint64_t)bits[0] | ((uint64_t)bits[1] << 32);
  __hip_atomic_store(reinterpret_cast<uint64_t*>(p), w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// s_waitcnt vmcnt(n) for an even run-time n in 0 .. 24 (the count is an immediate of the instruction).
__device__ __forceinline__ void wait_vmcnt_upto24(int n) {
  switch (n) {
    case 18: wait_vmcnt<18>(); return;
    case 20: wait_vmcnt<20>(); return;
    case 22: wait_vmcnt<22>(); return;
    case 24: wait_vmcnt<24>(); return;
    default: break;
  }
  switch (n) {
    case 0: wait_vmcnt<0>(); break;
    case 2: wait_vmcnt<2>(); break;
    case 4: wait_vmcnt<4>(); break;
    case 6: wait_vmcnt<6>(); break;
    case 8: wait_vmcnt<8>(); break;
    case 10: wait_vmcnt<10>(); break;
    case 12: wait_vmcnt<12>(); break;
    case 14: wait_vmcnt<14>(); break;
    default: wait_vmcnt<16>(); break;
  }
}
// The same for n in 0 .. 16.
__device__ __forceinline__ void wait_vmcnt_upto16(int n) {
  switch (n) {
    case 0: wait_vmcnt<0>(); break;
    case 2: wait_vmcnt<2>(); break;
    case 4: wait_vmcnt<4>(); break;
    case 6: wait_vmcnt<6>(); break;
    case 8: wait_vmcnt<8>(); break;
    case 10: wait_vmcnt<10>(); break;
    case 12: wait_vmcnt<12>(); break;
    case 14: wait_vmcnt<14>(); break;
    default: wait_vmcnt<16>(); break;
  }
}

// Lane i ^ 4 of every lane i (two row rotations, each written to the banks of four lanes it is
// right for: banks 0 and 2 take lane i + 4, banks 1 and 3 lane i - 4).
__device__ __forceinline__ uint32_t swap_lanes_xor4(uint32_t x) {
  int t = __builtin_amdgcn_update_dpp((int)x, (int)x, 0x12C, 0xf, 0x5, false);    // row_ror:12
  t = __builtin_amdgcn_update_dpp(t, (int)x, 0x124, 0xf, 0xA, false);             // row_ror:4
  return (uint32_t)t;
}
// Where float4 j (0 .. 31) of a parked row sits, before the exclusive-or with the row: the two low
// bits of j go to the top, so that the eight threads that read j = 4c + n (c = 0 .. 7, same n) of a
// row at once hit eight different 16-byte bank groups.
__device__ __forceinline__ int parked_position(int j) { return (j >> 2) | ((j & 3) << 3); }
// Lane N of every row of sixteen lanes, to all lanes of that row.
template <int N>
__device__ __forceinline__ uint32_t row_lane(uint32_t x) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x150 + N, 0xf, 0xf, true);    // row_newbcast:N
}
template <int N>
__device__ __forceinline__ void row_lanes_upto(uint32_t x, uint32_t (&out)[8]) {
  out[N] = row_lane<N>(x);
  if constexpr (N > 0) row_lanes_upto<N - 1>(x, out);
}

// Lanes B0 .. B0 + N of every row of sixteen lanes.
template <int B0, int N>
__device__ __forceinline__ void row_lanes_from(uint32_t x, uint32_t (&out)[8]) {
  out[N] = row_lane<B0 + N>(x);
  if constexpr (N > 0) row_lanes_from<B0, N - 1>(x, out);
}

// The eight 16-byte fragments of a lane's query row, loaded by hand: not valid before a wait of
// the caller's own has covered them and query_fragments_arrived() has been given the registers.
__device__ __forceinline__ void load_query_fragments(bf16x8 (&qf)[8], const void* row) {
#define SVF_QFRAG(i)                                                                                   \
  asm volatile("global_load_dwordx4 %0, %1, off offset:%2" : "=v"(qf[i]) : "v"(row), "n"((i) * 32) : "memory")
  SVF_QFRAG(0); SVF_QFRAG(1); SVF_QFRAG(2); SVF_QFRAG(3);
  SVF_QFRAG(4); SVF_QFRAG(5); SVF_QFRAG(6); SVF_QFRAG(7);
#undef SVF_QFRAG
}
__device__ __forceinline__ u32x2 load8_plain(const void* p) {
  u32x2 v;
  asm volatile("global_load_dwordx2 %0, %1, off" : "=v"(v) : "v"(p) : "memory");
  return v;
}
__device__ __forceinline__ uint32_t load4_plain(const void* p) {
  uint32_t v;
  asm volatile("global_load_dword %0, %1, off" : "=v"(v) : "v"(p) : "memory");
  return v;
}
__device__ __forceinline__ void front_loads_arrived(u32x2& a, u32x2& b, uint32_t& c, u32x2& d) {
  asm volatile("" : "+v"(a), "+v"(b), "+v"(c), "+v"(d) : : "memory");
}
__device__ __forceinline__ void query_fragments_arrived(bf16x8 (&qf)[8]) {
  asm volatile("" : "+v"(qf[0]), "+v"(qf[1]), "+v"(qf[2]), "+v"(qf[3]), "+v"(qf[4]), "+v"(qf[5]), "+v"(qf[6]), "+v"(qf[7])
               :
               : "memory");
}

// One 32-token tile against the workgroup's 32 query rows.  stage: LDS address of the stage;
// allowed: bit t set = token t of the tile is visible to this lane's row.  Register use is kept
// low (two wavefronts share a SIMD): fragment addresses are recomputed, K fragments come in two
// batches of four, the V rows of the second half reuse the registers of the first.
__device__ __forceinline__ void process_tile(uint32_t stage, const bf16x8 (&qf)[8], uint32_t allowed,
                                             bool all_visible, float scale_log2, int l32, int g, float& m_run,
                                             float& l_run, floatx16 (&oacc)[4]) {
  // K fragment of k-step ks: row l32, 16-byte chunk 2*ks + g at swizzled position
  const uint32_t kbase = stage + l32 * kRowBytes;
  const uint32_t kx = (uint32_t)((g ^ (l32 & 15)) << 4);
  // V^T fragments by transposing reads: A row m (= lane mod 32) of the nt-th product is channel
  // 32 * nt + m; k-slot e of lane group g is token 8*(e/4) + 4*g + e%4 (+16 for the second k-step).
  // This lane addresses, for piece h of a k-step, token 8*h + 4*g + (lane%16)/4 and the four
  // channels 32*nt + 16*((lane/16)%2) + 4*(lane%4): 16-byte chunk 4*nt + vc, half vh.
  const uint32_t vtok = (uint32_t)(4 * g + ((l32 & 15) >> 2));
  const uint32_t vc = (uint32_t)(2 * ((l32 >> 4) & 1) + ((l32 & 3) >> 1));
  const uint32_t vbase = stage + kTileBytes + vtok * kRowBytes + ((uint32_t)(l32 & 1) << 3);
  const uint32_t vswz = (vc ^ (vtok & 3u)) << 4;
  const uint32_t v_even = vbase + vswz + ((uint32_t)g << 6), v_odd = vbase + vswz - ((uint32_t)g << 6);

  // S^T = K Q^T : token = lane mod 32 (A rows), query row = lane mod 32 (B columns)
  floatx16 sacc;
#pragma unroll
  for (int v = 0; v < 16; ++v) sacc[v] = 0.f;
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    u32x4 kf[4];
#pragma unroll
    for (int k4 = 0; k4 < 4; ++k4) kf[k4] = lds_read16<0>(kbase + (kx ^ (uint32_t)((4 * half + k4) << 5)));
    lds_wait4(kf);
#pragma unroll
    for (int k4 = 0; k4 < 4; ++k4)
      sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kf[k4]), qf[4 * half + k4], sacc,
                                                     0, 0, 0);
  }
  // the V^T fragments of the first k-step: in flight while the softmax runs.  x[2 * nt + h]
  u32x2 x[8];
  lds_read_vt<0>(x, v_even, v_odd);

  // online softmax; value v of a lane is token 8*(v/4) + 4*g + v%4 of the tile.
  // Invisible tokens drop out by setting their raw score to -inf (the scale is positive).
  if (!all_visible) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int tok = 8 * (v >> 2) + 4 * g + (v & 3);
      if (!((allowed >> tok) & 1u)) sacc[v] = -INFINITY;
    }
  }
  float mx = sacc[0];
#pragma unroll
  for (int v = 1; v < 16; ++v) mx = fmaxf(mx, sacc[v]);
  mx = halves_max(mx) * scale_log2;
  // keep the old reference while the maximum has not run away from it
  float m_ref = m_run;
  const bool move = mx > m_ref + kRescaleGap;            // always true on a row's first visible tile
  if (__any(move)) {
    const float m_new = move ? mx : m_ref;
    if (__any(move && m_ref != -INFINITY)) {             // nothing to rescale while O is still zero
      const float alpha = m_new == m_ref ? 1.0f : fast_exp2(m_ref - m_new);   // -inf - finite -> 0
      l_run *= alpha;
#pragma unroll
      for (int nt = 0; nt < 4; ++nt)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[nt][v] *= alpha;
    }
    m_ref = m_new;
  }
  m_run = m_ref;
  const float m_use = m_ref == -INFINITY ? 0.f : m_ref;
  float ls = 0.f;
  float pe[16];
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    pe[v] = fast_exp2(__builtin_fmaf(sacc[v], scale_log2, -m_use));
    ls += pe[v];
  }
  l_run += ls;
  bf16x8 pf[2];
#pragma unroll
  for (int ks2 = 0; ks2 < 2; ++ks2) {
    u32x4 w;
#pragma unroll
    for (int j = 0; j < 4; ++j) w[j] = pack_bf16(pe[8 * ks2 + 2 * j], pe[8 * ks2 + 2 * j + 1]);
    pf[ks2] = __builtin_bit_cast(bf16x8, w);
  }

  // O^T += V^T P^T : A row m = lane mod 32 of product nt is channel 32*nt + m; k-slot e of lane
  // group g is token 16*ks2 + 8*(e/4) + 4*g + e%4.  x[2*nt + h] holds k-slots 4*h .. 4*h+3.
#pragma unroll
  for (int ks2 = 0; ks2 < 2; ++ks2) {
    if (ks2 == 1) lds_read_vt<1>(x, v_even, v_odd);
    lds_wait8(x);
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) {
      const u32x4 w = {x[2 * nt][0], x[2 * nt][1], x[2 * nt + 1][0], x[2 * nt + 1][1]};
      oacc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, w), pf[ks2], oacc[nt], 0, 0, 0);
    }
  }
}

// Merge of a group's split partials by one workgroup (512 threads), used behind the rows
// kernel: sixteen threads per row, 8 channels each.  All splits are read in split order; the
// loads of kMergeBatch splits are in flight before the first is used.  A split's (m, l) is
// loaded by one of the row's sixteen threads and handed round inside the row.
__device__ __forceinline__ void merge_splits(const AttnParams& p, int64_t g_row, int64_t orow, bool row_ok, int cg) {
  constexpr int kMergeBatch = 8;
  const uint16_t* part_o = reinterpret_cast<const uint16_t*>(p.part_o);
  float acc[8];
#pragma unroll
  for (int c = 0; c < 8; ++c) acc[c] = 0.f;
  float m_acc = -INFINITY, l_acc = 0.f;
  for (int s0 = 0; s0 < p.n_splits; s0 += kMergeBatch) {
    u32x4 t[kMergeBatch];
    u32x2 ml;                        // of split s0 + cg mod 8
    {
      const int64_t pr = g_row + (int64_t)min(s0 + (cg & (kMergeBatch - 1)), p.n_splits - 1) * p.Mpad;
      const u32x4 rec = *reinterpret_cast<const u32x4*>(p.part_rec + 4 * pr);     // (maximum, tag, denominator, tag)
      ml = u32x2{rec[0], rec[2]};
    }
#pragma unroll
    for (int u = 0; u < kMergeBatch; ++u) {
      // entries past the last split (index clamped) get weight 0 below
      const int64_t pr = g_row + (int64_t)min(s0 + u, p.n_splits - 1) * p.Mpad;
      t[u] = *reinterpret_cast<const u32x4*>(part_o + pr * kD + cg * 8);
    }
    uint32_t mbits[kMergeBatch], lbits[kMergeBatch];
    row_lanes_upto<kMergeBatch - 1>(ml[0], mbits);
    row_lanes_upto<kMergeBatch - 1>(ml[1], lbits);
    float pm[kMergeBatch], pl[kMergeBatch];
    float mb = m_acc;
#pragma unroll
    for (int u = 0; u < kMergeBatch; ++u) {
      pm[u] = s0 + u >= p.n_splits ? -INFINITY : __uint_as_float(mbits[u]);
      pl[u] = __uint_as_float(lbits[u]);
      mb = fmaxf(mb, pm[u]);
    }
    const float fa = m_acc == -INFINITY ? 0.f : fast_exp2(m_acc - mb);
    l_acc *= fa;
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[c] *= fa;
#pragma unroll
    for (int u = 0; u < kMergeBatch; ++u) {
      // weight of split s: exp2(m_s - m) * l_s, applied to its normalised output
      const float w = pm[u] != -INFINITY ? fast_exp2(pm[u] - mb) * pl[u] : 0.f;
      l_acc += w;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        acc[2 * c] += w * bf16_lo(t[u][c]);
        acc[2 * c + 1] += w * bf16_hi(t[u][c]);
      }
    }
    m_acc = mb;
  }
  if (row_ok) {
    const float inv = l_acc > 0.f ? 1.0f / l_acc : 0.f;      // a row that saw no key at all: zero, lse = -inf
    u32x4 o;
#pragma unroll
    for (int c = 0; c < 4; ++c) o[c] = pack_bf16(acc[2 * c] * inv, acc[2 * c + 1] * inv);
    store_coherent16(static_cast<__hip_bfloat16*>(p.out) + orow * kD + cg * 8, o);
    if (p.lse && cg == 0) p.lse[orow] = (m_acc + log2f(l_acc)) * 0.6931471805599453f;
  }
}

// ---- merging the splits of a group ----------------------------------------------------------------
// A split's partial of a row is its output normalised by its own denominator (bf16) and a 16-byte
// record (maximum, tag, denominator, tag); the record is written after the output has been
// acknowledged, so a record whose two tags are this call's vouches for the output beside it.
// Merge rule (log-sum-exp), the same sums in the same order whoever computes them: splits in
// order, in batches of eight, each batch brought to the running maximum.
// The merging threads are two wavefronts (128 threads): CH channels per thread (4 or 8), 128 / CH
// threads per row, 4 or 8 rows per pass.

// Device-scope loads of what other workgroups have written through (they bypass the per-CU cache;
// an L2 serves them, also for lines that a workgroup on another XCD has written through).  Issued
// by hand: scalar base + per-lane offset.  load_record_now() waits for its value; the values of
// load_chunk() are not valid before chunks_wait() has been given the registers.
__device__ __forceinline__ u32x4 load_record_now(const void* p) {
  u32x4 v;
  asm volatile("global_load_dwordx4 %0, %1, off sc1\n\ts_waitcnt vmcnt(0)" : "=v"(v) : "v"(p) : "memory");
  return v;
}
// The same, and a word of LDS read in the load's shadow (lds_word keeps its value in lanes that are off).
__device__ __forceinline__ u32x4 load_record_now(const void* p, uint32_t lds_addr, uint32_t& lds_word) {
  u32x4 v;
  asm volatile("ds_read_b32 %1, %3\n\tglobal_load_dwordx4 %0, %2, off sc1\n\ts_waitcnt vmcnt(0) lgkmcnt(0)"
               : "=v"(v), "+v"(lds_word)
               : "v"(p), "v"(lds_addr)
               : "memory");
  return v;
}
__device__ __forceinline__ void load_chunk(u32x2& v, uint64_t base, uint32_t off) {
  asm volatile("global_load_dwordx2 %0, %1, %2 sc1" : "=v"(v) : "v"(off), "s"(base) : "memory");
}
__device__ __forceinline__ void load_chunk(u32x4& v, uint64_t base, uint32_t off) {
  asm volatile("global_load_dwordx4 %0, %1, %2 sc1" : "=v"(v) : "v"(off), "s"(base) : "memory");
}
template <typename T>
__device__ __forceinline__ void chunks_wait(T (&o)[8]) {
  asm volatile("s_waitcnt vmcnt(0)"
               : "+v"(o[0]), "+v"(o[1]), "+v"(o[2]), "+v"(o[3]), "+v"(o[4]), "+v"(o[5]), "+v"(o[6]), "+v"(o[7])
               :
               : "memory");
}
template <int CH> struct ChunkOf;
template <> struct ChunkOf<4> { typedef u32x2 type; };
template <> struct ChunkOf<8> { typedef u32x4 type; };

constexpr int kMergeThreads = 128;          // wavefronts kMergeWave0 and kMergeWave0 + 1
constexpr int kMergeWave0 = 4;
constexpr int kLastResortPolls = 1 << 16;   // for waits that are known to end: every writer has arrived

// One merging thread's view of one pass over rows r0 .. r0 + rows per pass.
template <int CH>
struct MergeLane {
  typedef typename ChunkOf<CH>::type Chunk;
  static constexpr int kLanesPerRow = kD / CH;                  // 32 or 16
  static constexpr int kRowsPerPass = kMergeThreads / kLanesPerRow;
  int row;            // row of the row group (clamped to a valid one), cl: which CH channels
  int cl;
  bool active;        // the row is one of those to merge
  float acc[CH];
  float m_acc, l_acc;
  u32x4 rec;          // record of split c0 + cl % 16 of this row
  Chunk t0[8], t1[8]; // fetched outputs of splits c0 .. c0 + 7 and c0 + 8 .. c0 + 15
  // what the two batches weigh (formed while their outputs are on their way): the factor that
  // brings the running sums to the batch's maximum, that maximum, the splits' weights, and the own
  // split's output from LDS
  float fa0, fa1, mb0, mb1;
  float w0[8], w1[8];
  Chunk own_chunk;
  int64_t orow;       // where the merged row goes (row of out / lse), worked out in the same shadow
};

// This workgroup's own partial of the rows it merges, left in LDS by the threads that formed it:
// [rows][kD] bf16, then (maximum, denominator) per row.  own_split < 0: nothing is taken from LDS.
struct OwnRows {
  const unsigned char* o;
  const float* ml;
  int lo;             // first row held
  int split;
};

// Waits (at most `budget` polls) until the records of splits c0 .. c0 + 15 of the lane's row carry
// the tag; the own split's record is not waited for when its partial comes from LDS.  Returns false
// for the whole wavefront when some record is still missing.
// watch / watched_for (optional): the LDS word at address `watch` is read along with every poll;
// *watch_hit tells whether it was seen to hold `watched_for` (what the caller waits for next: by
// the time the records are in, it has usually happened, and no further look is needed).
template <int CH>
__device__ __forceinline__ bool poll_records(const AttnParams& p, MergeLane<CH>& L, int64_t g_row, int c0, uint32_t tag,
                                             int budget, int own_split, uint32_t watch = 0, uint32_t watched_for = 0,
                                             bool* watch_hit = nullptr) {
  const int S = p.n_splits;
  const int sp = c0 + (L.cl & 15);
  const uint32_t* recp = p.part_rec + (g_row + (int64_t)min(sp, S - 1) * p.Mpad) * 4;
  // (past the last split: a record that weighs nothing)
  L.rec = u32x4{sp < S ? 0u : 0xff800000u, 0u, 0u, 0u};
  bool pending = L.active && sp < S && sp != own_split;
  uint32_t word = ~watched_for;
  for (int it = 0;; ++it) {
    if (!__any(pending) || it >= budget) break;
    if (pending) {
      L.rec = watch_hit ? load_record_now(recp, watch, word) : load_record_now(recp);
      pending = !(L.rec[1] == tag && L.rec[3] == tag);
    }
  }
  if (watch_hit) *watch_hit = __any(word == watched_for);
  return !__any(pending);
}

// Requests the outputs of splits c0 + B0 .. c0 + B0 + 7 of the lane's row (past the last split: the
// batch's first split again, weight 0 later; the own split's is fetched like the others even when
// LDS holds it: one address chain, a step of one split's partial at a time).
template <int CH, int B0>
__device__ __forceinline__ void fetch_batch(const AttnParams& p, typename ChunkOf<CH>::type (&t)[8], int pair, uint32_t voff,
                                            int c0) {
  const int S = p.n_splits;
  const uint64_t step = (uint64_t)p.Mpad * kRowBytes;
  const uint64_t first = (uint64_t)(uintptr_t)p.part_o + ((uint64_t)pair * S + (uint64_t)(c0 + B0)) * step;
  const int n = S - c0 - B0;                             // splits of this batch that exist (>= 1)
  uint64_t at = first;
#pragma unroll
  for (int u = 0; u < 8; ++u) {
    load_chunk(t[u], u < n ? at : first, voff);
    at += step;
  }
}

template <int CH>
__device__ __forceinline__ float chunk_value(const typename ChunkOf<CH>::type& t, int c) {
  return (c & 1) ? bf16_hi(t[c >> 1]) : bf16_lo(t[c >> 1]);
}

// Splits c0 + B0 .. c0 + B0 + 7 into the running merge, in two steps.  batch_weights() needs the
// records only (and the own split's maximum and denominator from LDS): it runs while the outputs
// are being fetched, and is free of branches, because the compiler does not know that the
// registers of a hand-issued load are in flight (see merge_fetch_weigh).  m_before: the running
// maximum in front of the batch.
template <int CH, int B0>
__device__ __forceinline__ void batch_weights(MergeLane<CH>& L, int c0, const OwnRows& own, float m_before, float (&w)[8],
                                              float& fa, float& mb_out) {
  const int ou = own.split - c0 - B0;                  // (uniform) the own split's place in this batch
  const bool from_lds = ou >= 0 && ou < 8;
  // the own split's partial comes from LDS: its (maximum, denominator) into the lane that holds
  // that split's record, its output in place of what is fetched (the reads are unconditional: own.o
  // and own.ml always point into LDS)
  const int orow = min(max(L.row - own.lo, 0), 31);
  const typename ChunkOf<CH>::type oc =
      *reinterpret_cast<const typename ChunkOf<CH>::type*>(own.o + orow * kRowBytes + L.cl * (CH * 2));
  const uint32_t om = __float_as_uint(own.ml[2 * orow]), ol = __float_as_uint(own.ml[2 * orow + 1]);
  L.own_chunk = (B0 == 0 || from_lds) ? oc : L.own_chunk;        // (the own split lies in one batch at most)
  const bool here = from_lds && (L.cl & 15) == B0 + ou;
  const uint32_t mrec = here ? om : L.rec[0], lrec = here ? ol : L.rec[2];
  uint32_t mbits[8], lbits[8];
  row_lanes_from<B0, 7>(mrec, mbits);
  row_lanes_from<B0, 7>(lrec, lbits);
  float mb = m_before;
#pragma unroll
  for (int u = 0; u < 8; ++u) mb = fmaxf(mb, __uint_as_float(mbits[u]));
  // (a row that no split saw a token for: every maximum is -inf; exp2(-inf - 0) = 0 for all of them)
  const float ref = mb == -INFINITY ? 0.f : mb;
  fa = fast_exp2(m_before - ref);
#pragma unroll
  for (int u = 0; u < 8; ++u) {
    // weight of split s: exp2(m_s - m) * l_s, applied to its normalised output
    w[u] = fast_exp2(__uint_as_float(mbits[u]) - ref) * __uint_as_float(lbits[u]);
    asm volatile("" : "+v"(w[u]));                     // formed here, not behind the wait for the outputs
  }
  mb_out = mb;
}

template <int CH, int B0>
__device__ __forceinline__ void batch_accumulate(MergeLane<CH>& L, typename ChunkOf<CH>::type (&t)[8], int c0, const OwnRows& own,
                                                 const float (&w)[8], float fa, float mb) {
  const int ou = own.split - c0 - B0;
  if (ou >= 0 && ou < 8) {
    // (a tree of uniform branches with one assignment at each leaf: a store with a run-time index
    // would move the fetched outputs from registers to scratch memory, eight selects cost eight
    // times as much behind the wait)
    if (ou & 4) {
      if (ou & 2) { if (ou & 1) t[7] = L.own_chunk; else t[6] = L.own_chunk; }
      else { if (ou & 1) t[5] = L.own_chunk; else t[4] = L.own_chunk; }
    } else {
      if (ou & 2) { if (ou & 1) t[3] = L.own_chunk; else t[2] = L.own_chunk; }
      else { if (ou & 1) t[1] = L.own_chunk; else t[0] = L.own_chunk; }
    }
  }
  // (in front of the very first batch the sums are zero and stay zero: 0 x fa = +0)
  if (!(B0 == 0 && c0 == 0)) {
    L.l_acc *= fa;
#pragma unroll
    for (int c = 0; c < CH; ++c) L.acc[c] *= fa;
  }
#pragma unroll
  for (int u = 0; u < 8; ++u) {
    L.l_acc += w[u];
#pragma unroll
    for (int c = 0; c < CH; ++c) L.acc[c] += w[u] * chunk_value<CH>(t[u], c);
  }
  L.m_acc = mb;
}

template <int CH>
__device__ __forceinline__ void init_lane(MergeLane<CH>& L, int mt, int r0, int hi) {
  const int rr = r0 + mt / MergeLane<CH>::kLanesPerRow;
  L.cl = mt % MergeLane<CH>::kLanesPerRow;
  L.active = rr < hi && rr < 32;
  L.row = L.active ? rr : r0;
#pragma unroll
  for (int c = 0; c < CH; ++c) L.acc[c] = 0.f;
  L.m_acc = -INFINITY;
  L.l_acc = 0.f;
}

// The merged row goes out (CH channels per thread) with its log-sum-exp.
template <int CH>
__device__ __forceinline__ void merged_row_address(const AttnParams& p, MergeLane<CH>& L, int row0, int64_t orow_pair) {
  const int grow = row0 + L.row;
  const int oi = (int)(((uint64_t)(uint32_t)grow * p.g_magic) >> 32), oj = grow - oi * p.G;
  L.orow = (L.active && grow < p.M) ? orow_pair + (int64_t)oi * p.Hq + oj : -1;
  asm volatile("" : "+v"(L.orow));                       // worked out here, not behind the wait for the outputs
}
template <int CH>
__device__ __forceinline__ void store_merged(const AttnParams& p, const MergeLane<CH>& L) {
  const int64_t orow = L.orow;
  if (orow < 0) return;
  const float inv = L.l_acc > 0.f ? __builtin_amdgcn_rcpf(L.l_acc) : 0.f;   // a row that saw no key at all: zero, lse = -inf
  typename ChunkOf<CH>::type o;
#pragma unroll
  for (int c = 0; c < CH / 2; ++c) o[c] = pack_bf16(L.acc[2 * c] * inv, L.acc[2 * c + 1] * inv);
  *reinterpret_cast<typename ChunkOf<CH>::type*>(static_cast<__hip_bfloat16*>(p.out) + orow * kD + L.cl * CH) = o;
  if (p.lse && L.cl == 0) p.lse[orow] = (L.m_acc + log2f(L.l_acc)) * 0.6931471805599453f;
}

template <typename T>
__device__ __forceinline__ void chunks_wait16(T (&a)[8], T (&b)[8]) {
  asm volatile("s_waitcnt vmcnt(0)"
               : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(a[4]), "+v"(a[5]), "+v"(a[6]), "+v"(a[7]),
                 "+v"(b[0]), "+v"(b[1]), "+v"(b[2]), "+v"(b[3]), "+v"(b[4]), "+v"(b[5]), "+v"(b[6]), "+v"(b[7])
               :
               : "memory");
}

// Splits c0 .. c0 + 15 of the lane's row, once their records are in (poll_records): fetches their
// outputs and, while those are on their way, forms the weights.  The own split's rows, if LDS holds
// them, must be complete.
template <int CH>
__device__ __forceinline__ void merge_fetch_weigh(const AttnParams& p, MergeLane<CH>& L, int pair, int row0, int c0,
                                                  const OwnRows& own, int64_t orow_pair) {
  const int S = p.n_splits;
  const uint32_t voff = (uint32_t)(((row0 + L.row) * kD + L.cl * CH) * 2);
  // (straight-line code between every hand-issued load and its wait: the compiler does not know
  // that the registers are still in flight, and a copy it places at a branch or a join in between
  // would copy what was there before)
  if (c0 + 8 < S) {
    fetch_batch<CH, 0>(p, L.t0, pair, voff, c0);
    fetch_batch<CH, 8>(p, L.t1, pair, voff, c0);
    batch_weights<CH, 0>(L, c0, own, L.m_acc, L.w0, L.fa0, L.mb0);
    batch_weights<CH, 8>(L, c0, own, L.mb0, L.w1, L.fa1, L.mb1);
    merged_row_address(p, L, row0, orow_pair);
    chunks_wait16(L.t0, L.t1);
  } else {
    fetch_batch<CH, 0>(p, L.t0, pair, voff, c0);
    batch_weights<CH, 0>(L, c0, own, L.m_acc, L.w0, L.fa0, L.mb0);
    merged_row_address(p, L, row0, orow_pair);
    chunks_wait(L.t0);
  }
}
template <int CH>
__device__ __forceinline__ void merge_finish(const AttnParams& p, MergeLane<CH>& L, int c0, const OwnRows& own) {
  batch_accumulate<CH, 0>(L, L.t0, c0, own, L.w0, L.fa0, L.mb0);
  if (c0 + 8 < p.n_splits) batch_accumulate<CH, 8>(L, L.t1, c0, own, L.w1, L.fa1, L.mb1);
}

// Merges rows lo <= r < hi of the row group (all passes, all splits) and writes them out.  Returns
// false for the whole wavefront, with nothing of the current pass written, when a record was still
// missing after `budget` polls.  Called by the two merging wavefronts, each for itself.
template <int CH>
__device__ __forceinline__ bool merge_rows(const AttnParams& p, int lo, int hi, int budget, uint32_t tag, int pair, int row0,
                                           int64_t orow_pair, int mt, const OwnRows& own) {
  for (int r0 = lo; r0 < hi; r0 += MergeLane<CH>::kRowsPerPass) {
    MergeLane<CH> L;
    init_lane(L, mt, r0, hi);
    if (!__any(L.active)) continue;
    for (int c0 = 0; c0 < p.n_splits; c0 += 16) {
      const int64_t g_row = (int64_t)pair * p.n_splits * p.Mpad + row0 + L.row;
      if (!poll_records(p, L, g_row, c0, tag, budget, own.split)) return false;
      merge_fetch_weigh(p, L, pair, row0, c0, own, orow_pair);
      merge_finish(p, L, c0, own);
    }
    store_merged(p, L);
  }
  return true;
}

// Where the kernel learns which rows to fetch.
constexpr int kResolve = 0;   // sel_idx / sel_cnt in memory, page table walked per tile
constexpr int kGather = 1;    // gather list left behind by an earlier selection
constexpr int kSelect = 2;    // the workgroup retrieves for itself (scores + top-N), builds its own
                              // gather entries, then as kGather
constexpr int kTableLoads = 8;   // page-table entries a thread stages in LDS (rows up to 8 * kThreads pages)

constexpr int kMaxSelectBlocks = 1024;   // blocks per sequence the in-kernel retrieval handles

// Top-cnt of keys[0 .. nb) by the whole workgroup (Sec. 3.1 top-N rule; equal keys: lowest index
// first).  nb <= kMaxSelectBlocks = 2 * kThreads, so a thread holds keys tid and tid + kThreads.
// Four 8-bit radix passes find the key of the weakest kept block: LDS histogram (one per pass,
// zeroed by the caller), one barrier, then every wavefront scans the 256 bins for itself (four
// bins per lane, wavefront prefix sum), so no second barrier is needed to share the outcome.
// The final placement needs one more barrier: position of a kept block = blocks above the
// threshold before it + min(equal blocks before it, equal blocks wanted).  sel[0 .. cnt) ends up
// ascending.  Requires 1 <= cnt <= nb; all threads of the workgroup must call.
// first_counted: the caller has already counted every key's top digit into hist[0] and passed a
// barrier since (the keys were counted as they came in): the first pass starts at its scan.
struct SelectScratch {
  uint32_t hist[4][256];
  uint32_t seg[2 * kWaves][2];     // per (key slot, wavefront): blocks above / equal to the threshold
};
__device__ __forceinline__ void workgroup_select(const uint32_t* keys, SelectScratch* sc, int nb, int cnt,
                                                 int32_t* sel, int tid, int lane, int wave, bool first_counted) {
  const bool has0 = tid < nb, has1 = tid + kThreads < nb;
  const uint32_t k0 = has0 ? keys[tid] : 0u, k1 = has1 ? keys[tid + kThreads] : 0u;
  uint32_t prefix = 0, need = (uint32_t)cnt;
#pragma unroll
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    const uint32_t hi_mask = pass == 0 ? 0u : (0xffffffffu << (shift + 8));
    if (!(pass == 0 && first_counted)) {             // (uniform)
      if (has0 && (k0 & hi_mask) == prefix) atomicAdd(&sc->hist[pass][(k0 >> shift) & 0xff], 1u);
      if (has1 && (k1 & hi_mask) == prefix) atomicAdd(&sc->hist[pass][(k1 >> shift) & 0xff], 1u);
      __syncthreads();
    }
    // lane l owns bins 255 - 4l (in .w) down to 252 - 4l (in .x): higher bins in lower lanes
    const uint4 hq = *reinterpret_cast<const uint4*>(&sc->hist[pass][252 - 4 * lane]);
    const uint32_t own = hq.x + hq.y + hq.z + hq.w;
    const uint32_t incl = wave_inclusive_sum(own);
    uint32_t run = incl - own;                      // keys in bins above this lane's
    const bool cross = incl >= need && run < need;  // exactly one lane
    uint32_t bin = 255u - 4u * (uint32_t)lane, in_bin = hq.w;
    if (run + hq.w < need) {
      run += hq.w; --bin; in_bin = hq.z;
      if (run + hq.z < need) {
        run += hq.z; --bin; in_bin = hq.y;
        if (run + hq.y < need) { run += hq.y; --bin; in_bin = hq.x; }
      }
    }
    const int src = __builtin_ctzll(__ballot(cross));
    prefix |= (uint32_t)__builtin_amdgcn_readlane((int)bin, src) << shift;
    need -= (uint32_t)__builtin_amdgcn_readlane((int)run, src);   // still wanted from inside that bin
    // every key of that bin is wanted: no need to look at the lower digits (the threshold is the
    // bin's smallest possible key, and every key equal to it is kept)
    if (need == (uint32_t)__builtin_amdgcn_readlane((int)in_bin, src)) {
      need = 0xffffffffu;
      break;
    }
  }
  const uint32_t tau = prefix;
  const uint64_t below = (1ull << lane) - 1ull;
  const uint64_t gt0 = __ballot(has0 && k0 > tau), eq0 = __ballot(has0 && k0 == tau);
  const uint64_t gt1 = __ballot(has1 && k1 > tau), eq1 = __ballot(has1 && k1 == tau);
  if (lane == 0) {
    sc->seg[wave][0] = (uint32_t)__popcll(gt0);
    sc->seg[wave][1] = (uint32_t)__popcll(eq0);
    sc->seg[kWaves + wave][0] = (uint32_t)__popcll(gt1);
    sc->seg[kWaves + wave][1] = (uint32_t)__popcll(eq1);
  }
  __syncthreads();
  // Counts over the segments in front of a wavefront's keys: lane s of every wavefront reads
  // segment s (both counts in one word: neither sum exceeds 1024), a prefix sum over the sixteen
  // lanes, and the wavefront picks the entries in front of its own two segments - one LDS round
  // trip instead of one per segment.
  uint32_t packed = 0;
  if (lane < 2 * kWaves) {
    const uint2 sg = *reinterpret_cast<const uint2*>(&sc->seg[lane][0]);
    packed = sg.x | (sg.y << 16);
  }
  packed += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)packed, 0x111, 0xf, 0xf, true);   // row_shr:1
  packed += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)packed, 0x112, 0xf, 0xf, true);   // row_shr:2
  packed += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)packed, 0x114, 0xf, 0xf, true);   // row_shr:4
  packed += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)packed, 0x118, 0xf, 0xf, true);   // row_shr:8
  static_assert(2 * kWaves == 16, "one row of sixteen lanes holds the segments");
  const uint32_t before0 = wave > 0 ? (uint32_t)__builtin_amdgcn_readlane((int)packed, wave - 1) : 0u;
  uint32_t gt_before = before0 & 0xffffu, eq_before = before0 >> 16;
  {
    const uint32_t e = eq_before + (uint32_t)__popcll(eq0 & below);
    const bool is_gt = (gt0 >> lane) & 1ull, is_eq = (eq0 >> lane) & 1ull;
    if (is_gt || (is_eq && e < need)) sel[gt_before + (uint32_t)__popcll(gt0 & below) + min(e, need)] = tid;
  }
  if (nb > kThreads) {
    const uint32_t before1 = (uint32_t)__builtin_amdgcn_readlane((int)packed, kWaves + wave - 1);
    gt_before = before1 & 0xffffu;
    eq_before = before1 >> 16;
    const uint32_t e = eq_before + (uint32_t)__popcll(eq1 & below);
    const bool is_gt = (gt1 >> lane) & 1ull, is_eq = (eq1 >> lane) & 1ull;
    if (is_gt || (is_eq && e < need)) sel[gt_before + (uint32_t)__popcll(gt1 & below) + min(e, need)] = tid + kThreads;
  }
}

// ---- retrieval inside the attention kernel (anchor layers) ------------------------------------
// q0 = mean first-draft query of the group, key[j] = order-preserving key of q0 . rep[j] (forced
// sink / local blocks get the largest key), top-cnt by the workgroup.  With more than one split
// the workgroups of an exchange group share the scoring: each scores every n_splits-th pass of 64
// blocks and publishes its keys as 64-bit words (key, tag of this call); the others poll those
// words.  The tag is a per-group counter in the workspace that moves on by one per call.
constexpr int kScoreChunks = kD / (4 * kScoreLanes);   // 16-byte chunks of a representative per lane
constexpr int kScoreBatch = 8;                         // passes (of 64 blocks) in flight

// Polls a workgroup spends waiting for the other workgroups of its group, from the high half of
// the group's epoch word: 0 = the default, else the caller's number plus one.
__device__ __forceinline__ int wait_polls_of(int high_half) {
  return high_half == 0 ? kDefaultWaitPolls : min(high_half - 1, kMaxWaitPolls);
}

// The call with tag `tag` is over for this group (every workgroup has read the call counter and is
// past every wait on the others): the counter moves on, and the arrival word that the next call's
// workgroups will count in starts from zero.  Called by one thread.
__device__ __forceinline__ void finish_call(const AttnParams& p, int64_t group, uint32_t tag) {
  __hip_atomic_store(p.tickets + group * kTicketWords + ((tag & 1u) ^ 1u), 0ull, __ATOMIC_RELAXED,
                     __HIP_MEMORY_SCOPE_AGENT);
  __hip_atomic_store(p.tickets + group * kTicketWords + 4 + ((tag & 1u) ^ 1u), 0ull, __ATOMIC_RELAXED,
                     __HIP_MEMORY_SCOPE_AGENT);
  *reinterpret_cast<uint32_t*>(p.epochs + group) = tag;      // the low half
}

// What a retrieving workgroup loads up front, together with its query loads.
struct RetrievalLoads {
  QueryHeads<__hip_bfloat16> q0h;       // channel tid mod 128 of the group's first-draft query heads
  const __hip_bfloat16* q0ch;
  const int32_t* table_row;             // the sequence's page-table row ...
  int32_t tbl[kTableLoads];             // ... and this thread's entries of it, on their way to LDS
  bool table_in_lds;
  bool table_wide;                      // entries 4 tid .. 4 tid + 3 (16-byte loads) instead of tid, tid + 512, ...
  bool share_scores;
  uint64_t epoch_word;                  // the group's call counter (low half) and wait budget (high half) as loaded
  int rot;                              // first pass of a workgroup that scores alone
  float4 r[kScoreBatch][kScoreChunks];  // first batch of representative rows
};

__device__ __forceinline__ const float* reps_lane_ptr(const AttnParams& p, int pair, int tid) {
  return p.reps + (int64_t)pair * p.nb_max * kD + (tid % kScoreLanes) * 4;
}

// Loads the representative rows of passes first, first + stride, ... into r (pass = 64 blocks).
__device__ __forceinline__ void load_score_batch(const AttnParams& p, const float* rp, int jrow, int first, int stride,
                                                 bool rotate, int rot, float4 (&r)[kScoreBatch][kScoreChunks]) {
#pragma unroll
  for (int u = 0; u < kScoreBatch; ++u) {
    const int ps = first + stride * (rotate ? (u + rot) % kScoreBatch : u);
    if (ps * 64 < p.nb_max) {
      const float* row = rp + (int64_t)min(ps * 64 + jrow, p.nb_max - 1) * kD;
#pragma unroll
      for (int i = 0; i < kScoreChunks; ++i) r[u][i] = *reinterpret_cast<const float4*>(row + i * 4 * kScoreLanes);
    }
  }
}

__device__ __forceinline__ RetrievalLoads issue_retrieval_loads(const AttnParams& p, int b, int h, int pair, int split,
                                                                int xgroup, int rot, int tid, int vzero) {
  RetrievalLoads R;
  // first in the queue, so that nothing slower has to come back before it
  R.q0ch = static_cast<const __hip_bfloat16*>(p.q) + ((int64_t)b * p.gamma * p.Hq + (int64_t)h * p.G) * kD + (tid & (kD - 1));
  // (only the first kD threads use theirs.  A workgroup can hand the memory pipeline one load
  // instruction per ~20 cycles, whatever its size, so the instructions issued up front, not their
  // bytes, set how soon the retrieval starts.)
  if (tid < kD) R.q0h = load_query_heads<__hip_bfloat16>(R.q0ch, p.G, kD);
  // the page-table row goes to LDS while the scores are computed, so that turning kept blocks
  // into addresses afterwards costs no further trip to memory
  R.table_row = p.table + (int64_t)b * p.kv.max_pages;
  R.table_in_lds = p.kv.page_size != 0 && p.kv.max_pages <= kTableLoads * kThreads;
  R.share_scores = p.n_splits >= 2;
  R.epoch_word = p.epochs[xgroup + vzero];
  R.rot = rot;
  R.table_wide = (p.kv.max_pages & 3) == 0 && (reinterpret_cast<uintptr_t>(p.table) & 15) == 0;
  if (R.table_in_lds) {
    if (R.table_wide) {
#pragma unroll
      for (int u = 0; u < kTableLoads / 4; ++u)
        if (4 * u * kThreads < p.kv.max_pages) {
          const int4 t = *reinterpret_cast<const int4*>(R.table_row + min(4 * (tid + u * kThreads), p.kv.max_pages - 4));
          R.tbl[4 * u] = t.x;
          R.tbl[4 * u + 1] = t.y;
          R.tbl[4 * u + 2] = t.z;
          R.tbl[4 * u + 3] = t.w;
        }
    } else {
#pragma unroll
      for (int u = 0; u < kTableLoads; ++u)
        if (u * kThreads < p.kv.max_pages) R.tbl[u] = R.table_row[min(tid + u * kThreads, p.kv.max_pages - 1)];
    }
  }
  return R;
}

// The first batch of representative rows: this workgroup's share, or the first passes of all.
__device__ __forceinline__ void issue_first_score_batch(const AttnParams& p, RetrievalLoads& R, int pair, int split,
                                                        int tid) {
  const float* rp = reps_lane_ptr(p, pair, tid);
  if (R.share_scores) load_score_batch(p, rp, tid / kScoreLanes, split, p.n_splits, false, R.rot, R.r);
  else load_score_batch(p, rp, tid / kScoreLanes, 0, 1, true, R.rot, R.r);
}

struct Retrieved {
  int L, cnt;
  uint32_t tag;
  const int32_t* s_table;               // the page-table row in LDS (valid if table_in_lds)
};

// Scores, exchange, selection.  On return s_sel[0 .. cnt) holds the kept blocks (ascending) and
// every thread has passed the barrier behind the selection.  The scratch arrays live in stage 0
// and the page-table row in stage 1 (stages 2 and up are the caller's); the caller must not stream
// into them before its own next barrier.  L_raw: the sequence length as loaded (per lane, not yet uniform).
// meanwhile(): work of the caller's that may run behind the first barrier (what the caller wrote
// to its stages before the call is visible there) while the other workgroups' keys are on their way.
template <typename Meanwhile>
__device__ __forceinline__ Retrieved retrieve_blocks(const AttnParams& p, RetrievalLoads& R, unsigned char* smem,
                                                     int32_t* s_sel, int* s_exchange_failed, int L_raw, int pair,
                                                     int split, int xgroup, int tid, int lane, int wave,
                                                     Meanwhile&& meanwhile) {
  int32_t* s_table = reinterpret_cast<int32_t*>(smem + kStageBytes);
  float* s_q0 = reinterpret_cast<float*>(smem);
  uint32_t* s_keys = reinterpret_cast<uint32_t*>(smem + kD * 4);
  SelectScratch* s_sc = reinterpret_cast<SelectScratch*>(smem + kD * 4 + kMaxSelectBlocks * 4);
  const int sub = tid % kScoreLanes, jrow = tid / kScoreLanes;
  const float* rp = reps_lane_ptr(p, pair, tid);
  uint64_t* const xk = p.xkeys + (int64_t)xgroup * p.nb_max;

  if (tid < kD) s_q0[tid] = mean_query_channel<__hip_bfloat16>(R.q0h, R.q0ch, p.G, kD);
  for (int i = tid; i < 4 * 256; i += kThreads) (&s_sc->hist[0][0])[i] = 0;
  if (tid == 0) *s_exchange_failed = 0;
  if (R.table_in_lds) {
    if (R.table_wide) {
#pragma unroll
      for (int u = 0; u < kTableLoads / 4; ++u)
        if (4 * (tid + u * kThreads) < p.kv.max_pages)
          *reinterpret_cast<int4*>(s_table + 4 * (tid + u * kThreads)) =
              make_int4(R.tbl[4 * u], R.tbl[4 * u + 1], R.tbl[4 * u + 2], R.tbl[4 * u + 3]);
    } else {
#pragma unroll
      for (int u = 0; u < kTableLoads; ++u)
        if (tid + u * kThreads < p.kv.max_pages) s_table[tid + u * kThreads] = R.tbl[u];
    }
  }
  __syncthreads();
  Retrieved out;
  out.L = __builtin_amdgcn_readfirstlane(L_raw);
  out.s_table = s_table;
  const int nb = (out.L + p.block_size - 1) / p.block_size;
  out.cnt = min(p.k_blocks, nb);
  out.tag = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)R.epoch_word) + 1u;
  const uint32_t tag = out.tag;
  const int poll_budget = wait_polls_of(__builtin_amdgcn_readfirstlane((int)(uint32_t)(R.epoch_word >> 32)));
  float4 qv[kScoreChunks];
#pragma unroll
  for (int i = 0; i < kScoreChunks; ++i) qv[i] = *reinterpret_cast<const float4*>(s_q0 + sub * 4 + i * 4 * kScoreLanes);
  // scores the rows in R.r (passes first, first + stride, ...): keys go to LDS and, if published,
  // tagged to the group's exchange array through a write-through store
  // (publish: also counted into the first histogram of the selection, like the keys that come in
  // from the other workgroups below, so that the barrier behind the exchange is the first pass's)
  auto score_batch = [&](int first, int stride, bool rotate, bool publish) {
#pragma unroll
    for (int u = 0; u < kScoreBatch; ++u) {
      const int ps = first + stride * (rotate ? (u + R.rot) % kScoreBatch : u);
      if (ps * 64 < nb) {                              // uniform
        const float v = block_score<kScoreChunks>(R.r[u], qv);
        const int j = ps * 64 + jrow;
        if (sub == 0 && j < nb) {
          const uint32_t key = (j < p.n_sink || j >= nb - p.n_local) ? 0xffffffffu : score_key(v + 0.0f);
          s_keys[j] = key;
          if (publish) {
            __hip_atomic_store(xk + j, (uint64_t)key | ((uint64_t)tag << 32), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            atomicAdd(&s_sc->hist[0][key >> 24], 1u);
          }
        }
      }
    }
  };
  bool score_alone = !R.share_scores;
  if (R.share_scores) {
    // this workgroup's share (nb <= 1024 = 16 passes, at least two splits: one batch), then
    // the others' keys: a key is valid once its word carries this call's tag.  The wait is
    // bounded; a workgroup that runs out of patience scores everything itself.
    score_batch(split, p.n_splits, false, true);
    meanwhile();
    const int j0 = tid, j1 = tid + kThreads;
    bool need0 = j0 < nb && ((j0 >> 6) % p.n_splits) != split;
    bool need1 = j1 < nb && ((j1 >> 6) % p.n_splits) != split;
    const bool mine0 = need0, mine1 = need1;
    uint32_t got0 = 0, got1 = 0;
    for (int it = 0; it < poll_budget; ++it) {
      if (need0) {
        const uint64_t w = __hip_atomic_load(xk + j0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if ((uint32_t)(w >> 32) == tag) {
          got0 = (uint32_t)w;
          need0 = false;
          atomicAdd(&s_sc->hist[0][got0 >> 24], 1u);
        }
      }
      if (need1) {
        const uint64_t w = __hip_atomic_load(xk + j1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if ((uint32_t)(w >> 32) == tag) {
          got1 = (uint32_t)w;
          need1 = false;
          atomicAdd(&s_sc->hist[0][got1 >> 24], 1u);
        }
      }
      if (!__any(need0 || need1)) break;
    }
    if (need0 || need1) *s_exchange_failed = 1;
    if (mine0 && !need0) s_keys[j0] = got0;
    if (mine1 && !need1) s_keys[j1] = got1;
    __syncthreads();
    score_alone = *s_exchange_failed != 0;
    // (for the statistics of svf_diag_wait_fallbacks: no answer needed)
    if (score_alone && tid == 0)
      __hip_atomic_fetch_add(p.tickets + (int64_t)xgroup * kTicketWords + kTicketExchangeFallbacks, 1ull, __ATOMIC_RELAXED,
                             __HIP_MEMORY_SCOPE_AGENT);
  }
  if (!R.share_scores) meanwhile();
  if (score_alone) {                                   // (the same for the whole workgroup)
    // (a starved exchange has left some keys counted: the selection counts for itself; everybody is
    // past the barrier behind the exchange, and the barrier below comes before the selection's adds)
    if (R.share_scores)
      for (int i = tid; i < 256; i += kThreads) s_sc->hist[0][i] = 0;
    const bool loaded = !R.share_scores;               // the up-front batch was this one
    for (int f = 0; f * 64 < nb; f += kScoreBatch) {
      if (!(loaded && f == 0)) load_score_batch(p, rp, jrow, f, 1, true, R.rot, R.r);
      score_batch(f, 1, true, false);
    }
    __syncthreads();                                   // (after an exchange the barrier above has done this)
  }
  if (out.cnt > 0) workgroup_select(s_keys, s_sc, nb, out.cnt, s_sel, tid, lane, wave, !score_alone);
  __syncthreads();
  return out;
}

// Gather entry of the four selected-token slots 4e .. 4e+3 from the selection in LDS.
__device__ __forceinline__ uint64_t gather_entry_of(const AttnParams& p, const int32_t* s_sel, const Retrieved& rt,
                                                    const RetrievalLoads& R, int e, int b, int h) {
  const int slot0 = 4 * e;
  if (slot0 >= rt.cnt * p.block_size) return 0ull;
  const int bi = p.block_shift >= 0 ? slot0 >> p.block_shift : slot0 / p.block_size;
  const int tok0 = s_sel[bi] * p.block_size + (slot0 - bi * p.block_size);
  const int nv = min(max(rt.L - tok0, 0), 4);
  if (nv <= 0) return 0ull;
  int64_t row;                                         // element offset of the token's row of head 0
  if (p.kv.page_size == 0) {
    row = (int64_t)b * p.kv.stride_page + (int64_t)tok0 * p.kv.stride_tok;
  } else {
    const int pg = p.kv.page_shift >= 0 ? tok0 >> p.kv.page_shift : tok0 / p.kv.page_size;
    const int phys = R.table_in_lds ? rt.s_table[pg] : R.table_row[pg];
    row = (int64_t)phys * p.kv.stride_page + (int64_t)(tok0 - pg * p.kv.page_size) * p.kv.stride_tok;
  }
  const uint64_t off = (uint64_t)((row + (int64_t)h * p.kv.stride_head) * 2);
  return (off & kGatherOffsetMask) | ((uint64_t)nv << kGatherCountShift);
}

// One workgroup of the pair publishes the selection for the layers that reuse it.
__device__ __forceinline__ void publish_selection(const AttnParams& p, const int32_t* s_sel, int cnt, int pair, int tid) {
  int32_t* out_idx = p.sel_idx_out + (int64_t)pair * p.k_blocks;
  for (int i = tid; i < p.k_blocks; i += kThreads) out_idx[i] = i < cnt ? s_sel[i] : -1;
  if (tid == 0) p.sel_cnt_out[pair] = cnt;
}

// What the main loop has to know about a tile whose loads have been issued.
struct TileInfo {
  uint32_t valid;      // bit s set: slot s holds a real token
  int draft_base;      // >= 0: draft tile, index of its first draft; -1: cache tile
};

// grid: x = kXcds * n_splits, y = ceil(pairs / kXcds), z = row groups; pairs = B * Hkv.
// Workgroups are handed to the XCDs round-robin in x-fastest order and gridDim.x is a multiple
// of kXcds, so blockIdx.x mod kXcds names the XCD: all splits and all row groups of a pair
// share it (the second reader of a pair's K/V finds them in that XCD's L2).
// MODE kGather: the addresses of the selected rows come from the gather list that an earlier
// selection left behind (one load, issued together with the query loads) instead of the chain
// sel_idx -> page table -> address.
// MODE kSelect (anchor layers, Sec. 3.3): every workgroup first retrieves for its (sequence, KV
// head) itself: block scores from the representatives (Eq. 5), then the top-N rule, both in
// LDS; the workgroups of a pair repeat this work (they share an XCD, so the representatives
// come out of its L2 after the first), which costs less than two more launches.  The result is
// written to sel_idx / sel_cnt and, tile by tile, to the gather list for the layers that reuse it.
// kOneTile: no wavefront has more than one tile of the cache (the launcher knows).  Then only
// wavefronts 0 .. 3 compute: wavefront w takes its own tile and, after a barrier, the tile that
// wavefront w + 4 (same SIMD) has fetched into its stage - the second wavefront of a SIMD gets its
// loads out last anyway.  Four slices instead of eight go through the combination below (whose
// cost is its instruction count: 0.5 instead of 1.0 us), four wavefronts instead of eight load
// query fragments, and the tiles that arrive last are computed by wavefronts that have the SIMD
// to themselves.  Also (MODE kGather): which of the up-front loads go out first, see below.
template <int MODE, bool kOneTile>
__global__ __launch_bounds__(kThreads) void verify_attn_mfma_kernel(AttnParams p, int pairs) {
  // one stage per wavefront, plus one for draft tile 0 (its owner then streams its cache tile
  // at the same time); after the main loop stage w becomes wavefront w's fp32 output buffer
  __shared__ __attribute__((aligned(1024))) unsigned char smem[(kWaves + 1) * kStageBytes];
  __shared__ float sm_m[kWaves][32];
  __shared__ float sm_l[kWaves][32];
  __shared__ uint32_t sm_pair_valid[kWaves / 2];   // (kOneTile) what wavefront w + 4 fetched: valid slots,
  __shared__ int sm_pair_draft[kWaves / 2];        // draft base (-1: cache tile, -2: nothing)
  __shared__ int sm_last;
  __shared__ int sm_own_ready;                     // wavefronts 0 .. 3 that have left their part of the own rows in LDS
  __shared__ int sm_one_xcd;                       // every workgroup of the group is known to run on this XCD
  __shared__ int32_t s_sel[MODE == kSelect ? kMaxSelectBlocks : 1];   // kept blocks, ascending
  __shared__ int s_exchange_failed;

  // The kernel arguments are read piecemeal further down, and every scalar-memory wait is a wait
  // for all scalar loads: touch each 64-byte line of the argument block once now, so that the
  // later reads come out of the scalar cache.
  {
    const __attribute__((address_space(4))) uint32_t* ka =
        (const __attribute__((address_space(4))) uint32_t*)__builtin_amdgcn_kernarg_segment_ptr();
    static_assert(sizeof(AttnParams) > 5 * 64, "argument block shorter than the lines touched");
    const uint32_t w0 = ka[0], w1 = ka[16], w2 = ka[32], w3 = ka[48], w4 = ka[64], w5 = ka[80];
    asm volatile("" : : "s"(w0), "s"(w1), "s"(w2), "s"(w3), "s"(w4), "s"(w5));
  }
  // Values that are the same for the whole workgroup but come from device memory (lengths,
  // counts) are loaded through the vector path with this opaque zero in the address: a scalar
  // load would stall the next read of a kernel argument until it is back.
  int vzero;
  asm volatile("v_mov_b32 %0, 0" : "=v"(vzero));
  const int split = blockIdx.x / kXcds;
  const int pair = blockIdx.y * kXcds + blockIdx.x % kXcds;
  const int rg = blockIdx.z;
  if (pair >= pairs) return;
  const int group = rg * pairs + pair;                          // index of the group's ticket
  const int b = (int)(((uint64_t)(uint32_t)pair * p.hkv_magic) >> 32), h = pair - b * p.Hkv;   // pair / Hkv

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int l32 = lane & 31, g = lane >> 5;
  const int row0 = rg * 32;
  const int NW = kWaves * p.n_splits;
  const int gw = split * kWaves + wave;
  constexpr int kSlices = kOneTile ? kWaves / 2 : kWaves;      // wavefronts that compute
  const bool computes = wave < kSlices;                         // (wave-uniform)
  // Draft tile 0 has a stage of its own, of which only the four-token groups that hold a draft
  // are fetched (two of eight for eight drafts: 4 load instructions instead of 32).  The V rows
  // of the other groups must still be finite (their weights are zero, and 0 x NaN is not): the
  // wavefront that owns the tile clears them now, before it has any load in flight.  What the K
  // rows hold does not matter: the scores of slots without a token are replaced.
  if (gw == 0) {
    const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int k = 0; k < kTileBytes / 1024; ++k)
      *reinterpret_cast<u32x4*>(smem + kWaves * kStageBytes + kTileBytes + k * 1024 + lane * 16) = zero;
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  }
  const int tiles_d = (p.gamma + kTile - 1) / kTile;           // draft tiles come first

  const char* Kc = static_cast<const char*>(p.K);
  const char* Vc = static_cast<const char*>(p.V);
  const char* Kd = static_cast<const char*>(p.k_draft);
  const char* Vd = static_cast<const char*>(p.v_draft);
  const int32_t* __restrict__ sel_g = p.sel_idx + (int64_t)pair * p.k_blocks;

  // ---- this lane's query row as B operands (issued first: vector loads complete in order, so
  // a wait for these must not have the K/V stream in front of it), and the row's draft mask ----
  const int row = row0 + l32;
  const bool row_valid = row < p.M;
  int qi = 0, qj = 0;
  if (row_valid) {
    qi = (int)(((uint64_t)(uint32_t)row * p.g_magic) >> 32);            // row / G
    qj = row - qi * p.G;
  }
  // (retrieval only) what the retrieval needs goes out first, ahead of the query fragments
  RetrievalLoads rl;
  if (MODE == kSelect)
    rl = issue_retrieval_loads(p, b, h, pair, split, group, (split + rg * p.n_splits) % kScoreBatch, tid, vzero);
  const int32_t* const table_row = p.table + (int64_t)b * p.kv.max_pages;
  // With a gather list the tile loads wait for nothing but their gather entries.  Where a
  // wavefront has one tile (kOneTile) the entries (with the draft mask and the pair's block
  // count) go out ahead of the query fragments, which may then arrive while the tile is on its
  // way: 0.4 us per launch.  Where wavefronts walk several tiles one after the other the
  // fragments go first and everything is waited for: the earlier start loses there (measured:
  // 15.2 against 15.7 us per launch with two to three tiles per wavefront) - the compute units
  // then alternate between fetching and computing in step with each other.
  // Lane 8u + n holds the entry of group n of the wavefront's u-th tile.  All of these loads are
  // issued by hand (the compiler, which cannot see hand-issued loads, would make the wait for a
  // load of its own a wait for the fragments as well), unconditionally, from addresses that are
  // valid either way; nothing of them is used before front_loads_arrived().
  uint64_t rmask = 0;
  uint64_t gent = 0;
  u32x2 rmask_raw = {0u, 0u}, gent_raw = {0u, 0u}, epoch_raw = {0u, 0u};
  uint32_t cnt_raw = 0;
  bool gent_wanted = false;
  auto request_entries = [&]() {
    const int tc = gw + (lane >> 3) * NW - tiles_d;          // cache tile index
    const int e = tc * 8 + (lane & 7);
    gent_wanted = lane < 8 * kMaxTiles && tc >= 0 && e < p.gather_groups;
    const uint64_t* gsrc = p.gather + (int64_t)pair * p.gather_groups + (gent_wanted ? e : 0);
    const uint64_t* msrc = p.draft_mask ? p.draft_mask + (p.mask_per_batch ? (int64_t)b * p.gamma + qi : qi) : gsrc;
    gent_raw = load8_plain(gsrc);
    rmask_raw = load8_plain(msrc);
    cnt_raw = load4_plain(p.sel_cnt + pair + vzero);
    epoch_raw = load8_plain(p.epochs + group + vzero);
  };
  if (MODE == kGather && kOneTile) request_entries();
  bf16x8 qf[8];
  // A retrieving workgroup has barriers ahead anyway: its 32 query rows come in once (16 bytes
  // per thread) and reach the wavefronts' registers through LDS (chunk c of row r at position
  // c ^ (r & 15)), instead of eight loads per lane in each of the eight wavefronts.
  unsigned char* const q_stage = smem + 2 * kStageBytes;
  u32x4 qpiece = {0u, 0u, 0u, 0u};
  if (MODE == kSelect) {
    const int r = tid >> 4, rrow = row0 + r;
    int ri = 0, rj = 0;
    if (rrow < p.M) {
      ri = (int)(((uint64_t)(uint32_t)rrow * p.g_magic) >> 32);
      rj = rrow - ri * p.G;
    }
    qpiece = *reinterpret_cast<const u32x4*>(static_cast<const __hip_bfloat16*>(p.q) +
                                             (((int64_t)b * p.gamma + ri) * p.Hq + h * p.G + rj) * kD + (tid & 15) * 8);
  } else {
    const __hip_bfloat16* qrow = static_cast<const __hip_bfloat16*>(p.q) +
                                 (((int64_t)b * p.gamma + qi) * p.Hq + h * p.G + qj) * kD + g * 8;
    if (MODE == kGather) {
      // issued by hand: the fragments are in once at most one tile's loads are outstanding (see
      // below), which the compiler's own bookkeeping would turn into a full wait inside the loop
      if (computes) load_query_fragments(qf, qrow);
    } else if (computes) {
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) qf[ks] = *reinterpret_cast<const bf16x8*>(qrow + ks * 16);
    }
  }
  if (MODE == kGather && !kOneTile) request_entries();
  // Draft tile 0 into its own stage, by its owner, ahead of everything that depends on the kept
  // blocks (the draft rows need no gather entry, and they are measured to arrive last).  Not in
  // a retrieving launch: there every barrier of the retrieval, and every LDS access the compiler
  // issues, would wait for these loads (+0.3 us).
  int early_draft_loads = 0;
  auto request_draft_tile = [&]() {
    const int er = lane >> 4;
    const uint32_t ecx = (uint32_t)((lane & 15) ^ er);
    const uint32_t drow = (uint32_t)p.Hkv * kRowBytes;
    const char* kd = Kd + (((int64_t)b * p.gamma) * p.Hkv + h) * kRowBytes;
    const int64_t dvd = Vd - Kd;
    unsigned char* xs = smem + kWaves * kStageBytes;
#pragma unroll
    for (int n = 0; n < 8; ++n) {
      const int nvn = min(max(p.gamma - 4 * n, 0), 4);     // drafts in slots 4n .. 4n + 3 (uniform)
      if (nvn == 0) continue;
      const uint32_t off = (uint32_t)(4 * n + min(er, nvn - 1)) * drow + ((ecx ^ (uint32_t)((4 * n) & 15)) << 4);
      __builtin_amdgcn_global_load_lds(SVF_GLOBAL_PTR(kd + off), SVF_LDS_PTR(xs + n * 1024), 16, 0, 2);
      __builtin_amdgcn_global_load_lds(SVF_GLOBAL_PTR(kd + dvd + off), SVF_LDS_PTR(xs + kTileBytes + n * 1024), 16, 0, 2);
      early_draft_loads += 2;
    }
  };
  // (with a gather list: now, without waiting for the entries)
  if (MODE == kGather && gw == 0) request_draft_tile();
  if (MODE != kGather && p.draft_mask) rmask = p.draft_mask[p.mask_per_batch ? (int64_t)b * p.gamma + qi : qi];

  int L = 0;
  if (MODE != kGather) L = clamped_len(p.seq_lens, b + vzero, p.max_seq_len);
  if (MODE == kSelect) issue_first_score_batch(p, rl, pair, split, tid);
  if (MODE == kSelect) {
    const int r = tid >> 4;
    *reinterpret_cast<u32x4*>(q_stage + r * kRowBytes + (((tid & 15) ^ (r & 15)) << 4)) = qpiece;
  }
  int cnt;
  // the group's epoch word: this call's tag (for the key exchange of a retrieval and for the
  // split partials) is its low half plus one, its high half the wait budget
  uint64_t epoch_word = 0;
  if (MODE == kResolve) epoch_word = p.epochs[group + vzero];
  if (MODE == kSelect) {
    epoch_word = rl.epoch_word;
    const Retrieved rt = retrieve_blocks(p, rl, smem, s_sel, &s_exchange_failed, L, pair, split, group, tid, lane, wave, [&]() {
      if (computes) {
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
          qf[ks] = *reinterpret_cast<const bf16x8*>(q_stage + l32 * kRowBytes + (((2 * ks + g) ^ (l32 & 15)) << 4));
      }
    });
    L = rt.L;
    cnt = rt.cnt;
    // gather entries of this wavefront's tiles (lane 8u + n: group n of its u-th tile), kept for
    // the loads below and written out for the layers that reuse the selection, together with the
    // selection itself, right in front of the stream
    {
      const int tc = gw + (lane >> 3) * NW - tiles_d;                          // cache tile index
      const int e = tc * 8 + (lane & 7);
      if (lane < 8 * kMaxTiles && tc >= 0 && e < p.gather_groups) gent = gather_entry_of(p, s_sel, rt, rl, e, b, h);
    }
    __syncthreads();                 // the last reads of the staged page table and the query rows are done
  } else if (MODE == kGather) {
    // everything requested ahead of the eight query fragments (and of an early draft tile), or everything
    if (kOneTile && computes) wait_vmcnt_upto24(8 + early_draft_loads); else wait_vmcnt_upto24(early_draft_loads);
    front_loads_arrived(gent_raw, rmask_raw, cnt_raw, epoch_raw);
    epoch_word = (uint64_t)epoch_raw[0] | ((uint64_t)epoch_raw[1] << 32);
    if (gent_wanted) gent = (uint64_t)gent_raw[0] | ((uint64_t)gent_raw[1] << 32);
    if (p.draft_mask) rmask = (uint64_t)rmask_raw[0] | ((uint64_t)rmask_raw[1] << 32);
    cnt = __builtin_amdgcn_readfirstlane(min(max((int)cnt_raw, 0), p.k_blocks));
  } else {
    cnt = __builtin_amdgcn_readfirstlane(min(max(p.sel_cnt[pair + vzero], 0), p.k_blocks));
  }
  const int n_prefix = cnt * p.block_size;
  const int tiles = tiles_d + (n_prefix + kTile - 1) / kTile;
  int n_my = 0;
  if (gw < tiles) n_my = (tiles - gw + NW - 1) / NW;
  n_my = min(n_my, kMaxTiles);
  // Where the group's workgroups run.  Workgroups are dealt to the XCDs so that all splits of a
  // group should share one, but nothing guarantees it: every workgroup adds one to its XCD's
  // counter in a word of the group (no answer needed; by the last wavefront, which never waits
  // for a particular number of its loads), and looks at the word later.  A workgroup that then
  // finds all n_splits of them counted on its own XCD knows that every reader of its partial sits
  // behind the same L2, and may leave the partial there instead of writing it through to memory.
  uint64_t* const where_word = p.tickets + (int64_t)group * kTicketWords + 4 + (((uint32_t)epoch_word + 1u) & 1u);
  const bool counts_xcds = p.n_splits >= 2 && p.n_splits <= 255;
  if (counts_xcds && wave == kWaves - 1 && lane == 0)
    __hip_atomic_fetch_add(where_word, 1ull << (8 * xcc_id()), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);

  // per-lane parts of the load addresses: load n of a tile covers slots 4n .. 4n+3, sixteen lanes
  // per slot; chunk swizzle: 16-byte chunk c of the row in slot s sits at position c ^ (s & 15)
  const int lrow = lane >> 4;                              // row of this lane inside a load
  const uint32_t cx = (uint32_t)((lane & 15) ^ lrow);     // chunk of load n: cx ^ (4n & 15)
  const uint32_t tok_bytes = (uint32_t)p.kv.stride_tok * 2u;
  const uint32_t drow_bytes = (uint32_t)p.Hkv * kRowBytes;
  const int64_t dv_c = Vc - Kc, dv_d = Vd - Kd;
  const char* const kd_pair = Kd + (((int64_t)b * p.gamma) * p.Hkv + h) * kRowBytes;
  // cache rows of this pair: page 0 (or, without paging, the sequence's own slab), token 0
  const char* const kc_pair = Kc + ((int64_t)(p.kv.page_size == 0 ? b : 0) * p.kv.stride_page +
                                    (int64_t)h * p.kv.stride_head) * 2;
  const int64_t orow_pair = (int64_t)b * p.gamma * p.Hq + h * p.G;      // output row of (draft 0, head 0)

  // Resolves the addresses of tile t (the wavefront's u-th) and issues its 16 loads into the
  // stage at `dst`.  Lane 8u + n resolves the group of slots 4n .. 4n+3 (without a gather list
  // every lane with lane & 7 == n does); the groups' bases then move to scalar registers.  Rows that do not exist (past the drafts, past the kept blocks, past the
  // sequence's end) are redirected to the nearest valid row of their group, or, if the whole
  // group is void, to the first draft row (finite, always mapped); they are masked out of the
  // softmax through `valid`.
  auto issue_tile = [&](int t, int u, unsigned char* dst, bool skip_void_groups) -> TileInfo {
    TileInfo ti;
    const int n8 = lane & 7;
    const int src0 = __builtin_amdgcn_readfirstlane(8 * u);
    int nv;                         // valid rows in this lane's group (0..4)
    int64_t base;                   // byte address of the group's first K row
    bool from_draft;
    uint32_t row_bytes;
    if (t < tiles_d) {              // wave-uniform
      const int d0 = t * kTile + 4 * n8;
      nv = min(max(p.gamma - d0, 0), 4);
      base = (int64_t)(uintptr_t)kd_pair + (int64_t)(nv > 0 ? d0 : 0) * drow_bytes;
      from_draft = true;
      row_bytes = drow_bytes;
      ti.draft_base = t * kTile;
    } else if (MODE != kResolve) {
      nv = (int)(gent >> kGatherCountShift);
      base = nv > 0 ? (int64_t)(uintptr_t)Kc + (int64_t)(gent & kGatherOffsetMask) : (int64_t)(uintptr_t)kd_pair;
      from_draft = nv == 0;
      row_bytes = tok_bytes;
      ti.draft_base = -1;
    } else {
      const int slot0 = (t - tiles_d) * kTile + 4 * n8;
      const bool in_range = slot0 < n_prefix;
      const int sl = in_range ? slot0 : 0;
      const int bi = p.block_shift >= 0 ? sl >> p.block_shift : sl / p.block_size;
      const int blk = sel_g[bi];
      const int tok0 = blk * p.block_size + (sl - bi * p.block_size);
      nv = (in_range && blk >= 0) ? min(max(min(n_prefix - slot0, L - tok0), 0), 4) : 0;
      const int tk = nv > 0 ? tok0 : 0;
      int phys, sl_in_page;
      if (p.kv.page_size == 0) {
        phys = 0;
        sl_in_page = tk;
      } else {
        const int pg = p.kv.page_shift >= 0 ? tk >> p.kv.page_shift : tk / p.kv.page_size;
        sl_in_page = tk - pg * p.kv.page_size;
        phys = nv > 0 ? table_row[pg] : 0;
      }
      // byte offset of the group's first K row from the start of the pool
      const int64_t off = (kc_pair - Kc) + ((int64_t)phys * p.kv.stride_page + (int64_t)sl_in_page * p.kv.stride_tok) * 2;
      base = nv > 0 ? (int64_t)(uintptr_t)Kc + off : (int64_t)(uintptr_t)kd_pair;
      from_draft = nv == 0;
      row_bytes = tok_bytes;
      ti.draft_base = -1;
    }
    // slot validity: slot s is valid iff (s mod 4) < nv of group s / 4 (collected below from the
    // groups' counts as they pass through scalar registers)
    uint32_t valid = 0;
    unsigned char* vdst = dst + kTileBytes;
    // (one multiplication per tile, not one per group: min(row, k) x bytes = min(row x bytes, k x bytes))
    const uint32_t lrow_off = (uint32_t)lrow * row_bytes;
#pragma unroll
    for (int n = 0; n < 8; ++n) {
      const uint32_t lo = __builtin_amdgcn_readlane((uint32_t)base, src0 + n);
      const uint32_t hi = __builtin_amdgcn_readlane((uint32_t)((uint64_t)base >> 32), src0 + n);
      const int nvn = __builtin_amdgcn_readlane(nv, src0 + n);
      valid |= ((1u << nvn) - 1u) << (4 * n);
      const bool fd = __builtin_amdgcn_readlane((int)from_draft, src0 + n) != 0;
      const char* kb = reinterpret_cast<const char*>(((uint64_t)hi << 32) | lo);
      const char* vb = kb + (fd ? dv_d : dv_c);
      // rows past the group's last valid row re-read that row
      const uint32_t last_off = (uint32_t)max(nvn - 1, 0) * (uint32_t)__builtin_amdgcn_readfirstlane((int)row_bytes);
      const uint32_t off = min(lrow_off, last_off) + ((cx ^ (uint32_t)((4 * n) & 15)) << 4);
      if (skip_void_groups && nvn == 0) continue;        // (wave-uniform)
      __builtin_amdgcn_global_load_lds(SVF_GLOBAL_PTR(kb + off), SVF_LDS_PTR(dst + n * 1024), 16, 0, 2);
      __builtin_amdgcn_global_load_lds(SVF_GLOBAL_PTR(vb + off), SVF_LDS_PTR(vdst + n * 1024), 16, 0, 2);
    }
    ti.valid = valid;
    return ti;
  };

  float m_run = -INFINITY, l_run = 0.f;
  floatx16 oacc[4];
#pragma unroll
  for (int nt = 0; nt < 4; ++nt)
#pragma unroll
    for (int v = 0; v < 16; ++v) oacc[nt][v] = 0.f;

  // ---- main loop -----------------------------------------------------------------------------
  unsigned char* const my_stage = smem + wave * kStageBytes;
  unsigned char* const x_stage = smem + kWaves * kStageBytes;
  const bool own_x = gw == 0;            // owner of draft tile 0
  // Without a gather list everything loaded so far is needed before the stream starts anyway
  // (draining the counter here keeps later register reuse from being mistaken for a hazard
  // against the stream); with one, the query fragments may still be on their way.
  if (MODE != kGather) wait_vmcnt<0>();
  // The selection and the gather list for the layers that reuse them: stored here, in front of the
  // stream (their acknowledgements come back long before the first tile does; stored behind the
  // stream instead, an anchor launch took 0.14 us longer).  The workgroup with the least other work
  // publishes the selection (s_sel is not a stage).
  if (MODE == kSelect) {
    if (split == p.n_splits - 1 && rg == 0) publish_selection(p, s_sel, cnt, pair, tid);
    const int tc = gw + (lane >> 3) * NW - tiles_d;
    const int e = tc * 8 + (lane & 7);
    if (rg == 0 && lane < 8 * kMaxTiles && tc >= 0 && e < p.gather_groups)
      p.gather_out[(int64_t)pair * p.gather_groups + e] = gent;
  }
  if (!p.draft_mask) rmask = qi >= 63 ? ~0ull : ((2ull << qi) - 1ull);     // linear causal drafts
  if (!row_valid) rmask = 0;

  TileInfo cur = {0u, -1}, nxt = {0u, -1};
  int issued = 0;
  if (n_my > 0) {
    // (draft tile 0 in its own stage: only the groups that hold a draft are fetched)
    if (early_draft_loads) {
      cur.valid = p.gamma >= 32 ? 0xffffffffu : ((1u << p.gamma) - 1u);
      cur.draft_base = 0;
    } else {
      cur = issue_tile(gw, 0, own_x ? x_stage : my_stage, own_x);
    }
    issued = 1;
    if (own_x && n_my > 1) {
      nxt = issue_tile(gw + NW, 1, my_stage, false);
      issued = 2;
    }
    // The query fragments were requested before the tiles and loads complete in order: with at
    // most one tile's loads outstanding they are in (a second tile may still be in flight).
    if (MODE == kGather && computes) wait_vmcnt<16>();
  } else if (MODE == kGather) {
    wait_vmcnt<0>();
  }
  if (MODE == kGather && computes) query_fragments_arrived(qf);
  // (the word comes back behind this wavefront's tile, which it waits for anyway)
  uint64_t where = 0;
  if (counts_xcds && wave == kWaves - 1 && lane == 0)
    where = __hip_atomic_load(where_word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  for (int u = 0; computes && u < n_my; ++u) {
    if (u >= issued) {                   // the single stage is free again: fetch the next tile
      cur = issue_tile(gw + u * NW, u, my_stage, false);
      issued = u + 1;
    }
    // tiles are issued in order, 16 loads each
    if (issued - (u + 1) >= 1) wait_vmcnt<16>(); else wait_vmcnt<0>();
    uint32_t allowed = cur.valid;
    if (cur.draft_base >= 0) allowed &= (uint32_t)(rmask >> (cur.draft_base & 63));
    const bool all_visible = cur.draft_base < 0 && cur.valid == 0xffffffffu;
    const uint32_t stage = (uint32_t)(uintptr_t)SVF_LDS_PTR((own_x && u == 0) ? x_stage : my_stage);
    process_tile(stage, qf, allowed, all_visible, p.scale_log2, l32, g, m_run, l_run, oacc);
    cur = nxt;
  }
  if (kOneTile) {
    // wavefronts 4 .. 7 hand their tile over: once its loads have landed, what the tile holds
    // goes to LDS, and behind the barrier wavefront w continues with the stage of wavefront w + 4
    if (!computes) {
      wait_vmcnt<0>();
      if (lane == 0) {
        sm_pair_valid[wave - kSlices] = cur.valid;
        sm_pair_draft[wave - kSlices] = n_my > 0 ? cur.draft_base : -2;
      }
    }
    __syncthreads();
    if (computes) {
      const uint32_t pvalid = sm_pair_valid[wave];
      const int pdraft = sm_pair_draft[wave];
      if (pdraft != -2) {
        uint32_t allowed = pvalid;
        if (pdraft >= 0) allowed &= (uint32_t)(rmask >> (pdraft & 63));
        const bool all_visible = pdraft < 0 && pvalid == 0xffffffffu;
        const uint32_t stage = (uint32_t)(uintptr_t)SVF_LDS_PTR(smem + (wave + kSlices) * kStageBytes);
        process_tile(stage, qf, allowed, all_visible, p.scale_log2, l32, g, m_run, l_run, oacc);
      }
    }
  }

  // ---- combine the computing wavefronts through LDS ---------------------------------------------
  // Wavefront w parks its fp32 output, as it stands (relative to its own running maximum), in its
  // own stage as [32 rows][32 float4] straight out of the accumulator registers: float4 nt * 8 +
  // k * 2 + g of a row holds accumulator nt, values 4k .. 4k + 3, i.e. channels 32 nt + 8k + 4g +
  // 0 .. 3, which is channel block (that index): float4 j = channels 4j .. 4j + 3, at position
  // parked_position(j) ^ row, which keeps the writes (32 rows, one j per instruction) and the reads
  // (eight threads of a row, j = 4c .. 4c + 3 each) off each other's banks.  After the one
  // barrier wavefronts 0 .. 3 (256 threads: eight per row, sixteen consecutive channels = four
  // consecutive float4 each) bring the slices to the common maximum while they add them.
  l_run = halves_sum(l_run);
  if (computes) {
    if (g == 0) {
      sm_m[wave][l32] = m_run;
      sm_l[wave][l32] = l_run;
    }
    float4* mine = reinterpret_cast<float4*>(my_stage);
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
      for (int nt = 0; nt < 4; ++nt)
        mine[l32 * 32 + (parked_position(nt * 8 + k * 2 + g) ^ l32)] =
            make_float4(oacc[nt][4 * k], oacc[nt][4 * k + 1], oacc[nt][4 * k + 2], oacc[nt][4 * k + 3]);
  }
  if (tid == kMergeWave0 * 64) sm_own_ready = 0;
  if (wave == kWaves - 1 && lane == 0)
    sm_one_xcd = counts_xcds && where == (uint64_t)p.n_splits << (8 * xcc_id()) ? 1 : 0;
  __syncthreads();

  // ---- what happens to the workgroup's result --------------------------------------------------------
  // One split: wavefronts 0 .. 3 write out / lse.  Otherwise the splits of a group are merged by
  // all its workgroups, each a slice of p.slice_rows rows:
  //  - wavefronts 0 .. 3 write the workgroup's partial (normalised output in bf16) through to
  //    device-coherent memory, leave the rows of the workgroup's own slice in LDS as well, and,
  //    once the stores have been acknowledged, write a record per row (maximum, tag, denominator,
  //    tag; tag = this call's);
  //  - meanwhile wavefronts 4 and 5 wait (bounded) until the other splits' records of the slice's
  //    rows carry the tag and fetch those partials; behind one barrier they add the own rows from
  //    LDS, in split order (bit-stable: the same sums whoever computes them), and write out / lse.
  //    In the workgroup that is last of its group everything but that final sum has happened by
  //    the time its own partial exists; in the others the merge is one poll and one round of loads
  //    behind the last record.  No return trip through an atomic lies on that path.
  // The wait is bounded.  A wavefront that runs out of patience marks its workgroup's slice as given
  // up in the group's arrival word, unless that word shows that every workgroup has arrived (then
  // every partial is on its way and it keeps waiting).  Every workgroup takes a ticket from that
  // word when it has stored its partial; the one that arrives last sees which slices were given up
  // before it and merges them too.  So every row is merged whatever is resident when, and every
  // wait ends.  The words of calls with an even / odd tag alternate; the last arriver clears the
  // other one and moves the call counter on (which also works under graph replay).
  const int S = p.n_splits;
  const bool single = S == 1;
  const uint32_t tag = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)epoch_word) + 1u;
  const int wait_polls = wait_polls_of(__builtin_amdgcn_readfirstlane((int)(uint32_t)(epoch_word >> 32)));
  uint64_t* const arrivals = p.tickets + (int64_t)group * kTicketWords + (tag & 1u);
  const int R = p.slice_rows;
  const int lo = split * R, hi = min(lo + R, 32);            // the workgroup's own slice (empty if lo >= 32)
  unsigned char* const own_o = x_stage;                     // [R][kD] bf16, R <= 16
  float* const own_ml = reinterpret_cast<float*>(x_stage + 16 * kRowBytes);
  uint64_t prev = 0;
  int64_t pr_rec = 0;
  float mw = -INFINITY, lw = 0.f;
  const int r = tid >> 3, c16 = tid & 7;                     // (wavefronts 0 .. 3) row, block of 16 channels
  if (wave < 4) {
    float fw[kSlices];
#pragma unroll
    for (int w = 0; w < kSlices; ++w) {
      fw[w] = sm_m[w][r];
      mw = fmaxf(mw, fw[w]);
    }
#pragma unroll
    for (int w = 0; w < kSlices; ++w) {
      fw[w] = fw[w] == -INFINITY ? 0.f : fast_exp2(fw[w] - mw);      // a slice that saw no token counts nothing
      lw = __builtin_fmaf(sm_l[w][r], fw[w], lw);
    }
    float racc[16];
#pragma unroll
    for (int c = 0; c < 16; ++c) racc[c] = 0.f;
#pragma unroll
    for (int w = 0; w < kSlices; ++w)
#pragma unroll
      for (int nt = 0; nt < 4; ++nt) {
        const float4 t = reinterpret_cast<const float4*>(smem + w * kStageBytes)[r * 32 + (parked_position(c16 * 4 + nt) ^ r)];
        racc[4 * nt] = __builtin_fmaf(t.x, fw[w], racc[4 * nt]);
        racc[4 * nt + 1] = __builtin_fmaf(t.y, fw[w], racc[4 * nt + 1]);
        racc[4 * nt + 2] = __builtin_fmaf(t.z, fw[w], racc[4 * nt + 2]);
        racc[4 * nt + 3] = __builtin_fmaf(t.w, fw[w], racc[4 * nt + 3]);
      }
    const float inv = lw > 0.f ? __builtin_amdgcn_rcpf(lw) : 0.f;
    u32x4 o0, o1;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      o0[c] = pack_bf16(racc[2 * c] * inv, racc[2 * c + 1] * inv);
      o1[c] = pack_bf16(racc[8 + 2 * c] * inv, racc[8 + 2 * c + 1] * inv);
    }
    const int orow_row = row0 + r;
    if (single) {
      if (orow_row < p.M) {
        const int oi = (int)(((uint64_t)(uint32_t)orow_row * p.g_magic) >> 32), oj = orow_row - oi * p.G;
        const int64_t orow = orow_pair + (int64_t)oi * p.Hq + oj;
        __hip_bfloat16* dst = static_cast<__hip_bfloat16*>(p.out) + orow * kD + c16 * 16;
        *reinterpret_cast<u32x4*>(dst) = o0;
        *reinterpret_cast<u32x4*>(dst + 8) = o1;
        if (p.lse && c16 == 0) p.lse[orow] = (mw + log2f(lw)) * 0.6931471805599453f;
      }
    } else {
      pr_rec = ((int64_t)pair * S + split) * p.Mpad + orow_row;
      // Each of the two store instructions covers whole 128-byte lines (the eight threads of a row
      // write eight consecutive 16-byte chunks; threads c and c ^ 4 trade their second chunk): the
      // L2 then passes complete lines on instead of twice as many half-written ones.
      const bool low = c16 < 4;
      u32x4 got;
#pragma unroll
      for (int c = 0; c < 4; ++c) got[c] = swap_lanes_xor4(o1[c]);
      const u32x4 first = low ? o0 : got, second = low ? got : o0;
      uint16_t* dst = reinterpret_cast<uint16_t*>(p.part_o) + pr_rec * kD;
      uint16_t* dst0 = dst + (low ? 2 * c16 : 2 * c16 - 7) * 8;
      uint16_t* dst1 = dst + (low ? 2 * c16 + 9 : 2 * c16) * 8;
      const bool one_xcd = sm_one_xcd != 0;               // (the same for the whole workgroup)
      if (one_xcd) {
        store_l2_16(dst0, first);
        store_l2_16(dst1, second);
      } else {
        store_coherent16(dst0, first);
        store_coherent16(dst1, second);
      }
      if (r >= lo && r < hi) {
        *reinterpret_cast<u32x4*>(own_o + (r - lo) * kRowBytes + c16 * 32) = o0;
        *reinterpret_cast<u32x4*>(own_o + (r - lo) * kRowBytes + c16 * 32 + 16) = o1;
        if (c16 == 0) {
          own_ml[2 * (r - lo)] = mw;
          own_ml[2 * (r - lo) + 1] = lw;
        }
      }
      // The merging wavefronts are told through a counter in LDS, not through a barrier: this
      // wavefront must get its records out whatever they are waiting for (they wait for other
      // workgroups' records, and those workgroups' merging wavefronts for ours).  Only the LDS
      // writes above have to be complete, not the stores of the partial.
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      if (lane == 0) {
        const uint32_t ready = (uint32_t)(uintptr_t)SVF_LDS_PTR(&sm_own_ready);
        asm volatile("ds_add_u32 %0, %1" : : "v"(ready), "v"(1u) : "memory");
      }
      // every row is held by eight threads of one wavefront: its own acknowledgements are enough
      wait_vmcnt<0>();
      if (c16 == 0) {
        const u32x4 rec = {__float_as_uint(mw), tag, __float_as_uint(lw), tag};
        if (one_xcd) store_l2_16(p.part_rec + pr_rec * 4, rec);
        else store_coherent16(p.part_rec + pr_rec * 4, rec);
      }
      if (tid == 0) prev = __hip_atomic_fetch_add(arrivals, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
  if (single) return;

  const bool merger = wave == kMergeWave0 || wave == kMergeWave0 + 1;
  const int mt = tid - kMergeWave0 * 64;
  const bool ch4 = R <= 4;                                   // 4 channels per merging thread, else 8
  // one pass over the rows and one batch of records: the other splits' records are waited for now
  const bool prefetch = S <= 16 && R <= (ch4 ? 4 : 8) && lo < 32;
  MergeLane<4> L4;
  MergeLane<8> L8;
  bool records_in = false;
  // the own rows are in LDS once wavefronts 0 .. 3 have all said so (they wait for nobody); the
  // polls for the records look at that counter as well
  const uint32_t ready = (uint32_t)(uintptr_t)SVF_LDS_PTR(&sm_own_ready);
  bool own_rows_in = false;
  if (merger && prefetch) {
    const int64_t g_row0 = (int64_t)pair * S * p.Mpad + row0;
    if (ch4) {
      init_lane(L4, mt, lo, hi);
      records_in = !__any(L4.active) || poll_records(p, L4, g_row0 + L4.row, 0, tag, wait_polls, split, ready, 4u, &own_rows_in);
    } else {
      init_lane(L8, mt, lo, hi);
      records_in = !__any(L8.active) || poll_records(p, L8, g_row0 + L8.row, 0, tag, wait_polls, split, ready, 4u, &own_rows_in);
    }
  }
  if (merger && !own_rows_in) {
    for (int it = 0; it < kLastResortPolls; ++it) {
      uint32_t n;
      asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(n) : "v"(ready) : "memory");
      if (__builtin_amdgcn_readfirstlane((int)n) == 4) break;
      __builtin_amdgcn_s_sleep(1);
    }
  }
  // Slices this wavefront still has to merge (bit x: slice x), the patience it has with them, and
  // whether the last attempt ran out of it.
  uint32_t todo = (merger && lo < 32) ? 1u << split : 0u;
  int budget = wait_polls;
  bool gave_up = false;
  if (merger && prefetch) {
    todo = 0u;
    if (!records_in) {
      gave_up = true;
    } else {
      // the other splits' outputs are fetched; their weights (and the own split's, from LDS) are
      // formed in the meantime
      const OwnRows own = {own_o, own_ml, lo, split};
      if (ch4) {
        if (__any(L4.active)) {
          merge_fetch_weigh(p, L4, pair, row0, 0, own, orow_pair);
          merge_finish(p, L4, 0, own);
          store_merged(p, L4);
        }
      } else if (__any(L8.active)) {
        merge_fetch_weigh(p, L8, pair, row0, 0, own, orow_pair);
        merge_finish(p, L8, 0, own);
        store_merged(p, L8);
      }
    }
  }
  for (int round = 0; round < 2; ++round) {
    while (todo != 0u || gave_up) {
      int x = split;
      if (!gave_up) {
        x = __builtin_ctz(todo);
        todo &= todo - 1u;
        const bool from_lds = x == split;                  // the own slice's own rows are in LDS
        const OwnRows own = {own_o, own_ml, lo, from_lds ? split : -1};
        const bool ok = ch4 ? merge_rows<4>(p, x * R, min(x * R + R, 32), budget, tag, pair, row0, orow_pair, mt, own)
                            : merge_rows<8>(p, x * R, min(x * R + R, 32), budget, tag, pair, row0, orow_pair, mt, own);
        gave_up = !ok;                                     // (only with a bounded budget: the own slice in round 0)
      }
      if (gave_up) {
        gave_up = false;
        uint64_t seen = 0;
        if (lane == 0) {
          seen = __hip_atomic_fetch_or(arrivals, 1ull << (16 + x), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          __hip_atomic_fetch_add(arrivals - (tag & 1u) + kTicketMergeFallbacks, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        const uint32_t arrived = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)seen) & 0xffffu;
        // everybody has arrived, the last arriver may not have seen the mark: keep waiting (it ends)
        if (arrived == (uint32_t)S) {
          todo |= 1u << x;
          budget = kLastResortPolls;
        }
      }
    }
    if (round == 0) {
      __syncthreads();
      if (tid == 0) {
        const bool last = (prev & 0xffffull) == (uint64_t)(S - 1);
        sm_last = last ? (int)((uint32_t)(prev >> 16) & 0xffffu) : 0;
        if (last) finish_call(p, group, tag);
      }
      __syncthreads();
      // (only in the last arriver, and only after a starved wait somewhere in the group)
      todo = merger ? (uint32_t)sm_last : 0u;
      budget = kLastResortPolls;
    }
  }
}


// ---- many query rows per KV head (more than two row groups, e.g. a 60-node draft tree) ----------
// One workgroup per (pair, set of up to eight row groups, split); wavefront w owns row group w and
// all wavefronts walk the same tiles, so a key/value row is fetched once for up to 256 query rows
// instead of once per row group.  A tile is fetched by the eight wavefronts together (wavefront w
// fetches the four-token group w: one K and one V load) into a ring of nine 16 KB stages; one
// barrier per tile (after each wavefront has seen its own two loads land).  No combination through
// LDS at the end: every wavefront writes its rows itself: the output if there is one split, else
// a partial; the partials are merged by the group's workgroups themselves (up to 16 splits) or by
// merge_rows_kernel.
constexpr int kRowStages = kWaves + 1;
constexpr int kRowWindow = 3;                // most tiles between two barriers
constexpr int kRowAhead = 3;                 // tiles requested beyond the window at hand
constexpr int kRowFirst = 3;                 // tiles requested before the first window
static_assert(kRowFirst >= 1 && kRowFirst <= kRowStages, "the first window is one tile");
// (the tiles of a window are requested at the barrier of the window before, at the latest)
static_assert(kRowAhead >= kRowWindow && kRowWindow + kRowAhead <= kRowStages, "tiles in flight must cover the next window and fit the ring");
constexpr int kMaxRowTiles = 64;             // tiles per workgroup: one gather entry per lane
constexpr int kMaxSplitsMergedInKernel = 16; // one bit per split in the upper half of the arrival word's low 32 bits

// What a wavefront of the rows kernel needs to fetch its part of a tile.
struct RowTileIssue {
  unsigned char* smem;
  const char* Kc;
  const char* kd_pair;
  int64_t dv_c, dv_d;
  uint64_t gent;                 // lane u: gather entry of (u-th tile, this wavefront's group)
  int split, S, tiles_d, gamma, wave, lane;
  uint32_t lrow, cx, tok_bytes, drow_bytes;
  uint32_t lrow_tok_off, lrow_draft_off;     // lrow x tok_bytes, lrow x drow_bytes
};

// This wavefront's two loads of the workgroup's i-th tile (slots 4 * wave .. 4 * wave + 3).
__device__ __forceinline__ void issue_row_tile(const RowTileIssue& c, int i) {
  const int t = c.split + i * c.S;
  const int st = i % kRowStages;
  unsigned char* dst = c.smem + st * kStageBytes;
  int nv;
  const char* kb;
  bool from_draft;
  uint32_t row_bytes;
  if (t < c.tiles_d) {
    const int d0 = t * kTile + 4 * c.wave;
    nv = min(max(c.gamma - d0, 0), 4);
    kb = c.kd_pair + (int64_t)(nv > 0 ? d0 : 0) * c.drow_bytes;
    from_draft = true;
    row_bytes = c.drow_bytes;
  } else {
    const uint32_t lo = __builtin_amdgcn_readlane((uint32_t)c.gent, i);
    const uint32_t hi = __builtin_amdgcn_readlane((uint32_t)(c.gent >> 32), i);
    const uint64_t ge = ((uint64_t)hi << 32) | lo;
    nv = (int)(ge >> kGatherCountShift);
    // (selections between two struct members are written with masks: as conditional loads they
    // would pin the whole struct in scratch memory)
    const uint64_t has = (uint64_t)0 - (uint64_t)(nv > 0);
    kb = reinterpret_cast<const char*>(((uint64_t)(uintptr_t)c.Kc + (ge & kGatherOffsetMask)) & has |
                                       (uint64_t)(uintptr_t)c.kd_pair & ~has);
    from_draft = nv == 0;
    row_bytes = c.tok_bytes;
  }
  const uint64_t fd = (uint64_t)0 - (uint64_t)from_draft;
  const char* vb = kb + (int64_t)(((uint64_t)c.dv_d & fd) | ((uint64_t)c.dv_c & ~fd));
  // (min(row, k) x bytes = min(row x bytes, k x bytes): the lane's product is formed once)
  const uint32_t dt = 0u - (uint32_t)(t < c.tiles_d);          // (a draft tile: its rows lie drow_bytes apart)
  const uint32_t lrow_off = (c.lrow_draft_off & dt) | (c.lrow_tok_off & ~dt);
  const uint32_t off = min(lrow_off, (uint32_t)max(nv - 1, 0) * row_bytes) + ((c.cx ^ (uint32_t)((4 * c.wave) & 15)) << 4);
  __builtin_amdgcn_global_load_lds(SVF_GLOBAL_PTR(kb + off), SVF_LDS_PTR(dst + c.wave * 1024), 16, 0, 2);
  __builtin_amdgcn_global_load_lds(SVF_GLOBAL_PTR(vb + off), SVF_LDS_PTR(dst + kTileBytes + c.wave * 1024), 16, 0, 2);
}

template <int MODE>
__global__ __launch_bounds__(kThreads) void verify_attn_mfma_rows_kernel(AttnParams p, int pairs) {
  __shared__ __attribute__((aligned(1024))) unsigned char smem[kRowStages * kStageBytes];
  // per (tile of the workgroup, four-token group): bit s set = slot s of the group holds a real token
  __shared__ __attribute__((aligned(8))) unsigned char s_group_valid[kMaxRowTiles][kWaves];
  __shared__ int sm_last;
  __shared__ int32_t s_sel[MODE == kSelect ? kMaxSelectBlocks : 1];
  __shared__ int s_exchange_failed;

  {
    const __attribute__((address_space(4))) uint32_t* ka =
        (const __attribute__((address_space(4))) uint32_t*)__builtin_amdgcn_kernarg_segment_ptr();
    const uint32_t w0 = ka[0], w1 = ka[16], w2 = ka[32], w3 = ka[48], w4 = ka[64], w5 = ka[80];
    asm volatile("" : : "s"(w0), "s"(w1), "s"(w2), "s"(w3), "s"(w4), "s"(w5));
  }
  int vzero;
  asm volatile("v_mov_b32 %0, 0" : "=v"(vzero));
  const int S = p.n_splits;
  const int split = blockIdx.x / kXcds;
  const int pair = blockIdx.y * kXcds + blockIdx.x % kXcds;
  const int zs = blockIdx.z;                                   // which set of eight row groups
  if (pair >= pairs) return;
  const int b = (int)(((uint64_t)(uint32_t)pair * p.hkv_magic) >> 32), h = pair - b * p.Hkv;
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int l32 = lane & 31, g = lane >> 5;
  const int rgw = zs * kWaves + wave;                          // this wavefront's row group
  const bool has_rows = rgw < p.Mpad / 32;                     // wave-uniform
  const int row0 = rgw * 32;
  const int xgroup = zs * pairs + pair;                        // key-exchange group
  const int tiles_d = (p.gamma + kTile - 1) / kTile;

  const char* Kc = static_cast<const char*>(p.K);
  const char* Vc = static_cast<const char*>(p.V);
  const char* Kd = static_cast<const char*>(p.k_draft);
  const char* Vd = static_cast<const char*>(p.v_draft);
  const int32_t* __restrict__ sel_g = p.sel_idx + (int64_t)pair * p.k_blocks;
  const int32_t* const table_row = p.table + (int64_t)b * p.kv.max_pages;

  const int row = row0 + l32;
  const bool row_valid = has_rows && row < p.M;
  int qi = 0, qj = 0;
  if (row_valid) {
    qi = (int)(((uint64_t)(uint32_t)row * p.g_magic) >> 32);
    qj = row - qi * p.G;
  }
  RetrievalLoads rl;
  if (MODE == kSelect)
    rl = issue_retrieval_loads(p, b, h, pair, split, xgroup, (split + zs * S) % kScoreBatch, tid, vzero);
  // gather entries: lane u holds (the workgroup's u-th tile, group = this wavefront).  With a gather
  // list they and the pair's block count are all the first tile requests wait for: they are loaded
  // ahead of the query fragments (loads come back in the order issued), and the first tiles are
  // requested while the fragments are still on their way.
  const int tc_u = split + lane * S - tiles_d;                 // cache tile index of this lane's tile
  const int e_u = tc_u * 8 + wave;
  const bool e_ok = tc_u >= 0 && e_u < p.gather_groups;
  uint64_t gent = 0;
  int cnt_raw = 0;
  if (MODE == kGather) {
    if (e_ok) gent = p.gather[(int64_t)pair * p.gather_groups + e_u];
    cnt_raw = p.sel_cnt[pair + vzero];
  }
  bf16x8 qf[8];
  {
    const __hip_bfloat16* qrow = static_cast<const __hip_bfloat16*>(p.q) +
                                 (((int64_t)b * p.gamma + qi) * p.Hq + h * p.G + qj) * kD + g * 8;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qf[ks] = *reinterpret_cast<const bf16x8*>(qrow + ks * 16);
  }
  uint64_t rmask = 0;
  if (p.draft_mask) rmask = p.draft_mask[p.mask_per_batch ? (int64_t)b * p.gamma + qi : qi];
  int L = 0;
  if (MODE != kGather) L = clamped_len(p.seq_lens, b + vzero, p.max_seq_len);
  if (MODE == kSelect) issue_first_score_batch(p, rl, pair, split, tid);
  int cnt;
  // the group's epoch word: this call's tag is its low half plus one, its high half the wait budget
  uint64_t epoch_word = 0;
  if (MODE != kSelect) epoch_word = p.epochs[xgroup + vzero];
  if (MODE == kSelect) {
    epoch_word = rl.epoch_word;
    const Retrieved rt = retrieve_blocks(p, rl, smem, s_sel, &s_exchange_failed, L, pair, split, xgroup, tid, lane, wave, []() {});
    L = rt.L;
    cnt = rt.cnt;
    if (e_ok) gent = gather_entry_of(p, s_sel, rt, rl, e_u, b, h);
    __syncthreads();                 // the last reads of the staged page table are done
    // for the layers that reuse this retrieval (s_sel is not a stage): stored in front of the tile loop
    if (split == S - 1 && zs == 0) publish_selection(p, s_sel, cnt, pair, tid);
    if (e_ok && zs == 0) p.gather_out[(int64_t)pair * p.gather_groups + e_u] = gent;
  } else {
    if (MODE != kGather) cnt_raw = p.sel_cnt[pair + vzero];
    cnt = __builtin_amdgcn_readfirstlane(min(max(cnt_raw, 0), p.k_blocks));
    if (MODE == kResolve && tc_u >= 0 && 4 * e_u < cnt * p.block_size) {
      // sel_idx -> page table -> address, one tile per lane
      const int slot0 = 4 * e_u;
      const int bi = p.block_shift >= 0 ? slot0 >> p.block_shift : slot0 / p.block_size;
      const int blk = sel_g[bi];
      const int tok0 = blk * p.block_size + (slot0 - bi * p.block_size);
      const int nv = blk >= 0 ? min(max(L - tok0, 0), 4) : 0;
      if (nv > 0) {
        int64_t rowoff;
        if (p.kv.page_size == 0) {
          rowoff = (int64_t)b * p.kv.stride_page + (int64_t)tok0 * p.kv.stride_tok;
        } else {
          const int pg = p.kv.page_shift >= 0 ? tok0 >> p.kv.page_shift : tok0 / p.kv.page_size;
          rowoff = (int64_t)table_row[pg] * p.kv.stride_page + (int64_t)(tok0 - pg * p.kv.page_size) * p.kv.stride_tok;
        }
        const uint64_t off = (uint64_t)((rowoff + (int64_t)h * p.kv.stride_head) * 2);
        gent = (off & kGatherOffsetMask) | ((uint64_t)nv << kGatherCountShift);
      }
    }
  }
  const int n_prefix = cnt * p.block_size;
  const int tiles = tiles_d + (n_prefix + kTile - 1) / kTile;
  int n_my = 0;
  if (split < tiles) n_my = min((tiles - split + S - 1) / S, kMaxRowTiles);
  n_my = __builtin_amdgcn_readfirstlane(n_my);             // (the same for the whole workgroup)

  const int lrow = lane >> 4;
  const uint32_t cx = (uint32_t)((lane & 15) ^ lrow);
  const uint32_t tok_bytes = (uint32_t)p.kv.stride_tok * 2u;
  const uint32_t drow_bytes = (uint32_t)p.Hkv * kRowBytes;
  const int64_t dv_c = Vc - Kc, dv_d = Vd - Kd;
  const char* const kd_pair = Kd + (((int64_t)b * p.gamma) * p.Hkv + h) * kRowBytes;
  const int64_t orow_pair = (int64_t)b * p.gamma * p.Hq + h * p.G;

  RowTileIssue ic;
  ic.smem = smem;
  ic.Kc = Kc;
  ic.kd_pair = kd_pair;
  ic.dv_c = dv_c;
  ic.dv_d = dv_d;
  ic.gent = gent;
  ic.split = split;
  ic.S = S;
  ic.tiles_d = tiles_d;
  ic.gamma = p.gamma;
  ic.wave = wave;
  ic.lane = lane;
  ic.lrow = (uint32_t)lrow;
  ic.cx = cx;
  ic.tok_bytes = tok_bytes;
  ic.drow_bytes = drow_bytes;
  ic.lrow_tok_off = (uint32_t)lrow * tok_bytes;
  ic.lrow_draft_off = (uint32_t)lrow * drow_bytes;

  float m_run = -INFINITY, l_run = 0.f;
  floatx16 oacc[4];
#pragma unroll
  for (int nt = 0; nt < 4; ++nt)
#pragma unroll
    for (int v = 0; v < 16; ++v) oacc[nt][v] = 0.f;

  // (with a gather list nothing is waited for here: what the first requests need is in, the rest is
  // waited for where it is used, behind those requests)
  if (MODE != kGather) wait_vmcnt<0>();
  int issued = 0;
  if (MODE == kGather)
    for (; issued < min(n_my, kRowFirst); ++issued) issue_row_tile(ic, issued);
  if (!p.draft_mask) rmask = qi >= 63 ? ~0ull : ((2ull << qi) - 1ull);
  if (!row_valid) rmask = 0;

  // Which slots of each tile hold a real token: wavefront w knows it for group w of every tile
  // (lane u: the workgroup's u-th tile); the groups' four-bit masks meet in LDS once, and lane u
  // keeps the 32-bit mask of tile u for the loop below (one v_readlane per tile there).
  uint32_t valid_of_tile = 0;
  {
    const int t_u = split + lane * S;
    int nv_u = 0;
    if (lane < n_my) nv_u = t_u < tiles_d ? min(max(p.gamma - (t_u * kTile + 4 * wave), 0), 4) : (int)(gent >> kGatherCountShift);
    s_group_valid[lane][wave] = (unsigned char)((1u << nv_u) - 1u);
    // (a barrier of LDS traffic only: tile requests and query fragments may be in flight)
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    const u32x2 gv = *reinterpret_cast<const u32x2*>(&s_group_valid[lane][0]);
    // byte n of the pair of words = mask of group n: squeeze the eight low nibbles together
    const uint32_t a = gv[0] | (gv[0] >> 4), c = gv[1] | (gv[1] >> 4);
    valid_of_tile = ((a & 0xffu) | ((a >> 8) & 0xff00u)) | (((c & 0xffu) | ((c >> 8) & 0xff00u)) << 16);
  }

  // ---- main loop: nine stages, tiles taken in windows of one, two, then three ------------------------
  // One barrier per window rather than per tile: behind a barrier all eight wavefronts are in the
  // same phase (all reading LDS, then all on the matrix cores, then all in the softmax); over three
  // tiles they drift apart and one wavefront's MFMA runs under the other's vector work.  The first
  // windows are short so that the arithmetic starts when the first tile is in, not the third.
  // Stages of tiles that everybody has left take the next tiles.
  // Only the first tiles are requested up front and the others as the windows advance (the window
  // at hand plus kRowAhead tiles are in flight): with every tile of every workgroup requested at
  // once, a workgroup's first tile is served no sooner than most of the launch's bytes.
  for (; issued < min(n_my, kRowFirst); ++issued) issue_row_tile(ic, issued);
  for (int i0 = 0, nw = 0; i0 < n_my; i0 += nw) {
    nw = min(min(i0 == 0 ? 1 : (i0 == 1 ? 2 : kRowWindow), kRowWindow), n_my - i0);
    // this wavefront's loads of the window's tiles have landed (two loads per tile, issued in
    // order; the window's tiles were all requested at the barrier before, or up front)
    wait_vmcnt_upto16(2 * (issued - (i0 + nw)));
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    // everybody is done with the tiles in front of this window (at most kRowWindow more than at
    // the barrier before)
#pragma unroll 1
    while (issued < n_my && issued < i0 + nw + kRowAhead && issued < i0 + kRowStages) {
      issue_row_tile(ic, issued);
      ++issued;
    }
    for (int k = 0; k < nw; ++k) {
      const int i = i0 + k;
      const int t = split + i * S;
      const int st = i % kRowStages;
      const uint32_t valid = (uint32_t)__builtin_amdgcn_readlane((int)valid_of_tile, i);
      if (has_rows) {
        const int draft_base = t < tiles_d ? t * kTile : -1;
        uint32_t allowed = valid;
        if (draft_base >= 0) allowed &= (uint32_t)(rmask >> (draft_base & 63));
        const bool all_visible = draft_base < 0 && valid == 0xffffffffu;
        // (one scalar, so that every fragment address is one addition away from it)
        uint32_t stage = (uint32_t)(uintptr_t)SVF_LDS_PTR(smem + st * kStageBytes);
        asm volatile("" : "+s"(stage));
        process_tile(stage, qf, allowed, all_visible, p.scale_log2, l32, g, m_run, l_run, oacc);
      }
    }
  }
  // the other wavefronts may still be reading the last window's stages
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  if (S == 1 && !has_rows) return;   // (with one split: no barrier from here on)

  // ---- this wavefront's 32 rows: output or partial ------------------------------------------------
  // The normalised rows go through LDS once (bf16, [row][128 channels], 16-byte chunk c of row r
  // at position c ^ (r & 15)) so that they leave in whole 256-byte rows: a lane's registers hold
  // 8-byte pieces of 32 different rows.  Behind the barrier above nobody reads a stage any more
  // and no load is in flight.
  l_run = halves_sum(l_run);
  const float inv = l_run > 0.f ? 1.0f / l_run : 0.f;
  if (has_rows) {
    const int last_st = n_my > 0 ? (n_my - 1) % kRowStages : 0;
    unsigned char* mine = smem + ((last_st + 1 + wave) % kRowStages) * kStageBytes;
#pragma unroll
    for (int nt = 0; nt < 4; ++nt)
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        // accumulator nt, values 4k .. 4k + 3: channels 32 nt + 8k + 4g + 0 .. 3 (half g of chunk 4 nt + k)
        const u32x2 w = {pack_bf16(oacc[nt][4 * k] * inv, oacc[nt][4 * k + 1] * inv),
                         pack_bf16(oacc[nt][4 * k + 2] * inv, oacc[nt][4 * k + 3] * inv)};
        *reinterpret_cast<u32x2*>(mine + l32 * kRowBytes + ((((4 * nt + k) ^ (l32 & 15)) << 4) | (g << 3))) = w;
      }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const int rr = 4 * k + (lane >> 4), c = lane & 15;       // row of the group, 16-byte chunk
      const u32x4 w = *reinterpret_cast<const u32x4*>(mine + rr * kRowBytes + ((c ^ (rr & 15)) << 4));
      const int grow = row0 + rr;
      if (S == 1) {
        if (grow < p.M) {
          const int oi = (int)(((uint64_t)(uint32_t)grow * p.g_magic) >> 32);
          const int oj = grow - oi * p.G;
          store_coherent16(static_cast<__hip_bfloat16*>(p.out) + (orow_pair + (int64_t)oi * p.Hq + oj) * kD + c * 8, w);
        }
      } else {
        const int64_t pr = ((int64_t)pair * S + split) * p.Mpad + grow;
        store_coherent16(reinterpret_cast<uint16_t*>(p.part_o) + pr * kD + c * 8, w);
      }
    }
  }
  if (S == 1) {
    if (row_valid && p.lse && g == 0)
      p.lse[orow_pair + (int64_t)qi * p.Hq + qj] = (m_run + log2f(l_run)) * 0.6931471805599453f;
    return;
  }
  // ---- several splits: records, then the merge ------------------------------------------------------
  // Once its partial rows have been acknowledged the wavefront writes a record per row (maximum,
  // tag, denominator, tag; tag = this call's).  Up to 16 splits are then merged here, by all the
  // group's workgroups: workgroup `split` takes the row groups rg with rg mod S == split of its
  // set, pairs of wavefronts eight rows of a row group each, after a bounded wait for the other
  // splits' records (the protocol of verify_attn_mfma_kernel: a slice whose wait ran out is marked
  // in the group's arrival word and merged by the workgroup that arrives last; every wait ends).
  // More splits than that are merged by merge_rows_kernel behind this kernel.
  const uint32_t tag = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)epoch_word) + 1u;
  if (has_rows) {
    wait_vmcnt<0>();
    if (g == 0) {
      const u32x4 rec = {__float_as_uint(m_run), tag, __float_as_uint(l_run), tag};
      store_coherent16(p.part_rec + (((int64_t)pair * S + split) * p.Mpad + row) * 4, rec);
    }
  }
  if (S > kMaxSplitsMergedInKernel) return;            // (uniform)
  const int wait_polls = wait_polls_of(__builtin_amdgcn_readfirstlane((int)(uint32_t)(epoch_word >> 32)));
  uint64_t* const arrivals = p.tickets + (int64_t)xgroup * kTicketWords + (tag & 1u);
  __syncthreads();                                     // every wavefront's records are on their way
  uint64_t prev = 0;
  if (tid == 0) prev = __hip_atomic_fetch_add(arrivals, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  const int nrg = min(kWaves, p.Mpad / 32 - zs * kWaves);      // row groups of this set
  const int mt = (wave & 1) * 64 + lane;                       // thread of the wavefront pair
  const int r_lo = 8 * (wave >> 1);                            // the pair's rows of a row group
  // (what the merge reads of them without looking at it must still be LDS addresses)
  const OwnRows nothing_in_lds = {smem, reinterpret_cast<const float*>(smem), 0, -1};
  uint32_t todo = split < nrg ? 1u << split : 0u;
  int budget = wait_polls;
  bool gave_up = false;
  for (int round = 0; round < 2; ++round) {
    while (todo != 0u || gave_up) {
      int x = split;
      if (!gave_up) {
        x = __builtin_ctz(todo);
        todo &= todo - 1u;
        bool ok = true;
        for (int mrg = x; ok && mrg < nrg; mrg += S)
          ok = merge_rows<8>(p, r_lo, r_lo + 8, budget, tag, pair, (zs * kWaves + mrg) * 32, orow_pair, mt, nothing_in_lds);
        gave_up = !ok;
      }
      if (gave_up) {
        gave_up = false;
        uint64_t seen = 0;
        if (lane == 0) {
          seen = __hip_atomic_fetch_or(arrivals, 1ull << (16 + x), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          __hip_atomic_fetch_add(arrivals - (tag & 1u) + kTicketMergeFallbacks, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        const uint32_t arrived = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)seen) & 0xffffu;
        // everybody has arrived, the last arriver may not have seen the mark: keep waiting (it ends)
        if (arrived == (uint32_t)S) {
          todo |= 1u << x;
          budget = kLastResortPolls;
        }
      }
    }
    if (round == 0) {
      __syncthreads();
      if (tid == 0) {
        const bool last = (prev & 0xffffull) == (uint64_t)(S - 1);
        sm_last = last ? (int)((uint32_t)(prev >> 16) & 0xffffu) : 0;
        if (last) finish_call(p, xgroup, tag);
      }
      __syncthreads();
      // (only in the last arriver, and only after a starved wait somewhere in the group)
      todo = (uint32_t)sm_last;
      budget = kLastResortPolls;
    }
  }
}

// Merge of the rows kernel's split partials: one workgroup per (pair, row group), sixteen threads
// per row, splits in order (bit-stable).  Runs behind the rows kernel on the same stream; it also
// moves the key-exchange tag of a retrieving call on (every workgroup of that call has finished).
// grid: (pairs, row groups)
__global__ __launch_bounds__(kThreads) void merge_rows_kernel(AttnParams p, int pairs, int advance_tags) {
  const int pair = blockIdx.x, rg = blockIdx.y;
  const int tid = threadIdx.x;
  const int r = tid >> 4, cg = tid & 15;
  const int b = (int)(((uint64_t)(uint32_t)pair * p.hkv_magic) >> 32), h = pair - b * p.Hkv;
  const int orow_row = rg * 32 + r;
  const bool rok = orow_row < p.M;
  int oi = 0, oj = 0;
  if (rok) {
    oi = (int)(((uint64_t)(uint32_t)orow_row * p.g_magic) >> 32);
    oj = orow_row - oi * p.G;
  }
  const int64_t orow = (int64_t)b * p.gamma * p.Hq + h * p.G + (int64_t)oi * p.Hq + oj;
  const int64_t g_row = (int64_t)pair * p.n_splits * p.Mpad + orow_row;
  if (advance_tags && tid == 0 && rg % kWaves == 0) {
    const int64_t xg = (int64_t)(rg / kWaves) * pairs + pair;
    finish_call(p, xg, *reinterpret_cast<const uint32_t*>(p.epochs + xg) + 1u);
  }
  merge_splits(p, g_row, orow, rok, cg);
}

}  // namespace

// bf16, d = 128, and groups of four consecutive tokens never straddle a block or a page
bool mfma_supported(const svf_shape_t& s) {
  // (the last two keep the reciprocal-multiply divisions by Hkv and G exact)
  return s.dtype == SVF_BF16 && s.d == 128 && s.block_size % 4 == 0 && s.page_size % 4 == 0 &&
         (int64_t)s.kv_stride_tok * 2 * 3 + 256 < ((int64_t)1 << 31) && (int64_t)s.B * s.Hkv < 65536 &&
         s.Hq < 65536;
}

// Splits per (sequence, KV head, row group): enough workgroups to cover the 256 compute units,
// at most kMaxTiles tiles per wavefront, at least one tile per wavefront.
int mfma_splits(const svf_shape_t& s) {
  const int M = s.gamma * (s.Hq / s.Hkv);
  const int64_t groups = (int64_t)s.B * s.Hkv * ((M + 31) / 32);
  const int64_t tiles = ((int64_t)s.k_blocks * s.block_size + kTile - 1) / kTile + (s.gamma + kTile - 1) / kTile;
  const int64_t lo = (tiles + kWaves * kMaxTiles - 1) / (kWaves * kMaxTiles);
  const int64_t hi = (tiles - 1 + kWaves - 1) / kWaves > 0 ? (tiles - 1 + kWaves - 1) / kWaves : 1;
  int64_t want = (256 + groups - 1) / groups;
  if (want > hi) want = hi;
  if (want < lo) want = lo;
  return (int)want;
}

// More than two row groups: one workgroup takes up to eight of them (see the rows kernel).
constexpr int kRowsModeFrom = 3;
bool mfma_rows_mode(const svf_shape_t& s) {
  const int M = s.gamma * (s.Hq / s.Hkv);
  return (M + 31) / 32 >= kRowsModeFrom;
}

// Splits per (sequence, KV head, set of eight row groups) of the rows kernel: cover the compute
// units; at least one tile and at most kMaxRowTiles tiles per workgroup.
int mfma_rows_splits(const svf_shape_t& s) {
  const int M = s.gamma * (s.Hq / s.Hkv);
  const int row_groups = (M + 31) / 32;
  const int64_t groups = (int64_t)s.B * s.Hkv * ((row_groups + kWaves - 1) / kWaves);
  const int64_t tiles = ((int64_t)s.k_blocks * s.block_size + kTile - 1) / kTile + (s.gamma + kTile - 1) / kTile;
  const int64_t lo = (tiles + kMaxRowTiles - 1) / kMaxRowTiles;
  int64_t want = (256 + groups - 1) / groups;
  if (want > tiles) want = tiles;
  if (want < lo) want = lo;
  return (int)want;
}

// The retrieval of kSelect without the attention behind it (the stand-alone block selection of a
// shape the retrieving attention kernel handles): the workgroups of a (sequence, KV head) share
// the scoring through the key exchange, the last split publishes the kept blocks, and the
// workgroup that finishes last moves the group's tag on.  No page table is touched (p.kv.page_size
// must be 0 here) and no gather list is written.
// grid: x = kXcds * n_splits, y = ceil(pairs / kXcds)
__global__ __launch_bounds__(kThreads) void retrieve_only_kernel(AttnParams p, int pairs) {
  __shared__ __attribute__((aligned(1024))) unsigned char smem[kStageBytes];
  __shared__ int32_t s_sel[kMaxSelectBlocks];
  __shared__ int s_exchange_failed;
  {
    const __attribute__((address_space(4))) uint32_t* ka =
        (const __attribute__((address_space(4))) uint32_t*)__builtin_amdgcn_kernarg_segment_ptr();
    const uint32_t w0 = ka[0], w1 = ka[16], w2 = ka[32], w3 = ka[48], w4 = ka[64], w5 = ka[80];
    asm volatile("" : : "s"(w0), "s"(w1), "s"(w2), "s"(w3), "s"(w4), "s"(w5));
  }
  int vzero;
  asm volatile("v_mov_b32 %0, 0" : "=v"(vzero));
  const int split = blockIdx.x / kXcds;
  const int pair = blockIdx.y * kXcds + blockIdx.x % kXcds;
  if (pair >= pairs) return;
  const int b = (int)(((uint64_t)(uint32_t)pair * p.hkv_magic) >> 32), h = pair - b * p.Hkv;
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  RetrievalLoads rl = issue_retrieval_loads(p, b, h, pair, split, pair, split % kScoreBatch, tid, vzero);
  const int L = clamped_len(p.seq_lens, b + vzero, p.max_seq_len);
  issue_first_score_batch(p, rl, pair, split, tid);
  const Retrieved rt = retrieve_blocks(p, rl, smem, s_sel, &s_exchange_failed, L, pair, split, pair, tid, lane, wave, []() {});
  if (split == p.n_splits - 1) publish_selection(p, s_sel, rt.cnt, pair, tid);
  if (rl.share_scores && tid == 0) {
    // every workgroup that takes a ticket has read all the keys it needed
    uint64_t* const counter = p.tickets + (int64_t)pair * kTicketWords + 2;
    const uint64_t prev = __hip_atomic_fetch_add(counter, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (prev == (uint64_t)(p.n_splits - 1)) {
      __hip_atomic_store(counter, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      finish_call(p, pair, rt.tag);
    }
  }
}

hipError_t launch_retrieve_only(const AttnParams& p, hipStream_t st) {
  const int pairs = p.B * p.Hkv;
  const dim3 grid((unsigned)(kXcds * p.n_splits), (unsigned)((pairs + kXcds - 1) / kXcds));
  hipLaunchKernelGGL(retrieve_only_kernel, grid, dim3(kThreads), 0, st, p, pairs);
  return hipGetLastError();
}

hipError_t launch_verify_attn_mfma(const AttnParams& p, hipStream_t st) {
  const int row_groups = (p.M + 31) / 32;
  const int pairs = p.B * p.Hkv;
  if (row_groups >= kRowsModeFrom) {
    const dim3 grid((unsigned)(kXcds * p.n_splits), (unsigned)((pairs + kXcds - 1) / kXcds),
                    (unsigned)((row_groups + kWaves - 1) / kWaves));
    if (p.reps) hipLaunchKernelGGL(verify_attn_mfma_rows_kernel<kSelect>, grid, dim3(kThreads), 0, st, p, pairs);
    else if (p.gather) hipLaunchKernelGGL(verify_attn_mfma_rows_kernel<kGather>, grid, dim3(kThreads), 0, st, p, pairs);
    else hipLaunchKernelGGL(verify_attn_mfma_rows_kernel<kResolve>, grid, dim3(kThreads), 0, st, p, pairs);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || p.n_splits <= kMaxSplitsMergedInKernel) return e;
    const int advance_tags = p.reps != nullptr;
    hipLaunchKernelGGL(merge_rows_kernel, dim3((unsigned)pairs, (unsigned)row_groups), dim3(kThreads), 0, st, p, pairs,
                       advance_tags);
    return hipGetLastError();
  }
  const dim3 grid((unsigned)(kXcds * p.n_splits), (unsigned)((pairs + kXcds - 1) / kXcds), (unsigned)row_groups);
  // one tile per wavefront (the owner of draft tile 0 streams a second one beside it)?  The same
  // answer for the three modes: they have to add up in the same order (same bits).
  const int64_t tiles = ((int64_t)p.k_blocks * p.block_size + kTile - 1) / kTile + (p.gamma + kTile - 1) / kTile;
  const bool one_tile = tiles - 1 <= (int64_t)kWaves * p.n_splits;
#define SVF_LAUNCH_ATTN(MODE)                                                                              \
  do {                                                                                                     \
    if (one_tile) hipLaunchKernelGGL((verify_attn_mfma_kernel<MODE, true>), grid, dim3(kThreads), 0, st, p, pairs);  \
    else hipLaunchKernelGGL((verify_attn_mfma_kernel<MODE, false>), grid, dim3(kThreads), 0, st, p, pairs);          \
  } while (0)
  if (p.reps) SVF_LAUNCH_ATTN(kSelect);
  else if (p.gather) SVF_LAUNCH_ATTN(kGather);
  else SVF_LAUNCH_ATTN(kResolve);
#undef SVF_LAUNCH_ATTN
  return hipGetLastError();
}

}  // namespace svf
