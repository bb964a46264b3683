// Ceiling measurement for the verification-attention access pattern on one MI355X: plain streaming
// reads and a paged gather of 256-byte rows (16-token pages, 2 KiB token stride), with no compute.
// Build: hipcc -O3 --offload-arch=gfx950 -Xclang -target-feature -Xclang -packed-fp32-ops gather_bw.hip -o gather_bw
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <vector>
#include <algorithm>
#include <random>
#define CK(x) do{hipError_t e=(x); if(e!=hipSuccess){printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1);} }while(0)

// mode 0: contiguous stream read, each thread 16B loads, grid-stride, sum -> sink
__global__ void stream_read(const uint4* __restrict__ p, size_t n16, uint32_t* sink) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  uint32_t acc = 0;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    uint4 a = p[i], b = p[i + stride], c = p[i + 2 * stride], d = p[i + 3 * stride];
    acc += a.x ^ b.y ^ c.z ^ d.w;
  }
  for (; i < n16; i += stride) acc += p[i].x;
  if (acc == 0x12345678) *sink = acc;
}

// gather: work item = (page, head): 16 rows of 256B at 2KiB stride, from K pool and V pool.
// WG of 256 threads = 4 waves; wave handles `ppw` (page,head) items: per item 4 wave-loads for K + 4 for V (each 4 rows x 256B).
// variant REG: loads to registers, xor-accumulate. variant LDS: direct to LDS.
template <bool LDS>
__global__ __launch_bounds__(256) void gather(const char* __restrict__ K, const char* __restrict__ V,
                                              const int* __restrict__ items /* [n_items][2]: page, head */,
                                              int ppw, uint32_t* sink) {
  __shared__ __attribute__((aligned(1024))) char lds[4][32768];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int gw = blockIdx.x * 4 + wave;
  uint32_t acc = 0;
  for (int it = 0; it < ppw; ++it) {
    const int page = items[(gw * ppw + it) * 2], head = items[(gw * ppw + it) * 2 + 1];
    const size_t base = (size_t)page * 32768 + (size_t)head * 256 + (size_t)(lane >> 4) * 2048 + (lane & 15) * 16;
#pragma unroll
    for (int n = 0; n < 4; ++n) {
      const size_t off = base + (size_t)n * 4 * 2048;
      if (LDS) {
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(K + off),
            (__attribute__((address_space(3))) void*)(&lds[wave][(it & 3) * 8192 + n * 1024]), 16, 0, 0);
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(V + off),
            (__attribute__((address_space(3))) void*)(&lds[wave][(it & 3) * 8192 + 4096 + n * 1024]), 16, 0, 0);
      } else {
        uint4 a = *(const uint4*)(K + off), b = *(const uint4*)(V + off);
        acc += a.x ^ b.y;
      }
    }
  }
  if (LDS) {
    __builtin_amdgcn_s_waitcnt(0);
    acc = *(uint32_t*)&lds[wave][lane * 4];
  }
  if (acc == 0x12345678) *sink = acc;
}

int main(int argc, char** argv) {
  const size_t pool_pages = 8192 * 4;          // 1 GiB per pool "layer"; we allocate L layers
  const int L = 8;
  const size_t pool_bytes = pool_pages * 32768;
  char *K, *V; uint32_t* sink;
  CK(hipMalloc(&K, pool_bytes * L)); CK(hipMalloc(&V, pool_bytes * L)); CK(hipMalloc(&sink, 4));
  CK(hipMemset(K, 1, pool_bytes * L)); CK(hipMemset(V, 2, pool_bytes * L));
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  float ms;
  // stream
  for (int grid : {256, 512, 1024, 2048, 4096}) {
    size_t n16 = pool_bytes / 16;   // 1 GiB
    stream_read<<<grid, 256>>>((const uint4*)K, n16, sink);
    CK(hipEventRecord(e0));
    for (int l = 0; l < L; ++l) stream_read<<<grid, 256>>>((const uint4*)(K + l * pool_bytes), n16, sink);
    CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1)); CK(hipEventElapsedTime(&ms, e0, e1));
    printf("stream grid=%d: %.1f GB/s\n", grid, pool_bytes * L / (ms * 1e-3) / 1e9);
  }
  // small stream: 32 MiB per launch (like the attention problem), distinct region per launch
  for (int grid : {256, 512, 1024}) {
    size_t bytes = 32u << 20; size_t n16 = bytes / 16;
    CK(hipEventRecord(e0));
    for (int l = 0; l < 64; ++l) stream_read<<<grid, 256>>>((const uint4*)(K + (size_t)l * (96u << 20)), n16, sink);
    CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1)); CK(hipEventElapsedTime(&ms, e0, e1));
    printf("stream32MiB grid=%d: %.2f us/launch %.1f GB/s\n", grid, ms * 1e3 / 64, bytes * 64 / (ms * 1e-3) / 1e9);
  }
  // gather: per launch 4096 (page,head) items = 32 MiB of K+V (each item 4KiB K + 4KiB V)
  std::mt19937 rng(1);
  const int n_items = 4096;
  std::vector<int> h_items(L * 8 * n_items * 2);
  for (int l = 0; l < L * 8; ++l) {
    std::vector<int> pages(pool_pages); for (size_t i = 0; i < pool_pages; ++i) pages[i] = i;
    std::shuffle(pages.begin(), pages.end(), rng);
    for (int i = 0; i < n_items; ++i) { h_items[(l * n_items + i) * 2] = pages[i]; h_items[(l * n_items + i) * 2 + 1] = rng() % 8; }
  }
  int* items; CK(hipMalloc(&items, h_items.size() * 4)); CK(hipMemcpy(items, h_items.data(), h_items.size() * 4, hipMemcpyHostToDevice));
  for (int lds = 0; lds < 2; ++lds)
    for (int ppw : {1, 2, 4, 8}) {
      int waves = n_items / ppw, grid = waves / 4;
      auto launch = [&](int l) {
        const char* Kl = K + (size_t)(l % L) * pool_bytes; const char* Vl = V + (size_t)(l % L) * pool_bytes;
        if (lds) gather<true><<<grid, 256>>>(Kl, Vl, items + (size_t)l * n_items * 2, ppw, sink);
        else gather<false><<<grid, 256>>>(Kl, Vl, items + (size_t)l * n_items * 2, ppw, sink);
      };
      launch(0); CK(hipDeviceSynchronize());
      CK(hipEventRecord(e0));
      for (int l = 0; l < L * 8; ++l) launch(l);
      CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1)); CK(hipEventElapsedTime(&ms, e0, e1));
      double bytes = (double)n_items * 8192;
      printf("gather lds=%d ppw=%d grid=%d: %.2f us/launch %.1f GB/s\n", lds, ppw, grid, ms * 1e3 / (L * 8), bytes * L * 8 / (ms * 1e-3) / 1e9);
    }
  CK(hipGetLastError());
  return 0;
}
