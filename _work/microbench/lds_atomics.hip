// micro-benchmark: LDS atomic throughput on gfx950 (all addresses masked into the array)
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <vector>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1);} } while (0)
constexpr int NB = 16384;  // 64 KiB of floats
template <int MODE>
__global__ __launch_bounds__(512) void k(const unsigned* __restrict__ idx, float* out, int iters) {
  __shared__ float bins[NB];
  for (int x = threadIdx.x; x < NB; x += 512) bins[x] = 0.f;
  __syncthreads();
  unsigned a = idx[blockIdx.x * 512 + threadIdx.x];
  float p = 1.0f + threadIdx.x * 1e-3f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      unsigned ad = (a + u * 1031u + it * 7919u) & (NB - 1);
      if (MODE == 0) atomicAdd(&bins[ad], p);                                   // ds_add_f32
      else if (MODE == 1) atomicAdd(reinterpret_cast<unsigned*>(bins) + ad, 3u); // ds_add_u32
      else if (MODE == 2) atomicAdd(reinterpret_cast<unsigned long long*>(bins) + (ad >> 1), 3ull); // ds_add_u64
      else if (MODE == 3) bins[ad] = p;                                         // plain store
      else if (MODE == 4) p += bins[ad];                                        // plain load
      else if (MODE == 5) { ad = (ad & ~63u) | (threadIdx.x & 63); atomicAdd(&bins[ad], p); } // conflict-free f32
      else if (MODE == 6) { ad = (u * 64 + it) & (NB - 1); atomicAdd(&bins[ad], p); } // all lanes same address
      else if (MODE >= 7) {  // ds_add_u64, random 256-byte row, the lane's bank pair (8-byte column) by pattern
        const unsigned l = threadIdx.x & 63;
        const unsigned bp = MODE == 7 ? l & 31                              // halves of the wavefront conflict-free
                          : MODE == 8 ? (4 * (l & 15) + (l >> 4)) & 31      // lanes l, l + 8 of a half collide
                          : MODE == 9 ? (l & 15) | (l >> 5) << 4            // lanes l, l + 16 of a half collide
                                      : (l >> 1) & 31;                      // lanes 2i, 2i + 1 collide
        atomicAdd(reinterpret_cast<unsigned long long*>(bins) + (((ad >> 1) & ~31u) | bp), 3ull);
      }
    }
  }
  __syncthreads();
  float s = p;
  for (int x = threadIdx.x; x < NB; x += 512) s += bins[x];
  out[blockIdx.x * 512 + threadIdx.x] = s;
}
template <int MODE> void run(const char* name, unsigned* d_idx, float* d_out, int grid, int iters) {
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  hipLaunchKernelGGL(k<MODE>, dim3(grid), dim3(512), 0, 0, d_idx, d_out, iters);
  CK(hipDeviceSynchronize());
  CK(hipEventRecord(e0));
  hipLaunchKernelGGL(k<MODE>, dim3(grid), dim3(512), 0, 0, d_idx, d_out, iters);
  CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
  float ms; CK(hipEventElapsedTime(&ms, e0, e1));
  double ops = (double)grid * 512 * iters * 16;
  double per_cu_clk = ops / (ms * 1e-3) / 256 / 2.4e9;
  printf("%-28s %8.3f ms  %8.2f Gops/s  %.2f lane-ops/clk/CU\n", name, ms, ops / ms / 1e6, per_cu_clk);
}
int main() {
  int grid = 512, iters = 64;
  std::vector<unsigned> h(grid * 512);
  for (auto& v : h) v = rand();
  unsigned* d_idx; float* d_out;
  CK(hipMalloc(&d_idx, h.size() * 4)); CK(hipMalloc(&d_out, h.size() * 4));
  CK(hipMemcpy(d_idx, h.data(), h.size() * 4, hipMemcpyHostToDevice));
  run<0>("ds_add_f32 random", d_idx, d_out, grid, iters);
  run<1>("ds_add_u32 random", d_idx, d_out, grid, iters);
  run<2>("ds_add_u64 random", d_idx, d_out, grid, iters);
  run<3>("ds_write_b32 random", d_idx, d_out, grid, iters);
  run<4>("ds_read_b32 random", d_idx, d_out, grid, iters);
  run<5>("ds_add_f32 conflict-free", d_idx, d_out, grid, iters);
  run<6>("ds_add_f32 same address", d_idx, d_out, grid, iters);
  run<7>("ds_add_u64 banks l%32", d_idx, d_out, grid, iters);
  run<8>("ds_add_u64 l,l+8 collide", d_idx, d_out, grid, iters);
  run<9>("ds_add_u64 l,l+16 collide", d_idx, d_out, grid, iters);
  run<10>("ds_add_u64 2i,2i+1 collide", d_idx, d_out, grid, iters);
  return 0;
}
