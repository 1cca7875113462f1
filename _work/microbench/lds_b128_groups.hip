// micro-benchmark: which lanes of a ds_read_b128 are checked against each other for bank conflicts?
// 64 KiB table = 256 rows x 256 B (16 columns of 16 B).  Every lane reads (random row, column by pattern).
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <vector>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1);} } while (0)
typedef unsigned u4 __attribute__((ext_vector_type(4)));
template <int PAT>
__device__ __forceinline__ unsigned col_of(unsigned l, unsigned rnd) {
  switch (PAT) {
    case 0: return (rnd >> 8) & 15;
    case 1: return l & 15;
    case 2: return (l >> 2) & 15;
    case 3: return ((l & 3) << 2) | (l >> 4);
    case 4: return (l & 7) | ((l >> 5) << 3);
    case 5: return 0;
    case 6: return (l & 7) | (((l >> 4) & 1) << 3);
    case 7: return (l >> 1) & 15;
    case 8: return (l & 3) | (((l >> 4) & 3) << 2);
    default: return (l + (l >> 4)) & 15;
  }
}
template <int PAT>
__global__ __launch_bounds__(1024) void k(const unsigned* __restrict__ codes, float* out, int iters) {
  extern __shared__ __attribute__((aligned(16))) unsigned tab[];
  for (int x = threadIdx.x; x < 16384; x += 1024) tab[x] = x * 2654435761u;
  __syncthreads();
  unsigned cw[4];
  for (int j = 0; j < 4; ++j) cw[j] = codes[(blockIdx.x * 1024 + threadIdx.x) * 4 + j];
  const unsigned l = threadIdx.x & 63;
  unsigned acc[4] = {0, 0, 0, 0};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int m = 0; m < 16; ++m) {
      const unsigned rnd = cw[m / 4] >> (8 * (m % 4));
      const unsigned row = rnd & 0xffu;
      const unsigned col = col_of<PAT>(l, cw[(m + 1) & 3] >> (4 * (m & 3)));
      u4 v = *reinterpret_cast<const u4*>(tab + row * 64 + col * 4);
      for (int e = 0; e < 4; ++e) acc[e] ^= v[e];
    }
    for (int j = 0; j < 4; ++j) cw[j] = (cw[j] >> 1) | (cw[j] << 31);
  }
  out[blockIdx.x * 1024 + threadIdx.x] = __builtin_bit_cast(float, acc[0] ^ acc[1] ^ acc[2] ^ acc[3]);
}
template <int PAT> void run(const unsigned* d_codes, float* d_out, const char* what) {
  int grid = 256, iters = 256;
  CK(hipFuncSetAttribute(reinterpret_cast<const void*>(&k<PAT>), hipFuncAttributeMaxDynamicSharedMemorySize, 65536));
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  for (int rep = 0; rep < 2; ++rep) {
    CK(hipEventRecord(e0));
    hipLaunchKernelGGL((k<PAT>), dim3(grid), dim3(1024), 65536, 0, d_codes, d_out, iters);
    CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
  }
  float ms; CK(hipEventElapsedTime(&ms, e0, e1));
  double instr_per_cu = 16.0 * iters * 16;
  printf("pattern %d %-44s: %7.3f ms  %6.2f ns per wave-read per CU (%.1f clk @2.1GHz)\n", PAT, what, ms, ms * 1e6 / instr_per_cu, ms * 1e6 / instr_per_cu * 2.1);
  fflush(stdout);
}
int main() {
  std::vector<unsigned> h(256 * 1024 * 4);
  for (auto& v : h) v = rand() ^ (rand() << 16);
  unsigned* d_codes; float* d_out;
  CK(hipMalloc(&d_codes, h.size() * 4)); CK(hipMalloc(&d_out, h.size() * 4));
  CK(hipMemcpy(d_codes, h.data(), h.size() * 4, hipMemcpyHostToDevice));
  run<0>(d_codes, d_out, "random column");
  run<1>(d_codes, d_out, "col = l & 15");
  run<2>(d_codes, d_out, "col = (l >> 2) & 15");
  run<3>(d_codes, d_out, "col = (l & 3) * 4 + (l >> 4)");
  run<4>(d_codes, d_out, "col = (l & 7) + 8 * (l >> 5)");
  run<5>(d_codes, d_out, "col = 0");
  run<6>(d_codes, d_out, "col = (l & 7) + 8 * ((l >> 4) & 1)");
  run<7>(d_codes, d_out, "col = (l >> 1) & 15");
  run<8>(d_codes, d_out, "col = (l & 3) + 4 * ((l >> 4) & 3)");
  run<9>(d_codes, d_out, "col = (l + (l >> 4)) & 15");
  return 0;
}
