// micro-benchmark: do vector-ALU instructions issue while a matrix instruction of the same / another wave executes?
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1);} } while (0)
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx4_t __attribute__((ext_vector_type(4)));
typedef unsigned uint4_t __attribute__((ext_vector_type(4)));
// MF: 0 none, 1 bf16 16x16x32 (dependent chain), 2 f32 16x16x4 (dependent chain), 3 bf16 two independent chains
template <int MF, int KV>
__global__ __launch_bounds__(1024) void k(float* out, int iters, float seed) {
  uint4_t au = {0x3f803f80u, 0x3f803f80u, 0x3f803f80u, threadIdx.x};
  bf16x8_t a = __builtin_bit_cast(bf16x8_t, au), b = a;
  floatx4_t acc = {0.f, 0.f, 0.f, 0.f}, acc2 = acc;
  float f[8];
  for (int i = 0; i < 8; ++i) f[i] = seed + i + threadIdx.x;
  const float m = seed * 0.5f, c = seed;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int rep = 0; rep < 8; ++rep) {
      if (MF == 1) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc, 0, 0, 0);
      if (MF == 2) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(m, c, acc, 0, 0, 0);
      if (MF == 3) { if (rep & 1) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc, 0, 0, 0); else acc2 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc2, 0, 0, 0); }
#pragma unroll
      for (int j = 0; j < KV; ++j) f[(rep * KV + j) & 7] = __builtin_fmaf(f[(rep * KV + j) & 7], m, c);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  float s = acc[0] + acc[1] + acc[2] + acc[3] + acc2[0];
  for (int i = 0; i < 8; ++i) s += f[i];
  out[blockIdx.x * 1024 + threadIdx.x] = s;
}
template <int MF, int KV> void run(float* d_out, int threads) {
  int grid = 256, iters = 2000;
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  for (int rep = 0; rep < 2; ++rep) {
    CK(hipEventRecord(e0));
    hipLaunchKernelGGL((k<MF, KV>), dim3(grid), dim3(threads), 0, 0, d_out, iters, 1.0f);
    CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
  }
  float ms; CK(hipEventElapsedTime(&ms, e0, e1));
  double ns_per_rep_per_wave = ms * 1e6 / (iters * 8.0);
  printf("mfma kind %d + %d fma per mfma, %4d threads/CU: %7.3f ms  %6.1f ns per (mfma + fmas) group per wave-slot\n", MF, KV, threads, ms, ns_per_rep_per_wave);
  fflush(stdout);
}
int main() {
  float* d_out; CK(hipMalloc(&d_out, 256 * 1024 * 4));
  for (int threads : {256, 1024}) {
    run<0, 4>(d_out, threads); run<0, 8>(d_out, threads);
    run<1, 0>(d_out, threads); run<1, 2>(d_out, threads); run<1, 4>(d_out, threads); run<1, 8>(d_out, threads);
    run<2, 0>(d_out, threads); run<2, 4>(d_out, threads); run<2, 8>(d_out, threads);
    run<3, 0>(d_out, threads); run<3, 4>(d_out, threads);
  }
  return 0;
}
