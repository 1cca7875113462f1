// micro-benchmark: per-lane random row reads from a 128 KiB LDS table (ds_read_b128 / b64)
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <vector>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1);} } while (0)
typedef unsigned u4 __attribute__((ext_vector_type(4)));
typedef unsigned u2 __attribute__((ext_vector_type(2)));
// ROWB: bytes per row (16 or 32); table = 16 codebooks x 256 rows x ROWB... scaled to fill 128 KiB:  nrows = 131072 / ROWB
template <int ROWB, int WIDTH, int PLANES>
__global__ __launch_bounds__(1024) void k(const unsigned* __restrict__ codes, float* out, int iters) {
  extern __shared__ __attribute__((aligned(16))) unsigned tab[];
  for (int x = threadIdx.x; x < 32768; x += 1024) tab[x] = x * 2654435761u;
  __syncthreads();
  constexpr unsigned NROWS = 131072 / ROWB;
  // 16 random bytes per lane (4 dwords); row = m * (NROWS/16) + byte (when NROWS/16 < 256 the byte is masked)
  unsigned cw[4];
  for (int j = 0; j < 4; ++j) cw[j] = codes[(blockIdx.x * 1024 + threadIdx.x) * 4 + j];
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  constexpr unsigned RPM = NROWS / 16;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int m = 0; m < 16; ++m) {
      unsigned row = m * RPM + (((cw[m / 4] >> (8 * (m % 4))) & 0xffu) & (RPM - 1));
      if (PLANES) {   // ROWB/16 planes of 16-byte pieces: piece h of a row at plane h
#pragma unroll
        for (int h = 0; h < ROWB / 16; ++h) { u4 v = *reinterpret_cast<const u4*>(tab + h * (NROWS * 4) + row * 4);
          for (int e = 0; e < 4; ++e) { unsigned ve = v[e]; acc[e] += __builtin_bit_cast(float, ve); } }
      } else if (WIDTH == 16) {
#pragma unroll
        for (int h = 0; h < ROWB / 16; ++h) { u4 v = *reinterpret_cast<const u4*>(tab + row * (ROWB / 4) + 4 * h);
          for (int e = 0; e < 4; ++e) { unsigned ve = v[e]; acc[e] += __builtin_bit_cast(float, ve); } }
      } else {
#pragma unroll
        for (int h = 0; h < ROWB / 8; ++h) { u2 v = *reinterpret_cast<const u2*>(tab + row * (ROWB / 4) + 2 * h);
          for (int e = 0; e < 2; ++e) { unsigned ve = v[e]; acc[e] += __builtin_bit_cast(float, ve); } }
      }
    }
    for (int j = 0; j < 4; ++j) cw[j] = (cw[j] >> 1) | (cw[j] << 31);
  }
  out[blockIdx.x * 1024 + threadIdx.x] = acc[0] + acc[1] + acc[2] + acc[3];
}
template <int ROWB, int WIDTH, int PLANES> void run(const unsigned* d_codes, float* d_out) {
  int grid = 256, iters = 256;
  CK(hipFuncSetAttribute(reinterpret_cast<const void*>(&k<ROWB, WIDTH, PLANES>), hipFuncAttributeMaxDynamicSharedMemorySize, 131072));
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  for (int rep = 0; rep < 2; ++rep) {
    CK(hipEventRecord(e0));
    hipLaunchKernelGGL((k<ROWB, WIDTH, PLANES>), dim3(grid), dim3(1024), 131072, 0, d_codes, d_out, iters);
    CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
  }
  float ms; CK(hipEventElapsedTime(&ms, e0, e1));
  double bytes = (double)grid * 1024 * iters * 16 * ROWB;
  printf("row %2d B, ds_read_b%-3d planes=%d : %7.3f ms  %6.2f TB/s  %6.1f B/clk/CU @2.4GHz\n", ROWB, WIDTH * 8, PLANES, ms, bytes / ms / 1e9, bytes / (ms * 1e-3) / 256 / 2.4e9);
}
int main() {
  std::vector<unsigned> h(256 * 1024 * 4);
  for (auto& v : h) v = rand();
  unsigned* d_codes; float* d_out;
  CK(hipMalloc(&d_codes, h.size() * 4)); CK(hipMalloc(&d_out, h.size() * 4));
  CK(hipMemcpy(d_codes, h.data(), h.size() * 4, hipMemcpyHostToDevice));
  run<16, 16, 0>(d_codes, d_out);
  run<32, 16, 0>(d_codes, d_out);
  run<32, 16, 1>(d_codes, d_out);
  run<64, 16, 1>(d_codes, d_out);
  run<16, 8, 0>(d_codes, d_out);
  return 0;
}
