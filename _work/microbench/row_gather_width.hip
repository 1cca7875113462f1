// micro-benchmark: 256-byte row gathers with 1, 2 or 4 rows per wave-level load instruction
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <vector>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1);} } while (0)
typedef unsigned u4 __attribute__((ext_vector_type(4)));
typedef unsigned u2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
// RPI rows per instruction: lanes are split in RPI groups; group r handles token (t*RPI + r).
template <int WAVES, int RPI>
__global__ __launch_bounds__(WAVES * 64) void k(const unsigned* __restrict__ table, const unsigned char* __restrict__ codes, float* out, int ntok, unsigned nrows_per_m) {
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  constexpr int LPR = 64 / RPI;        // lanes per row
  constexpr int BPL = 256 / LPR;       // bytes per lane
  const int grp = lane / LPR, sub = lane % LPR;
  __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void*)table, 0, (int)(16u * nrows_per_m * 256u), 0x00020000);
  const unsigned char* cp = codes + ((size_t)(blockIdx.x * WAVES + wave) * ntok) * 16;
  unsigned sel_lo = 0x3f80u, sel_hi = 0x3f800000u; asm volatile("" : "+s"(sel_lo)); asm volatile("" : "+s"(sel_hi));
  float acc[BPL / 2];
#pragma unroll
  for (int e = 0; e < BPL / 2; ++e) acc[e] = 0.f;
  for (int t = 0; t < ntok; t += RPI) {
    const u4 c4 = *reinterpret_cast<const u4*>(cp + (size_t)(t + grp) * 16);   // this lane's token codes
#pragma unroll
    for (int m = 0; m < 16; ++m) {
      unsigned voff;
      if (BPL == 16 && nrows_per_m == 256) voff = __builtin_amdgcn_perm(c4[m / 4], sub * BPL, 0x0c0c0000u | ((4u + (m % 4)) << 8));
      else { unsigned c = (c4[m / 4] >> (8 * (m % 4))) & 0xffu; if (nrows_per_m < 256) c &= (nrows_per_m - 1); voff = c * 256u + sub * BPL; }
      unsigned soff = m * nrows_per_m * 256u;
      if (BPL == 4) { unsigned v = __builtin_amdgcn_raw_buffer_load_b32(rs, voff, soff, 0); acc[0] += __builtin_bit_cast(float, v << 16); acc[1] += __builtin_bit_cast(float, v & 0xffff0000u); }
      else if (BPL == 8) { u2 v = __builtin_amdgcn_raw_buffer_load_b64(rs, voff, soff, 0);
#pragma unroll
        for (int e = 0; e < 2; ++e) { acc[2*e] += __builtin_bit_cast(float, v[e] << 16); acc[2*e+1] += __builtin_bit_cast(float, v[e] & 0xffff0000u);} }
      else { u4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, voff, soff, 0);
#pragma unroll
        for (int e = 0; e < 4; ++e) { const unsigned ve = v[e]; acc[2*e] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf2, ve), __builtin_bit_cast(bf2, sel_lo), acc[2*e], false); acc[2*e+1] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf2, ve), __builtin_bit_cast(bf2, sel_hi), acc[2*e+1], false);} }
    }
  }
  float s = 0.f;
#pragma unroll
  for (int e = 0; e < BPL / 2; ++e) s += acc[e];
  out[(size_t)blockIdx.x * WAVES * 64 + threadIdx.x] = s;
}
template <int RPI> void run(const unsigned* d_table, const unsigned char* d_codes, float* d_out, int grid, int ntok, unsigned nrows, size_t ncodes) {
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  for (int rep = 0; rep < 2; ++rep) {
    CK(hipEventRecord(e0));
    hipLaunchKernelGGL((k<4, RPI>), dim3(grid), dim3(256), 0, 0, d_table, d_codes, d_out, ntok, nrows);
    CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
  }
  float ms; CK(hipEventElapsedTime(&ms, e0, e1));
  double bytes = (double)ncodes * 256;
  printf("rows/instr %d  rows/codebook %3u (table %6.0f KiB): %7.3f ms  %6.2f TB/s  %5.1f B/clk/CU@2.4  %5.2f clk/CU per wave-load\n", RPI, nrows, 16 * nrows * 0.25, ms, bytes / ms / 1e9,
         bytes / (ms * 1e-3) / 256 / 2.4e9, (ms * 1e-3) * 2.4e9 * 256 / ((double)ncodes / RPI));
}
int main() {
  int grid = 2048, ntok = 128;
  size_t ncodes = (size_t)grid * 4 * ntok * 16;
  std::vector<unsigned char> h(ncodes);
  for (auto& v : h) v = rand() & 255;
  unsigned char* d_codes; unsigned* d_table; float* d_out;
  CK(hipMalloc(&d_codes, ncodes)); CK(hipMalloc(&d_table, (size_t)16 * 256 * 256)); CK(hipMalloc(&d_out, (size_t)grid * 256 * 4));
  CK(hipMemset(d_table, 0, (size_t)16 * 256 * 256));
  CK(hipMemcpy(d_codes, h.data(), ncodes, hipMemcpyHostToDevice));
  for (unsigned nrows : {4u, 256u}) {
    run<1>(d_table, d_codes, d_out, grid, ntok, nrows, ncodes);
    run<2>(d_table, d_codes, d_out, grid, ntok, nrows, ncodes);
    run<4>(d_table, d_codes, d_out, grid, ntok, nrows, ncodes);
  }
  return 0;
}
