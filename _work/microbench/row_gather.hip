// micro-benchmark: x4 (16 B per lane) row gathers, 4 rows per wave instruction, different consumers
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <vector>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1);} } while (0)
typedef unsigned u4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
// MODE 0: xor-reduce (1 int op per dword)  1: dot2 x2 per dword  2: shift/and/add  3: fp32 add of raw bits (1 op/dword)
// ADDR 0: perm  1: bfe+mad   UNI 1: all 64 lanes read one contiguous KiB (row index uniform)
template <int MODE, int ADDR, int UNI>
__global__ __launch_bounds__(256) void k(const unsigned* __restrict__ table, const unsigned char* __restrict__ codes, float* out, int ntok) {
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  const int grp = UNI ? 0 : lane / 16;
  const unsigned sub16 = UNI ? lane * 16 : (lane % 16) * 16;
  __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void*)table, 0, (int)(16u * 256u * 256u), 0x00020000);
  const unsigned char* cp = codes + ((size_t)(blockIdx.x * 4 + wave) * ntok) * 16;
  unsigned sel_lo = 0x3f80u, sel_hi = 0x3f800000u; asm volatile("" : "+s"(sel_lo)); asm volatile("" : "+s"(sel_hi));
  float acc[8]; unsigned x = 0;
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = 0.f;
  for (int t = 0; t < ntok; t += 4) {
    const u4 c4 = *reinterpret_cast<const u4*>(cp + (size_t)(t + grp) * 16);
#pragma unroll
    for (int m = 0; m < 16; ++m) {
      unsigned voff;
      if (ADDR == 0) voff = __builtin_amdgcn_perm(c4[m / 4], sub16, 0x0c0c0000u | ((4u + (m % 4)) << 8));
      else { unsigned c = (c4[m / 4] >> (8 * (m % 4))) & 0xffu; voff = c * 256u + sub16; }
      if (UNI) voff &= 0xfc00u | 0x3f0u;   // 1 KiB aligned block + lane*16
      u4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, voff, m * 65536u, 0);
#pragma unroll
      for (int e = 0; e < 4; ++e) { const unsigned ve = v[e];
        if (MODE == 0) x ^= v[e];
        else if (MODE == 1) { acc[2*e] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf2, ve), __builtin_bit_cast(bf2, sel_lo), acc[2*e], false);
                              acc[2*e+1] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf2, ve), __builtin_bit_cast(bf2, sel_hi), acc[2*e+1], false); }
        else if (MODE == 2) { acc[2*e] += __builtin_bit_cast(float, v[e] << 16); acc[2*e+1] += __builtin_bit_cast(float, v[e] & 0xffff0000u); }
        else acc[e] += __builtin_bit_cast(float, ve);
      }
    }
  }
  float s = __builtin_bit_cast(float, x);
#pragma unroll
  for (int e = 0; e < 8; ++e) s += acc[e];
  out[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}
template <int MODE, int ADDR, int UNI> void run(const char* name, const unsigned* d_table, const unsigned char* d_codes, float* d_out, int grid, int ntok, size_t ncodes) {
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  for (int rep = 0; rep < 2; ++rep) {
    CK(hipEventRecord(e0));
    hipLaunchKernelGGL((k<MODE, ADDR, UNI>), dim3(grid), dim3(256), 0, 0, d_table, d_codes, d_out, ntok);
    CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
  }
  float ms; CK(hipEventElapsedTime(&ms, e0, e1));
  double bytes = (double)ncodes * 256;
  printf("%-40s %7.3f ms  %6.2f TB/s  %5.1f B/clk/CU@2.4  %5.2f clk/CU per x4 load\n", name, ms, bytes / ms / 1e9, bytes / (ms * 1e-3) / 256 / 2.4e9, (ms * 1e-3) * 2.4e9 * 256 / ((double)ncodes / 4));
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
  run<0, 0, 0>("xor consumer, perm addr, 4 rows", d_table, d_codes, d_out, grid, ntok, ncodes);
  run<0, 1, 0>("xor consumer, bfe addr, 4 rows", d_table, d_codes, d_out, grid, ntok, ncodes);
  run<1, 0, 0>("dot2 consumer, perm addr, 4 rows", d_table, d_codes, d_out, grid, ntok, ncodes);
  run<2, 0, 0>("shift/and/add consumer, perm, 4 rows", d_table, d_codes, d_out, grid, ntok, ncodes);
  run<2, 1, 0>("shift/and/add consumer, bfe, 4 rows", d_table, d_codes, d_out, grid, ntok, ncodes);
  run<3, 0, 0>("f32 add consumer, perm, 4 rows", d_table, d_codes, d_out, grid, ntok, ncodes);
  run<0, 0, 1>("xor consumer, 1 KiB contiguous", d_table, d_codes, d_out, grid, ntok, ncodes);
  run<1, 0, 1>("dot2 consumer, 1 KiB contiguous", d_table, d_codes, d_out, grid, ntok, ncodes);
  return 0;
}
