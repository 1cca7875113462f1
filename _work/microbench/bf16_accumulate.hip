// micro-benchmark: issue rate of candidate "add a bf16 half into fp32" instruction sequences
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1);} } while (0)
typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
typedef _Float16 h2 __attribute__((ext_vector_type(2)));
template <int MODE>
__global__ __launch_bounds__(256) void k(const unsigned* __restrict__ in, float* out, int iters) {
  unsigned v[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) v[e] = in[threadIdx.x + 256 * e];
  unsigned sel_lo = 0x3f80u, sel_hi = 0x3f800000u; asm volatile("" : "+s"(sel_lo)); asm volatile("" : "+s"(sel_hi));
  unsigned hsel_lo = 0x3c00u, hsel_hi = 0x3c000000u; asm volatile("" : "+s"(hsel_lo)); asm volatile("" : "+s"(hsel_hi));
  float a[16];
#pragma unroll
  for (int e = 0; e < 16; ++e) a[e] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      if (MODE == 0) { a[2*e] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf2, v[e]), __builtin_bit_cast(bf2, sel_lo), a[2*e], false);
                       a[2*e+1] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf2, v[e]), __builtin_bit_cast(bf2, sel_hi), a[2*e+1], false); }
      else if (MODE == 1) { a[2*e] += __builtin_bit_cast(float, v[e] << 16); a[2*e+1] += __builtin_bit_cast(float, v[e] & 0xffff0000u); }
      else if (MODE == 2) { a[2*e] += __builtin_bit_cast(float, v[e]); a[2*e+1] += __builtin_bit_cast(float, v[e] ^ 0x1234u); }   // 1 add + 1 xor + 1 add
      else if (MODE == 3) { a[2*e] = __builtin_amdgcn_fdot2(__builtin_bit_cast(h2, v[e]), __builtin_bit_cast(h2, hsel_lo), a[2*e], false);
                            a[2*e+1] = __builtin_amdgcn_fdot2(__builtin_bit_cast(h2, v[e]), __builtin_bit_cast(h2, hsel_hi), a[2*e+1], false); }
      else if (MODE == 4) { h2 h = __builtin_bit_cast(h2, v[e]); a[2*e] += (float)h.x; a[2*e+1] += (float)h.y; }  // cvt (+sdwa) + add
      else if (MODE == 5) { a[2*e] = fmaf(__builtin_bit_cast(float, v[e]), 1.0001f, a[2*e]); a[2*e+1] = fmaf(__builtin_bit_cast(float, v[e]), 0.999f, a[2*e+1]); } // 2 fma
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) asm volatile("" : "+v"(v[e]));
  }
  float s = 0.f;
#pragma unroll
  for (int e = 0; e < 16; ++e) s += a[e];
  out[blockIdx.x * 256 + threadIdx.x] = s;
}
template <int MODE> void run(const char* name, const unsigned* d_in, float* d_out) {
  int grid = 4096, iters = 2000;
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  for (int rep = 0; rep < 2; ++rep) {
    CK(hipEventRecord(e0));
    hipLaunchKernelGGL(k<MODE>, dim3(grid), dim3(256), 0, 0, d_in, d_out, iters);
    CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
  }
  float ms; CK(hipEventElapsedTime(&ms, e0, e1));
  double elems = (double)grid * 4 /*waves*/ * iters * 16;  // wave-level element-adds (one per accumulate)
  printf("%-34s %7.3f ms   %6.2f SIMD-clk per wave-level element add (@2.4GHz, 1024 SIMDs)\n", name, ms, ms * 1e-3 * 2.4e9 * 1024 / elems);
}
int main() {
  unsigned* d_in; float* d_out;
  CK(hipMalloc(&d_in, 256 * 8 * 4)); CK(hipMalloc(&d_out, 4096 * 256 * 4));
  CK(hipMemset(d_in, 0, 256 * 8 * 4));
  run<0>("v_dot2c_f32_bf16 (1 op/elem)", d_in, d_out);
  run<1>("shift|and + v_add_f32 (2 op/elem)", d_in, d_out);
  run<2>("v_add_f32 (+0.5 xor) (1.5 op/elem)", d_in, d_out);
  run<3>("v_dot2c_f32_f16 (1 op/elem)", d_in, d_out);
  run<4>("cvt_f32_f16 + add (2 op/elem)", d_in, d_out);
  run<5>("v_fma_f32 (1 op/elem)", d_in, d_out);
  return 0;
}
