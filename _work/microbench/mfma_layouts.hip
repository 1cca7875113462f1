// probe: operand / result lane layouts of v_mfma_f32_16x16x32_bf16 and v_mfma_f32_4x4x1_16b_f32, the lane
// exchange done by v_permlane16_swap / v_permlane32_swap, and the 16x16x32 issue rate on gfx950
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <vector>
#include <cstring>
#include <cmath>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1);} } while (0)
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef unsigned u4 __attribute__((ext_vector_type(4)));
typedef float floatx4_t __attribute__((ext_vector_type(4)));
// A[i][k] = value table a(i,k); B[k][n]; D = A*B.  Lane l supplies A[l%16][8*(l/16)..+7], B[8*(l/16)..+7][l%16] (assumed).
__global__ void layout(const unsigned short* Abits, const unsigned short* Bbits, float* D) {
  int l = threadIdx.x;
  unsigned short a[8], b[8];
  for (int e = 0; e < 8; ++e) { a[e] = Abits[(l % 16) * 32 + 8 * (l / 16) + e]; b[e] = Bbits[(8 * (l / 16) + e) * 16 + (l % 16)]; }
  u4 au; for (int e = 0; e < 4; ++e) au[e] = (unsigned)a[2*e] | ((unsigned)a[2*e+1] << 16);
  u4 bu; for (int e = 0; e < 4; ++e) bu[e] = (unsigned)b[2*e] | ((unsigned)b[2*e+1] << 16);
  floatx4 c = {0, 0, 0, 0};
  c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, au), __builtin_bit_cast(bf16x8, bu), c, 0, 0, 0);
  for (int r = 0; r < 4; ++r) D[l * 4 + r] = c[r];
}
__global__ __launch_bounds__(256) void rate(float* out, int iters) {
  u4 au = {threadIdx.x, 1, 2, 3}, bu = {0x3f803f80u, 0, 0, 0};
  floatx4 c0 = {0, 0, 0, 0}, c1 = c0, c2 = c0, c3 = c0;
  for (int it = 0; it < iters; ++it) {
    c0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, au), __builtin_bit_cast(bf16x8, bu), c0, 0, 0, 0);
    c1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, au), __builtin_bit_cast(bf16x8, bu), c1, 0, 0, 0);
    c2 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, au), __builtin_bit_cast(bf16x8, bu), c2, 0, 0, 0);
    c3 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, au), __builtin_bit_cast(bf16x8, bu), c3, 0, 0, 0);
  }
  out[blockIdx.x * 256 + threadIdx.x] = c0[0] + c1[1] + c2[2] + c3[3];
}
__global__ void small_and_swaps(float* out, unsigned* sw) {
  const int l = threadIdx.x;
  const float a = 1.0f + l, b = 100.0f + 3.0f * l;
  floatx4_t c = {0.f, 0.f, 0.f, 0.f};
  c = __builtin_amdgcn_mfma_f32_4x4x1f32(a, b, c, 0, 0, 0);
  for (int r = 0; r < 4; ++r) out[l * 4 + r] = c[r];
  unsigned x = 1000u + l, y = 2000u + l;
  auto r16 = __builtin_amdgcn_permlane16_swap(x, y, false, false);
  auto r32 = __builtin_amdgcn_permlane32_swap(x, y, false, false);
  sw[l * 4 + 0] = r16[0]; sw[l * 4 + 1] = r16[1]; sw[l * 4 + 2] = r32[0]; sw[l * 4 + 3] = r32[1];
}
static unsigned short f2bf(float f) { unsigned u; std::memcpy(&u, &f, 4); return (unsigned short)(u >> 16); }
int main() {
  std::vector<unsigned short> A(16 * 32), B(32 * 16);
  std::vector<float> Af(16 * 32), Bf(32 * 16);
  for (int i = 0; i < 16; ++i) for (int k = 0; k < 32; ++k) { Af[i * 32 + k] = (float)((i * 7 + k * 3) % 13 - 6); A[i * 32 + k] = f2bf(Af[i * 32 + k]); }
  for (int k = 0; k < 32; ++k) for (int n = 0; n < 16; ++n) { Bf[k * 16 + n] = (float)((k * 5 + n * 11) % 7 - 3); B[k * 16 + n] = f2bf(Bf[k * 16 + n]); }
  unsigned short *dA, *dB; float* dD;
  CK(hipMalloc(&dA, A.size() * 2)); CK(hipMalloc(&dB, B.size() * 2)); CK(hipMalloc(&dD, 256 * 4));
  CK(hipMemcpy(dA, A.data(), A.size() * 2, hipMemcpyHostToDevice)); CK(hipMemcpy(dB, B.data(), B.size() * 2, hipMemcpyHostToDevice));
  hipLaunchKernelGGL(layout, dim3(1), dim3(64), 0, 0, dA, dB, dD);
  std::vector<float> D(256); CK(hipMemcpy(D.data(), dD, 1024, hipMemcpyDeviceToHost));
  int bad = 0;
  for (int l = 0; l < 64; ++l) for (int r = 0; r < 4; ++r) {
    int i = 4 * (l / 16) + r, n = l % 16; float ref = 0; for (int k = 0; k < 32; ++k) ref += Af[i * 32 + k] * Bf[k * 16 + n];
    if (ref != D[l * 4 + r]) { if (bad < 5) printf("mismatch lane %d r %d: got %g want %g\n", l, r, D[l * 4 + r], ref); ++bad; }
  }
  printf("layout check (A[l%%16][8(l/16)+e], B[8(l/16)+e][l%%16], D[4(l/16)+r][l%%16]): %s (%d mismatches)\n", bad ? "WRONG" : "OK", bad);
  float* dO; CK(hipMalloc(&dO, 4096 * 256 * 4));
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  int iters = 4000, grid = 2048;
  for (int rep = 0; rep < 2; ++rep) { CK(hipEventRecord(e0)); hipLaunchKernelGGL(rate, dim3(grid), dim3(256), 0, 0, dO, iters); CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1)); }
  float ms; CK(hipEventElapsedTime(&ms, e0, e1));
  double n = (double)grid * 4 * iters * 4;
  printf("mfma_f32_16x16x32_bf16: %.3f ms, %.2f SIMD-clk per MFMA @2.4GHz, %.1f TFLOP/s\n", ms, ms * 1e-3 * 2.4e9 * 1024 / n, n * 16384 / ms / 1e9);
  {
  float* d; unsigned* s; CK(hipMalloc(&d, 64 * 4 * 4)); CK(hipMalloc(&s, 64 * 4 * 4));
  hipLaunchKernelGGL(small_and_swaps, dim3(1), dim3(64), 0, 0, d, s);
  float hsm[256]; unsigned hs[256];
  CK(hipMemcpy(hsm, d, sizeof hsm, hipMemcpyDeviceToHost)); CK(hipMemcpy(hs, s, sizeof hs, hipMemcpyDeviceToHost));
  // hypothesis: block = l / 4; D_b[i][j] = A_b[i] * B_b[j], A_b[i] from lane 4b + i, B_b[j] from lane 4b + j; lane 4b + j holds D_b[r][j] in register r
  int bad = 0;
  for (int l = 0; l < 64; ++l) for (int r = 0; r < 4; ++r) {
    int bk = l / 4, j = l % 4;
    float want = (1.0f + 4 * bk + r) * (100.0f + 3.0f * (4 * bk + j));
    if (fabsf(hsm[l * 4 + r] - want) > 1e-3f * fabsf(want)) { if (bad < 8) printf("mismatch lane %d reg %d: got %f want %f\n", l, r, hsm[l * 4 + r], want); ++bad; }
  }
  printf("4x4x1 layout hypothesis: %s (%d mismatches)\n", bad ? "WRONG" : "confirmed", bad);
  // permlane16_swap(vdst = x, src0 = y): hypothesis: odd rows of x <-> even rows of y
  bad = 0;
  for (int l = 0; l < 64; ++l) {
    int row = l / 16;
    unsigned wx = (row & 1) ? 2000u + (l - 16) : 1000u + l;        // odd rows of x receive the even row below from y
    unsigned wy = (row & 1) ? 2000u + l : 1000u + (l + 16);        // even rows of y receive the odd row above from x
    if (hs[l * 4 + 0] != wx || hs[l * 4 + 1] != wy) { if (bad < 8) printf("swap16 lane %d: got %u %u want %u %u\n", l, hs[l * 4], hs[l * 4 + 1], wx, wy); ++bad; }
  }
  printf("permlane16_swap hypothesis: %s\n", bad ? "WRONG" : "confirmed");
  bad = 0;
  for (int l = 0; l < 64; ++l) {
    unsigned wx = l >= 32 ? 2000u + (l - 32) : 1000u + l;
    unsigned wy = l >= 32 ? 2000u + l : 1000u + (l + 32);
    if (hs[l * 4 + 2] != wx || hs[l * 4 + 3] != wy) { if (bad < 8) printf("swap32 lane %d: got %u %u want %u %u\n", l, hs[l * 4 + 2], hs[l * 4 + 3], wx, wy); ++bad; }
  }
  printf("permlane32_swap hypothesis: %s\n", bad ? "WRONG" : "confirmed");
  }
  return 0;
}
