// Checks where global_load_lds_dwordx4 (gfx950: 16 bytes per lane straight from global memory into LDS, no
// VGPR destination) puts its data: LDS byte address = M0 + 16 * (lane of the wavefront).  Issued from inline
// asm so that the compiler inserts no wait of its own before unrelated LDS reads; the consumer waits with an
// explicit s_waitcnt vmcnt(0).  Build: hipcc --offload-arch=gfx950 -O3 -o /tmp/lds_direct_load lds_direct_load.hip
#include <hip/hip_runtime.h>

#include <cstdio>
#include <vector>

__device__ __forceinline__ void dma16(const void *gptr, unsigned lds_byte_addr_uniform)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(lds_byte_addr_uniform), "v"(gptr) : "memory");
}

__global__ __launch_bounds__(256) void k(const uint4 *__restrict__ src, uint4 *__restrict__ out)
{
    extern __shared__ __attribute__((aligned(16))) uint4 buf[];  // dynamic LDS starts at address 0 (no static LDS here)
    const unsigned tid = threadIdx.x;
    for (int x = 0; x < 4; ++x) buf[x * 256 + tid] = make_uint4(0xdeadu, 0, 0, 0);
    __syncthreads();
    // piece x of thread t goes to slot x * 256 + t: wave-uniform base (x * 256 + 64 * wave) * 16 in M0
    for (int x = 0; x < 4; ++x) {
        const unsigned base = __builtin_amdgcn_readfirstlane((x * 256u + (tid & ~63u)) * 16u);
        dma16(src + (size_t)tid * 4 + x, base);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    for (int x = 0; x < 4; ++x) out[x * 256 + tid] = buf[x * 256 + tid];
}

int main()
{
    const int n = 1024;
    std::vector<uint4> h(n), r(n);
    for (int i = 0; i < n; ++i) h[i] = make_uint4(i, i * 3 + 1, ~i, i ^ 0x5555);
    uint4 *d, *o;
    hipMalloc(&d, n * sizeof(uint4));
    hipMalloc(&o, n * sizeof(uint4));
    hipMemcpy(d, h.data(), n * sizeof(uint4), hipMemcpyHostToDevice);
    hipLaunchKernelGGL(k, dim3(1), dim3(256), n * sizeof(uint4), 0, d, o);
    if (hipDeviceSynchronize() != hipSuccess) { printf("launch failed\n"); return 1; }
    hipMemcpy(r.data(), o, n * sizeof(uint4), hipMemcpyDeviceToHost);
    int bad = 0;
    for (int x = 0; x < 4; ++x)
        for (int t = 0; t < 256; ++t) {
            const uint4 want = h[t * 4 + x], got = r[x * 256 + t];
            if (want.x != got.x || want.y != got.y || want.z != got.z || want.w != got.w) ++bad;
        }
    printf("global_load_lds_dwordx4 placement (M0 + 16 * lane): %s (%d mismatches)\n", bad ? "WRONG" : "confirmed", bad);
    return bad != 0;
}
