// Lane layouts of v_smfmac_f32_16x16x64_bf16 (gfx950: structured-sparse first operand, two of every four
// consecutive k kept).  One first-operand entry is set to 1.0 at a time -- lane LA, stored slot s (0..7), position p
// (0..3) within its group of four -- and the second operand carries one bit of the code 16 * lane + j of the element
// (lane, j) that supplies it, ten runs for ten bits, so every non-zero output names the element it came from.
// Hypothesis checked:  first operand: lane l holds row l % 16, k = 16 (l / 16) + 4 (s / 2) + p for its slot s;
// second: lane l, element j: k = 16 (l / 16) + j, column l % 16;  result: lane l, register r: row 4 (l / 16) + r,
// column l % 16;  index register: bits 2 s .. 2 s + 1 = p of slot s (ABID 0).
// Build: hipcc --offload-arch=gfx950 -O3 -o /tmp/smfmac_layouts smfmac_layouts.hip
#include <hip/hip_runtime.h>

#include <cstdio>
#include <vector>

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x16_t __attribute__((ext_vector_type(16)));
typedef float floatx4_t __attribute__((ext_vector_type(4)));
typedef unsigned short u16x8_t __attribute__((ext_vector_type(8)));
typedef unsigned short u16x16_t __attribute__((ext_vector_type(16)));

// out[(cfg * 64 + lane) * 4 + r] = code of the source element, or -1 if that output is zero
__global__ __launch_bounds__(64) void k(int *__restrict__ out, int partner_mode)
{
    const int lane = threadIdx.x;
    for (int cfg = blockIdx.x; cfg < 64 * 8 * 4; cfg += gridDim.x) {
        const int LA = cfg / 32, s = (cfg / 4) % 8, p = cfg % 4;
        u16x8_t a = {0, 0, 0, 0, 0, 0, 0, 0};
        unsigned idx = 0;
        for (int t = 0; t < 8; ++t) {
            unsigned pos = (t & 1) ? 1u : 0u;  // default positions (0, 1) of every pair
            if (t == s) pos = (unsigned)p;
            else if (t == (s ^ 1)) {
                // the tested slot's partner holds 0.0 at another position
                if (partner_mode == 0) pos = (s & 1) ? (p > 0 ? (unsigned)p - 1u : 1u) : (p < 3 ? (unsigned)p + 1u : 2u);
                else pos = (p == 0) ? 1u : 0u;
            }
            idx |= pos << (2 * t);
        }
        idx |= idx << 16;
        if (lane == LA) a[s] = 0x3f80;  // 1.0
        int code[4] = {0, 0, 0, 0};
        bool any[4] = {false, false, false, false};
        for (int bit = 0; bit < 11; ++bit) {  // bit 10: all ones, marks "this output received something"
            u16x16_t b;
            for (int j = 0; j < 16; ++j) b[j] = (bit == 10 || (((lane * 16 + j) >> bit) & 1)) ? 0x3f80 : 0;
            floatx4_t c = {0.f, 0.f, 0.f, 0.f};
            c = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x16_t, b), c, (int)idx, 0, 0);
            for (int r = 0; r < 4; ++r) {
                if (bit == 10) any[r] = c[r] != 0.f;
                else if (c[r] != 0.f) code[r] |= 1 << bit;
            }
        }
        for (int r = 0; r < 4; ++r) out[(cfg * 64 + lane) * 4 + r] = any[r] ? code[r] : -1;
    }
}

int main()
{
    const int ncfg = 64 * 8 * 4;
    int *d;
    if (hipMalloc(&d, (size_t)ncfg * 256 * sizeof(int)) != hipSuccess) return 1;
    std::vector<int> h((size_t)ncfg * 256);
    for (int mode = 0; mode < 2; ++mode) {
        hipLaunchKernelGGL(k, dim3(256), dim3(64), 0, 0, d, mode);
        if (hipDeviceSynchronize() != hipSuccess) { printf("launch failed\n"); return 1; }
        if (hipMemcpy(h.data(), d, h.size() * sizeof(int), hipMemcpyDeviceToHost) != hipSuccess) return 1;
        if (mode == 0) {
            // the observed map, from column 0: first-operand (lane block, slot, position) -> second-operand (lane block, element)
            for (int kq = 0; kq < 4; ++kq)
                for (int s2 = 0; s2 < 8; ++s2) {
                    printf("  A lane block %d slot %d:", kq, s2);
                    for (int p2 = 0; p2 < 4; ++p2) {
                        const int cfg = (16 * kq) * 32 + s2 * 4 + p2;
                        const int got = h[((size_t)cfg * 64 + 0) * 4 + 0];  // D lane 0 reg 0 = row 0, column 0
                        printf("  pos %d -> B lane block %d elem %2d;", p2, got >= 0 ? (got / 16) / 16 : -1, got >= 0 ? got % 16 : -1);
                    }
                    printf("\n");
                }
        }
        long bad = 0, shown = 0;
        for (int cfg = 0; cfg < ncfg; ++cfg) {
            const int LA = cfg / 32, s = (cfg / 4) % 8, p = cfg % 4;
            const int row = LA % 16, kq = LA / 16, j = 4 * (s / 2) + p;
            for (int l = 0; l < 64; ++l)
                for (int r = 0; r < 4; ++r) {
                    const int got = h[((size_t)cfg * 64 + l) * 4 + r];
                    const int want = (4 * (l / 16) + r == row) ? ((l % 16) + 16 * kq) * 16 + j : -1;
                    if (got != want) {
                        ++bad;
                        if (shown < 0) {
                            printf("  mode %d: A lane %d slot %d pos %d -> D lane %d reg %d: source %d (lane %d, j %d), expected %d\n", mode, LA, s, p,
                                   l, r, got, got >= 0 ? got / 16 : -1, got >= 0 ? got % 16 : -1, want);
                            ++shown;
                        }
                    }
                }
        }
        printf("smfmac_f32_16x16x64_bf16 layout hypothesis, partner positions mode %d: %s (%ld mismatches of %d)\n", mode,
               bad ? "NOT confirmed" : "confirmed", bad, ncfg * 256);
    }
    return 0;
}
