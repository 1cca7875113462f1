/*
 * Host check of the row order of the binary-code value stage (csrc/commvq_vbits.hpp): vbits_code_bit must be a
 * permutation of every run of 128 rows, and must send the row that lane n of a 16-lane row stores in pass p of the
 * wavefront's W-th run (128 W + 16 p + n) to the code bit that this lane multiplies in that pass: record dword
 * 4 W + n / 4, byte n % 4, bit p.
 */
#include <cstdio>
#include <vector>

#include "commvq_vbits.hpp"

int main()
{
    const int Nc = 4096;
    std::vector<int> seen(Nc, 0);
    for (int r = 0; r < Nc; ++r) {
        const int c = vbits_code_bit(r);
        if (c < 0 || c >= Nc || (c >> 7) != (r >> 7)) { std::printf("row %d leaves its run of 128: %d\n", r, c); return 1; }
        if (seen[c]++) { std::printf("code bit %d reached twice\n", c); return 1; }
    }
    for (int W = 0; W < Nc / 128; ++W)
        for (int p = 0; p < 8; ++p)
            for (int n = 0; n < 16; ++n) {
                const int row = 128 * W + 16 * p + n;
                const int bit = 32 * (4 * W + n / 4) + 8 * (n % 4) + p;
                if (vbits_code_bit(row) != bit) { std::printf("row %d -> %d, lane mapping says %d\n", row, vbits_code_bit(row), bit); return 1; }
            }
    std::puts("vbits_rows: ok");
    return 0;
}
