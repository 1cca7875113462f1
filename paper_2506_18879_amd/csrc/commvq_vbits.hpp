// Value stage for the paper's binary value code (Sec. 4.1): interface between commvq.hip and commvq_vbits.hip.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

// Geometry shared by the planner and the kernel: a workgroup takes kVbitsHeads query heads x kVbitsCols code bits of
// one token range.
constexpr int kVbitsHeads = 16;
constexpr int kVbitsCols = 1024;

// Row r of a KV head's bins holds code bit vbits_code_bit(r): within every run of 128 rows the seven low bits are
// permuted so that the 16 lanes of a matrix-instruction result column block (lane n, pass p -> dword n / 4 of the
// wavefront's four, byte n % 4, bit p) own 16 consecutive rows r = 16 p + n and store them as one contiguous run.
__host__ __device__ inline int vbits_code_bit(int r)
{
    return (r & ~127) | (((r >> 2) & 3) << 5) | ((r & 3) << 3) | ((r >> 4) & 7);
}

struct VbitsArgs {
    const uint8_t *val_bits;  // sequence b: [L_b][Nc / 8] at byte offset cu[b] * Nc / 8
    const int32_t *cu;        // [B + 1]
    const float *scores;      // scaled logits, (b, h, i) at cu[b] * Hq + h * L_b + i
    const float2 *sstat;      // [B * Hq][nsplit] (max, sum of exp(logit - max)) of the score-stage tiles
    unsigned *bins;           // [B * Hkv][nvsplit][Nc rows][G], row r = code bit vbits_code_bit(r)
    float *vscale, *lsum;     // [B * Hq][nvsplit]
    int Hq, Hkv, G;
    int nsplit, split_len;    // statistics tiles of the score stage
    int nvsplit, vsplit_len;  // token ranges of this stage
    int Nc;                   // code bits per token (multiple of kVbitsCols)
    int batch;
};

// Enqueues k_vbits for every (sequence, token range, head group, column group).  The caller has checked the shapes.
hipError_t commvq_launch_vbits(const VbitsArgs &a, hipStream_t stream);
