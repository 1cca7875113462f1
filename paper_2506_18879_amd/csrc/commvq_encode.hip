// libcommvq: key encoding for cache append (residual nearest-centre search), hand-written for gfx950.
#include "commvq_internal.hpp"

namespace {

// ------------------------------------------------------------------ key encoding (cache append)
// Residual nearest-centre search (Sec. 4.2: the E step's assignment, level by level on the error of the
// previous levels; App. A.1 for the paired centres).  ||res - c||^2 = ||res||^2 - 2 res.c + ||c||^2, so a
// level needs the dot products of the residual with that level's rows and a table of squared norms:
//   norms[g][level][K]            ||C[g][level][c]||^2
//   cross[g][level][K][K]         paired only: 2 C[a] . (i C[b])   (K = 64), so that a paired centre costs
//                                 norms[a] + norms[b] + cross[a][b] - 2 (res.C[a] + res.(i C[b]))
template <bool BF16>
__global__ __launch_bounds__(256) void k_encode_tables(const void *__restrict__ cb, float *__restrict__ norms,
                                                       float *__restrict__ cross, int rows_total, int K, int paired)
{
    const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (t < (size_t)rows_total) {
        float acc = 0.f;
        for (int e = 0; e < kD; ++e) {
            const float v = cb_elem<BF16>(cb, t * kD + e);
            acc = __builtin_fmaf(v, v, acc);
        }
        norms[t] = acc;
    }
    if (paired && t < (size_t)rows_total * K) {
        const size_t level = t / ((size_t)K * K);   // g * R + r
        const int a = (int)(t / K % K), b = (int)(t % K);
        const size_t ra = (level * K + a) * kD, rb = (level * K + b) * kD;
        float acc = 0.f;
        for (int j = 0; j < kJ; ++j) {  // (x_a, y_a) . (-y_b, x_b)
            const float xa = cb_elem<BF16>(cb, ra + 2 * j), ya = cb_elem<BF16>(cb, ra + 2 * j + 1);
            const float xb = cb_elem<BF16>(cb, rb + 2 * j), yb = cb_elem<BF16>(cb, rb + 2 * j + 1);
            acc = __builtin_fmaf(ya, xb, __builtin_fmaf(-xa, yb, acc));
        }
        cross[t] = 2.f * acc;
    }
}

struct EncodeDims {
    int Hkv, levels, K, key_bf16, record_bytes;
    long long token_stride, head_stride;
};

// Index-form keys, fp32 codebooks: one workgroup per (token, KV head), one thread per centre of the level, rows
// straight from L2.  Ties go to the lowest index.  (bf16 codebooks: k_encode_dma and k_encode_batch below.)
template <bool BF16>
__global__ __launch_bounds__(256) void k_encode(const void *__restrict__ keys, const void *__restrict__ cb,
                                                const float *__restrict__ norms, uint8_t *__restrict__ out, const EncodeDims a)
{
    __shared__ float res[kD];
    __shared__ float wbest[4];
    __shared__ int wcand[4];
    __shared__ int chosen[32];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = blockIdx.x % a.Hkv;
    const size_t tok = blockIdx.x / a.Hkv;
    const int K = a.K;  // 256 = the workgroup size
    if (tid < kD) {
        const size_t i = (tok * a.Hkv + g) * kD + tid;
        res[tid] = a.key_bf16 ? __builtin_bit_cast(float, (unsigned)static_cast<const uint16_t *>(keys)[i] << 16)
                              : static_cast<const float *>(keys)[i];
    }
    __syncthreads();
    for (int l = 0; l < a.levels; ++l) {
        const size_t level = (size_t)g * a.levels + l;
        const size_t base = level * K * kD;
        float acc = 0.f;
#pragma unroll 16
        for (int e = 0; e < kD; ++e) acc = __builtin_fmaf(res[e], cb_elem<BF16>(cb, base + (size_t)tid * kD + e), acc);
        const float best = norms[level * K + tid] - 2.f * acc;
        // argmin over the workgroup, lowest index on ties
        const float wm = -wave_max(-best);
        int wc = best == wm ? tid : 0x7fffffff;
        for (int off = 32; off > 0; off >>= 1) wc = min(wc, __shfl_xor(wc, off));
        if (lane == 0) { wbest[wave] = wm; wcand[wave] = wc; }
        __syncthreads();
        float m = wbest[0];
        int c = wcand[0];
        for (int w = 1; w < 4; ++w)
            if (wbest[w] < m || (wbest[w] == m && wcand[w] < c)) { m = wbest[w]; c = wcand[w]; }
        if (tid == 0) chosen[l] = c;
        if (tid < kD) res[tid] -= cb_elem<BF16>(cb, base + (size_t)c * kD + tid);
        __syncthreads();
    }
    if (tid < a.levels) out[tok * a.token_stride + (long long)g * a.head_stride + tid] = (uint8_t)chosen[tid];
}

// Index-form keys, few tokens (a decode step appends one token per sequence): the levels are a dependent chain,
// so what counts is the latency of one level.  The rows of level l + 1 do not depend on the residual: they travel
// from memory straight into LDS (global_load_lds_dwordx4: 16 bytes per lane, no register destination) while
// level l is searched, into the other half of a double buffer; a level then reads its rows -- and the winning
// row for the residual update -- from LDS instead of waiting for memory twice.  Image of a level: row-major,
// [256 rows][16 slots] x 16 bytes, with piece x of row t in slot (x + t) mod 16 of its row: a thread then reads its
// own row without bank conflicts, and one load instruction (64 lanes -> 64 consecutive slots from the slot in
// M0) still covers four whole rows = 1 KiB of contiguous memory, only permuted within each row: lane (r, col) of
// the instruction fetches piece (col - t) mod 16 of row t = first row + r.  (One row per lane, the obvious
// mapping, touches 64 different cache lines per instruction: 2 us per level instead of 0.5.)
// The loads are issued from inline asm: the compiler
// then knows nothing of them and makes no LDS access wait for them; the kernel waits itself (s_waitcnt vmcnt(0))
// at the top of the next level.  No static LDS: the images sit at LDS address 0.
constexpr int kEdImg = 16 * 256;  // 16-byte pieces of one level's rows
constexpr int kEdLds = 2 * kEdImg * 16 + kD * 4 + 8 * 4 + 8 * 4 + 32 * 4;
__global__ __launch_bounds__(256) void k_encode_dma(const void *__restrict__ keys, const uint4 *__restrict__ cb,
                                                    const float *__restrict__ norms, uint8_t *__restrict__ out, const EncodeDims a)
{
    extern __shared__ __attribute__((aligned(16))) uint4 ed_lds[];
    uint4 *img = ed_lds;                                              // [2][16][256]
    float *res = reinterpret_cast<float *>(ed_lds + 2 * kEdImg);      // [d]
    float *wbest = res + kD;                                          // [2][4]
    int *wcand = reinterpret_cast<int *>(wbest + 8);                  // [2][4]
    int *chosen = wcand + 8;                                          // [32]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = blockIdx.x % a.Hkv;
    const size_t tok = blockIdx.x / a.Hkv;
    const uint4 *rows = cb + (size_t)g * a.levels * kK * 16;  // level 0 of this head; a level is kK * 16 pieces on
    auto dma_level = [&](int l, int buf) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {  // instruction i of the wavefront: rows 64 wave + 4 i .. + 3
            const int t = wave * 64 + 4 * i + (lane >> 4);
            const unsigned slot = __builtin_amdgcn_readfirstlane((unsigned)(buf * kEdImg + (wave * 64 + 4 * i) * 16));
            lds_dma16(rows + ((size_t)l * kK + t) * 16 + ((lane - t) & 15), slot * 16u);
        }
    };
    dma_level(0, 0);
    if (tid < kD) {
        const size_t i = (tok * a.Hkv + g) * kD + tid;
        res[tid] = a.key_bf16 ? __builtin_bit_cast(float, (unsigned)static_cast<const uint16_t *>(keys)[i] << 16)
                              : static_cast<const float *>(keys)[i];
    }
    float nrm = norms[(size_t)g * a.levels * kK + tid];
    for (int l = 0; l < a.levels; ++l) {
        const int buf = l & 1;
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this wavefront's rows of level l have landed
        __syncthreads();                                   // ... and everybody's; the residual is up to date
        uint4 pc[16];
#pragma unroll
        for (int x = 0; x < 16; ++x) pc[x] = img[buf * kEdImg + tid * 16 + ((x + tid) & 15)];
        float nrm_next = 0.f;
        if (l + 1 < a.levels) {
            // the other image was last read during level l - 1, before the barrier above
            dma_level(l + 1, buf ^ 1);
            nrm_next = norms[((size_t)g * a.levels + l + 1) * kK + tid];
        }
        float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
#pragma unroll
        for (int x = 0; x < 16; ++x) {
            const unsigned v[4] = {pc[x].x, pc[x].y, pc[x].z, pc[x].w};
            const float4 r0 = *reinterpret_cast<const float4 *>(res + 8 * x), r1 = *reinterpret_cast<const float4 *>(res + 8 * x + 4);
            a0 = __builtin_fmaf(r0.x, bf16_lo(v[0]), a0); a1 = __builtin_fmaf(r0.y, bf16_hi(v[0]), a1);
            a2 = __builtin_fmaf(r0.z, bf16_lo(v[1]), a2); a3 = __builtin_fmaf(r0.w, bf16_hi(v[1]), a3);
            a0 = __builtin_fmaf(r1.x, bf16_lo(v[2]), a0); a1 = __builtin_fmaf(r1.y, bf16_hi(v[2]), a1);
            a2 = __builtin_fmaf(r1.z, bf16_lo(v[3]), a2); a3 = __builtin_fmaf(r1.w, bf16_hi(v[3]), a3);
        }
        const float best = nrm - 2.f * ((a0 + a1) + (a2 + a3));
        // argmin over the workgroup, lowest index on ties
        const float wm = -wave_max(-best);
        const unsigned long long hit = __ballot(best == wm);
        if (lane == 0) { wbest[buf * 4 + wave] = wm; wcand[buf * 4 + wave] = wave * 64 + (int)__builtin_ctzll(hit); }
        __syncthreads();
        float m = wbest[buf * 4];
        int c = wcand[buf * 4];
        for (int w = 1; w < 4; ++w)
            if (wbest[buf * 4 + w] < m || (wbest[buf * 4 + w] == m && wcand[buf * 4 + w] < c)) { m = wbest[buf * 4 + w]; c = wcand[buf * 4 + w]; }
        if (tid == 0) chosen[l] = c;
        if (tid < kD / 2) {  // dword tid of row c: piece tid / 4
            const unsigned v = reinterpret_cast<const unsigned *>(img)[(buf * kEdImg + c * 16 + (((tid >> 2) + c) & 15)) * 4 + (tid & 3)];
            res[2 * tid] -= bf16_lo(v);
            res[2 * tid + 1] -= bf16_hi(v);
        }
        nrm = nrm_next;
    }
    __syncthreads();
    if (tid < a.levels) out[tok * a.token_stride + (long long)g * a.head_stride + tid] = (uint8_t)chosen[tid];
}

// Index-form keys, many tokens at once (prefill-sized chunks): the dot products of a level are a
// (256 rows x 128) x (128 x tokens) matrix product, so they run on the matrix cores.  A workgroup takes 64
// tokens of one KV head (16 per wavefront) and stages the level's 256 bf16 rows in LDS once for all of them.
// The fp32 residual of a token is split EXACTLY into three bf16 parts (its 24 mantissa bits are 8 + 8 + 8:
// truncate, subtract, truncate, subtract), each multiplied with the exact bf16 rows and accumulated in fp32:
// the same dot product as the fp32 FMA chain of k_encode up to summation order.
//   first operand : 16 rows x 32 elements from LDS (row stride 288 bytes: the 16 lanes of a k-group and the two
//                   k-groups that are checked together hit different banks)
//   second operand: lane (n, g) supplies elements 32 kc + 8 g .. + 7 of token n, the part of the residual it keeps
//   result        : lane (n, g) receives rows 4 g .. 4 g + 3 of the row tile for token n
constexpr int kEbTokens = 64;
constexpr int kEbRowBytes = 288;
constexpr int kEbLds = 256 * kEbRowBytes + 256 * 4 + (kEbTokens * 32);
__global__ __launch_bounds__(256) void k_encode_batch(const void *__restrict__ keys, const uint4 *__restrict__ cb,
                                                      const float *__restrict__ norms, uint8_t *__restrict__ out,
                                                      const EncodeDims a, int n_tokens)
{
    extern __shared__ __attribute__((aligned(16))) uint4 eb_lds[];
    char *rows = reinterpret_cast<char *>(eb_lds);
    float *nrm = reinterpret_cast<float *>(rows + 256 * kEbRowBytes);
    uint8_t *chosen = reinterpret_cast<uint8_t *>(nrm + 256);  // [64 tokens][32 levels]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, gk = lane >> 4;
    const int g = blockIdx.x % a.Hkv;
    const int tl = wave * 16 + n;                                // token within the workgroup
    const long long tok = (long long)(blockIdx.x / a.Hkv) * kEbTokens + tl;
    const size_t tokc = (size_t)(tok < n_tokens ? tok : n_tokens - 1);
    float res[4][8];
#pragma unroll
    for (int kc = 0; kc < 4; ++kc) {
        const size_t i = (tokc * a.Hkv + g) * kD + kc * 32 + 8 * gk;
        if (a.key_bf16) {
            const uint4 v = *reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(keys) + i);
            const unsigned w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) { res[kc][2 * e] = bf16_lo(w[e]); res[kc][2 * e + 1] = bf16_hi(w[e]); }
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) res[kc][e] = static_cast<const float *>(keys)[i + e];
        }
    }
    for (int l = 0; l < a.levels; ++l) {
        const size_t level = (size_t)g * a.levels + l;
        __syncthreads();  // the previous level's rows are no longer read
        for (int x = tid; x < 256 * 16; x += 256)
            *reinterpret_cast<uint4 *>(rows + (x >> 4) * kEbRowBytes + (x & 15) * 16) = cb[level * 256 * 16 + x];
        nrm[tid] = norms[level * 256 + tid];
        __syncthreads();
        // exact three-way bf16 split of the lane's part of the residual, packed as MFMA operands
        uint4_t part[3][4];
#pragma unroll
        for (int kc = 0; kc < 4; ++kc)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float v0 = res[kc][2 * e], v1 = res[kc][2 * e + 1];
#pragma unroll
                for (int s3 = 0; s3 < 3; ++s3) {
                    const unsigned t0 = __builtin_bit_cast(unsigned, v0) & 0xffff0000u, t1 = __builtin_bit_cast(unsigned, v1) & 0xffff0000u;
                    part[s3][kc][e] = (t0 >> 16) | t1;
                    v0 -= __builtin_bit_cast(float, t0);
                    v1 -= __builtin_bit_cast(float, t1);
                }
            }
        float best = INFINITY;
        int brow = 0;
#pragma unroll 2
        for (int rt = 0; rt < 16; ++rt) {
            floatx4_t D = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kc = 0; kc < 4; ++kc) {
                const uint4 pc = *reinterpret_cast<const uint4 *>(rows + (rt * 16 + n) * kEbRowBytes + kc * 64 + gk * 16);
                const uint4_t pv = {pc.x, pc.y, pc.z, pc.w};
                const bf16x8_t A = __builtin_bit_cast(bf16x8_t, pv);
#pragma unroll
                for (int s3 = 0; s3 < 3; ++s3) D = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, __builtin_bit_cast(bf16x8_t, part[s3][kc]), D, 0, 0, 0);
            }
            const float4 nr = *reinterpret_cast<const float4 *>(nrm + rt * 16 + 4 * gk);
            const float nv[4] = {nr.x, nr.y, nr.z, nr.w};
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float sc = nv[r] - 2.f * D[r];
                if (sc < best) { best = sc; brow = rt * 16 + 4 * gk + r; }  // rows come in increasing order: ties keep the lowest
            }
        }
        // the four lanes of a token hold the minima of disjoint row sets
#pragma unroll
        for (int off = 16; off <= 32; off <<= 1) {
            const float ov = __shfl_xor(best, off);
            const int orow = __shfl_xor(brow, off);
            if (ov < best || (ov == best && orow < brow)) { best = ov; brow = orow; }
        }
        if (gk == 0) chosen[tl * 32 + l] = (uint8_t)brow;
        // residual -= chosen row (the lane's 32 elements of it)
#pragma unroll
        for (int kc = 0; kc < 4; ++kc) {
            const uint4 pc = *reinterpret_cast<const uint4 *>(rows + brow * kEbRowBytes + kc * 64 + gk * 16);
            const unsigned w[4] = {pc.x, pc.y, pc.z, pc.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) { res[kc][2 * e] -= bf16_lo(w[e]); res[kc][2 * e + 1] -= bf16_hi(w[e]); }
        }
    }
    __syncthreads();
    if (tok < n_tokens) {
        uint8_t *dst = out + tok * a.token_stride + (long long)g * a.head_stride;
        for (int l = gk; l < a.levels; l += 4) dst[l] = chosen[tl * 32 + l];
    }
}

// Paired-format keys, many tokens at once.  Same scheme as k_encode_batch for the two sets of 64 dot products of a
// level -- P[a] = res . C[a] and Q[b] = res . (i C[b]) = res' . C[b] with res' = (res_y, -res_x) per sub-space, whose
// bf16 parts are the parts of res with halves swapped and one sign flipped -- then every lane scans 16 x 64 of the
// token's 4096 centres:  ||c_ab||^2 - 2 res . c_ab = (N[a] - 2 P[a]) + (N[b] - 2 Q[b]) + X[a][b].
constexpr int kEpRowBytes = 288;
constexpr int kEpVecBytes = 272;  // padded stride of a token's 64 floats: 16 tokens hit 64 different banks
constexpr int kEpLds = 64 * kEpRowBytes + 64 * 64 * 4 + 64 * 4 + 2 * kEbTokens * kEpVecBytes + kEbTokens * 64;
__global__ __launch_bounds__(256) void k_encode_pair_batch(const void *__restrict__ keys, const uint4 *__restrict__ cb,
                                                           const float *__restrict__ norms, const float *__restrict__ cross,
                                                           uint8_t *__restrict__ out, const EncodeDims a, int n_tokens)
{
    extern __shared__ __attribute__((aligned(16))) uint4 ep_lds[];
    char *rows = reinterpret_cast<char *>(ep_lds);                        // [64][288 B]
    float *xs = reinterpret_cast<float *>(rows + 64 * kEpRowBytes);       // [64][64]
    float *nrm = xs + 64 * 64;                                            // [64]
    char *uvec = reinterpret_cast<char *>(nrm + 64);                      // [64 tokens][272 B]: N[a] - 2 P[a]
    char *vvec = uvec + kEbTokens * kEpVecBytes;                          // [64 tokens][272 B]: N[b] - 2 Q[b]
    uint8_t *chosen = reinterpret_cast<uint8_t *>(vvec + kEbTokens * kEpVecBytes);  // [64 tokens][32 levels][2]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, gk = lane >> 4;
    const int g = blockIdx.x % a.Hkv;
    const int tl = wave * 16 + n;
    const long long tok = (long long)(blockIdx.x / a.Hkv) * kEbTokens + tl;
    const size_t tokc = (size_t)(tok < n_tokens ? tok : n_tokens - 1);
    float res[4][8];
#pragma unroll
    for (int kc = 0; kc < 4; ++kc) {
        const size_t i = (tokc * a.Hkv + g) * kD + kc * 32 + 8 * gk;
        if (a.key_bf16) {
            const uint4 v = *reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(keys) + i);
            const unsigned w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) { res[kc][2 * e] = bf16_lo(w[e]); res[kc][2 * e + 1] = bf16_hi(w[e]); }
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) res[kc][e] = static_cast<const float *>(keys)[i + e];
        }
    }
    // a level's tables do not depend on the residual: they are fetched into registers one level ahead
    uint4 prow0, prow1, prow2, prow3;
    float4 pcr0, pcr1, pcr2, pcr3;
    float pnorm = 0.f;
#define COMMVQ_EP_FETCH(l_)                                                                        \
    {                                                                                              \
        const size_t level_ = (size_t)g * a.levels + (l_);                                         \
        const uint4 *r_ = cb + level_ * 64 * 16 + tid;                                             \
        const float4 *c_ = reinterpret_cast<const float4 *>(cross + level_ * 64 * 64) + tid;       \
        prow0 = r_[0]; prow1 = r_[256]; prow2 = r_[512]; prow3 = r_[768];                          \
        pcr0 = c_[0]; pcr1 = c_[256]; pcr2 = c_[512]; pcr3 = c_[768];                              \
        if (tid < 64) pnorm = norms[level_ * 64 + tid];                                            \
    }
    COMMVQ_EP_FETCH(0)
    for (int l = 0; l < a.levels; ++l) {
        __syncthreads();  // the previous level's tables are no longer read
        {
            char *rp = rows + (tid >> 4) * kEpRowBytes + (tid & 15) * 16;  // element tid + 256 x: 16 rows further on
            *reinterpret_cast<uint4 *>(rp) = prow0;
            *reinterpret_cast<uint4 *>(rp + 16 * kEpRowBytes) = prow1;
            *reinterpret_cast<uint4 *>(rp + 32 * kEpRowBytes) = prow2;
            *reinterpret_cast<uint4 *>(rp + 48 * kEpRowBytes) = prow3;
            float4 *xp = reinterpret_cast<float4 *>(xs) + tid;
            xp[0] = pcr0; xp[256] = pcr1; xp[512] = pcr2; xp[768] = pcr3;
        }
        if (tid < 64) nrm[tid] = pnorm;
        if (l + 1 < a.levels) COMMVQ_EP_FETCH(l + 1)
        __syncthreads();
        uint4_t part[3][4];
#pragma unroll
        for (int kc = 0; kc < 4; ++kc)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float v0 = res[kc][2 * e], v1 = res[kc][2 * e + 1];
#pragma unroll
                for (int s3 = 0; s3 < 3; ++s3) {
                    const unsigned t0 = __builtin_bit_cast(unsigned, v0) & 0xffff0000u, t1 = __builtin_bit_cast(unsigned, v1) & 0xffff0000u;
                    part[s3][kc][e] = (t0 >> 16) | t1;
                    v0 -= __builtin_bit_cast(float, t0);
                    v1 -= __builtin_bit_cast(float, t1);
                }
            }
        // P and Q for the 64 rows, 16 at a time; lane (n, gk) receives rows 16 rt + 4 gk .. + 3 of token n
#pragma unroll
        for (int rt = 0; rt < 4; ++rt) {
            floatx4_t DP = {0.f, 0.f, 0.f, 0.f}, DQ = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kc = 0; kc < 4; ++kc) {
                const uint4 pc = *reinterpret_cast<const uint4 *>(rows + (rt * 16 + n) * kEpRowBytes + kc * 64 + gk * 16);
                const uint4_t pv = {pc.x, pc.y, pc.z, pc.w};
                const bf16x8_t A = __builtin_bit_cast(bf16x8_t, pv);
#pragma unroll
                for (int s3 = 0; s3 < 3; ++s3) {
                    DP = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, __builtin_bit_cast(bf16x8_t, part[s3][kc]), DP, 0, 0, 0);
                    uint4_t rot;  // (x, y) -> (y, -x): swap the halves, flip the sign of the new upper half
#pragma unroll
                    for (int e = 0; e < 4; ++e) rot[e] = __builtin_amdgcn_alignbit(part[s3][kc][e], part[s3][kc][e], 16) ^ 0x80000000u;
                    DQ = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, __builtin_bit_cast(bf16x8_t, rot), DQ, 0, 0, 0);
                }
            }
            const float4 nr = *reinterpret_cast<const float4 *>(nrm + rt * 16 + 4 * gk);
            *reinterpret_cast<float4 *>(uvec + tl * kEpVecBytes + (rt * 16 + 4 * gk) * 4) =
                make_float4(nr.x - 2.f * DP[0], nr.y - 2.f * DP[1], nr.z - 2.f * DP[2], nr.w - 2.f * DP[3]);
            *reinterpret_cast<float4 *>(vvec + tl * kEpVecBytes + (rt * 16 + 4 * gk) * 4) =
                make_float4(nr.x - 2.f * DQ[0], nr.y - 2.f * DQ[1], nr.z - 2.f * DQ[2], nr.w - 2.f * DQ[3]);
        }
        __syncthreads();
        // scan in two stages, with the result of a sequential scan in increasing a * 64 + b under a strict "<":
        // rounding is monotone, so min over b of fl(u + t[b]) is fl(u + min t[b]), and stage one needs only an add
        // and half a three-way minimum per centre.  Lane (n, gk) takes a = 16 gk .. 16 gk + 15 and all b of token n.
        float vb[64];
#pragma unroll
        for (int b4 = 0; b4 < 16; ++b4) {
            const float4 v4 = *reinterpret_cast<const float4 *>(vvec + tl * kEpVecBytes + b4 * 16);
            vb[4 * b4] = v4.x; vb[4 * b4 + 1] = v4.y; vb[4 * b4 + 2] = v4.z; vb[4 * b4 + 3] = v4.w;
        }
        float best = INFINITY;
        int ca = 0;
        {
            // the cross terms are read a quarter row (four float4) ahead of their use; the read ahead of the last
            // quarter of row 63 lands on the norms that follow the cross table in LDS and is not used
            const float4 *xrow = reinterpret_cast<const float4 *>(xs) + 16 * gk * 16;
            float4 cur[4], nxt[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) cur[q] = xrow[q];
            for (int ai = 0; ai < 16; ++ai) {
                float m = INFINITY;
#pragma unroll
                for (int c = 0; c < 4; ++c) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) nxt[q] = xrow[ai * 16 + (c + 1) * 4 + q];
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int b = 16 * c + 4 * q;
                        m = fminf(fminf(m, vb[b] + cur[q].x), vb[b + 1] + cur[q].y);
                        m = fminf(fminf(m, vb[b + 2] + cur[q].z), vb[b + 3] + cur[q].w);
                    }
#pragma unroll
                    for (int q = 0; q < 4; ++q) cur[q] = nxt[q];
                }
                const int a2 = 16 * gk + ai;
                const float sc = *reinterpret_cast<const float *>(uvec + tl * kEpVecBytes + a2 * 4) + m;
                if (sc < best) { best = sc; ca = a2; }
            }
        }
#pragma unroll
        for (int off = 16; off <= 32; off <<= 1) {
            const float ov = __shfl_xor(best, off);
            const int oc = __shfl_xor(ca, off);
            if (ov < best || (ov == best && oc < ca)) { best = ov; ca = oc; }
        }
        // stage two: the lowest b of row ca whose sum rounds to the minimum; the four lanes of a token take 16 b each
        int cb2 = 64;
        {
            const float ua = *reinterpret_cast<const float *>(uvec + tl * kEpVecBytes + ca * 4);
#pragma unroll
            for (int b4 = 3; b4 >= 0; --b4) {
                const float4 v4 = *reinterpret_cast<const float4 *>(vvec + tl * kEpVecBytes + (4 * gk + b4) * 16);
                const float4 xb = *reinterpret_cast<const float4 *>(xs + ca * 64 + (4 * gk + b4) * 4);
                const int b0 = 16 * gk + 4 * b4;
                if (ua + (v4.w + xb.w) == best) cb2 = b0 + 3;
                if (ua + (v4.z + xb.z) == best) cb2 = b0 + 2;
                if (ua + (v4.y + xb.y) == best) cb2 = b0 + 1;
                if (ua + (v4.x + xb.x) == best) cb2 = b0;
            }
#pragma unroll
            for (int off = 16; off <= 32; off <<= 1) cb2 = min(cb2, __shfl_xor(cb2, off));
            cb2 &= 63;  // always below 64 for finite input; keeps the row read in range otherwise
        }
        if (gk == 0) { chosen[(tl * 32 + l) * 2] = (uint8_t)ca; chosen[(tl * 32 + l) * 2 + 1] = (uint8_t)cb2; }
        // residual -= C[a] + i C[b]: per sub-space (x_a - y_b, y_a + x_b)
#pragma unroll
        for (int kc = 0; kc < 4; ++kc) {
            const uint4 pa = *reinterpret_cast<const uint4 *>(rows + ca * kEpRowBytes + kc * 64 + gk * 16);
            const uint4 pb = *reinterpret_cast<const uint4 *>(rows + cb2 * kEpRowBytes + kc * 64 + gk * 16);
            const unsigned wa[4] = {pa.x, pa.y, pa.z, pa.w}, wb[4] = {pb.x, pb.y, pb.z, pb.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                res[kc][2 * e] -= bf16_lo(wa[e]) - bf16_hi(wb[e]);
                res[kc][2 * e + 1] -= bf16_hi(wa[e]) + bf16_lo(wb[e]);
            }
        }
    }
    __syncthreads();
    if (tok < n_tokens) {
        uint8_t *dst = out + tok * a.token_stride + (long long)g * a.head_stride;
        for (int byte = gk; byte < a.record_bytes; byte += 4) {
            unsigned v = 0;
            for (int r = (8 * byte) / 12; r < a.levels && 12 * r < 8 * byte + 8; ++r) {
                const unsigned pr = (unsigned)chosen[(tl * 32 + r) * 2] | (unsigned)chosen[(tl * 32 + r) * 2 + 1] << 6;
                const int sh = 12 * r - 8 * byte;
                v |= sh >= 0 ? pr << sh : pr >> -sh;
            }
            dst[byte] = (uint8_t)(v & 0xffu);
        }
    }
}

#undef COMMVQ_EP_FETCH

// Paired-format keys (and the template's index-form variant, not dispatched: staging 64 KiB of rows that are
// used once does not pay), shaped for latency (a decode step appends one token per sequence, and the R
// levels are a dependent chain): the rows, norms and cross terms of level l + 1 do not depend on the
// residual, so they are fetched into registers while level l is searched and parked in the other half
// of a double-buffered LDS image; every level then runs out of LDS.  Rows are padded to 65 dwords so
// that 64 lanes reading 64 different rows hit 64 different banks.
constexpr int kEncRowDw = kD / 2 + 1;  // dwords per padded bf16 row
template <bool PAIRED>
__global__ __launch_bounds__(256) void k_encode_lds(const void *__restrict__ keys, const unsigned *__restrict__ cb,
                                                    const float *__restrict__ norms, const float *__restrict__ cross,
                                                    uint8_t *__restrict__ out, const EncodeDims a)
{
    constexpr int K = PAIRED ? 64 : 256;
    constexpr int ROWS_DW = K * kEncRowDw;             // one level's rows
    constexpr int CROSS = PAIRED ? K * K : 0;
    constexpr int RPT = K * (kD / 2) / 256;            // row dwords per thread: 16 (paired) or 64
    constexpr int XPT = CROSS / 256;
    extern __shared__ __attribute__((aligned(16))) unsigned enc_lds[];
    unsigned *rows = enc_lds;                                          // [2][K][65]
    float *xs = reinterpret_cast<float *>(enc_lds + 2 * ROWS_DW);      // [2][K * K]  (paired)
    float *ns = xs + 2 * CROSS;                                        // [2][K]
    float *res = ns + 2 * K;                                           // [d]
    float *dots = res + kD;                                            // [256]
    float *wbest = dots + 256;                                         // [4]
    int *wcand = reinterpret_cast<int *>(wbest + 4);                   // [4]
    int *chosen = wcand + 4;                                           // [32]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = blockIdx.x % a.Hkv;
    const size_t tok = blockIdx.x / a.Hkv;

    unsigned prow[RPT];
    float pcross[XPT > 0 ? XPT : 1], pnorm = 0.f;
    auto fetch_level = [&](int l) {
        const size_t level = (size_t)g * a.levels + l;
#pragma unroll
        for (int x = 0; x < RPT; ++x) prow[x] = cb[level * K * (kD / 2) + x * 256 + tid];
#pragma unroll
        for (int x = 0; x < XPT; ++x) pcross[x] = cross[level * CROSS + x * 256 + tid];
        if (tid < K) pnorm = norms[level * K + tid];
    };
    auto park_level = [&](int buf) {
#pragma unroll
        for (int x = 0; x < RPT; ++x) {
            const int i = x * 256 + tid;  // dword i of the level: row i / 64, column i % 64
            rows[buf * ROWS_DW + (i >> 6) * kEncRowDw + (i & 63)] = prow[x];
        }
#pragma unroll
        for (int x = 0; x < XPT; ++x) xs[buf * CROSS + x * 256 + tid] = pcross[x];
        if (tid < K) ns[buf * K + tid] = pnorm;
    };
    fetch_level(0);
    if (tid < kD) {
        const size_t i = (tok * a.Hkv + g) * kD + tid;
        res[tid] = a.key_bf16 ? __builtin_bit_cast(float, (unsigned)static_cast<const uint16_t *>(keys)[i] << 16)
                              : static_cast<const float *>(keys)[i];
    }
    park_level(0);
    __syncthreads();
    for (int l = 0; l < a.levels; ++l) {
        const int buf = l & 1;
        if (l + 1 < a.levels) fetch_level(l + 1);
        const unsigned *R = rows + buf * ROWS_DW;
        float best = INFINITY;
        int cand = 0x7fffffff;
        if (!PAIRED) {
            float acc = 0.f;
#pragma unroll 16
            for (int j = 0; j < kJ; ++j) {
                const unsigned v = R[tid * kEncRowDw + j];
                acc = __builtin_fmaf(res[2 * j], bf16_lo(v), acc);
                acc = __builtin_fmaf(res[2 * j + 1], bf16_hi(v), acc);
            }
            best = ns[buf * K + tid] - 2.f * acc;
            cand = tid;
        } else {
            // thread = (row c, a-dot or b-dot, which half of the sub-spaces); the two halves are added in a fixed order
            const int c = tid & 63, second = (tid >> 6) & 1, hj = tid >> 7;
            float acc0 = 0.f, acc1 = 0.f;  // two chains (even / odd sub-spaces), added in a fixed order
#pragma unroll 16
            for (int j = 32 * hj; j < 32 * hj + 32; j += 2) {
                const unsigned v = R[c * kEncRowDw + j], w = R[c * kEncRowDw + j + 1];
                const float4 r = *reinterpret_cast<const float4 *>(res + 2 * j);
                const float x = bf16_lo(v), y = bf16_hi(v), x1 = bf16_lo(w), y1 = bf16_hi(w);
                acc0 = second ? __builtin_fmaf(r.y, x, __builtin_fmaf(-r.x, y, acc0)) : __builtin_fmaf(r.y, y, __builtin_fmaf(r.x, x, acc0));
                acc1 = second ? __builtin_fmaf(r.w, x1, __builtin_fmaf(-r.z, y1, acc1)) : __builtin_fmaf(r.w, y1, __builtin_fmaf(r.z, x1, acc1));
            }
            dots[tid] = acc0 + acc1;
            __syncthreads();
            // candidate k * 256 + tid is the pair (a = 4 k + tid / 64, b = tid % 64): b is the thread's own
            const int cb2 = tid & (K - 1);
            const float vb = ns[buf * K + cb2] - 2.f * (dots[64 + cb2] + dots[192 + cb2]);
#pragma unroll
            for (int k = 0; k < K * K / 256; ++k) {
                const int cc = k * 256 + tid, ca = cc / K;
                const float ua = ns[buf * K + ca] - 2.f * (dots[ca] + dots[128 + ca]);
                const float sc = ua + (vb + xs[buf * CROSS + cc]);
                if (sc < best) { best = sc; cand = cc; }
            }
        }
        const float wm = -wave_max(-best);
        int wc = best == wm ? cand : 0x7fffffff;
        for (int off = 32; off > 0; off >>= 1) wc = min(wc, __shfl_xor(wc, off));
        if (lane == 0) { wbest[wave] = wm; wcand[wave] = wc; }
        __syncthreads();
        {
            float m = wbest[0];
            int c = wcand[0];
            for (int w = 1; w < 4; ++w)
                if (wbest[w] < m || (wbest[w] == m && wcand[w] < c)) { m = wbest[w]; c = wcand[w]; }
            if (tid == 0) chosen[l] = c;
            if (tid < kD) {
                const int e2 = tid >> 1;
                if (!PAIRED) {
                    const unsigned v = R[c * kEncRowDw + e2];
                    res[tid] -= (tid & 1) ? bf16_hi(v) : bf16_lo(v);
                } else {
                    const unsigned va = R[(c / K) * kEncRowDw + e2], vb = R[(c % K) * kEncRowDw + e2];
                    // element of i C[b]: (-y_b, x_b) of its sub-space
                    res[tid] -= (tid & 1) ? bf16_hi(va) + bf16_lo(vb) : bf16_lo(va) - bf16_hi(vb);
                }
            }
        }
        if (l + 1 < a.levels) park_level(buf ^ 1);
        __syncthreads();
    }
    uint8_t *dst = out + tok * a.token_stride + (long long)g * a.head_stride;
    if (!PAIRED) {
        if (tid < a.levels) dst[tid] = (uint8_t)chosen[tid];
    } else if (tid < a.record_bytes) {
        unsigned v = 0;
        for (int r = (8 * tid) / 12; r < a.levels && 12 * r < 8 * tid + 8; ++r) {
            const unsigned pr = (unsigned)(chosen[r] / K) | (unsigned)(chosen[r] % K) << 6;
            const int sh = 12 * r - 8 * tid;
            v |= sh >= 0 ? pr << sh : pr >> -sh;
        }
        dst[tid] = (uint8_t)(v & 0xffu);
    }
}

}  // namespace

namespace {

// What is encoded: the keys (the configured key format) or the values (always index form, m_val codebooks).
struct EncodeWhat {
    bool paired;
    int levels, K, rec;
};
EncodeWhat encode_what(const commvq_config &c, bool values)
{
    EncodeWhat w;
    w.paired = !values && c.key_format == COMMVQ_KEYS_PAIRED;
    w.levels = values ? c.m_val : w.paired ? c.key_levels : c.m_key;
    w.K = w.paired ? 64 : kK;
    w.rec = w.paired ? (12 * w.levels + 7) / 8 : w.levels;
    return w;
}

commvq_status encoder_table_bytes(const commvq_handle *h, bool values, size_t *bytes)
{
    if (!h || !bytes) return COMMVQ_ERR_NULL;
    const EncodeWhat w = encode_what(h->cfg, values);
    *bytes = (size_t)h->cfg.n_kv_heads * w.levels * w.K * sizeof(float) * (w.paired ? 1 + w.K : 1);
    return COMMVQ_OK;
}

commvq_status encoder_prepare(commvq_handle *h, bool values, const void *cb, void *tables, void *stream)
{
    if (!h || !cb || !tables) return COMMVQ_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(tables) & 15u) return COMMVQ_ERR_SHAPE;
    if (h->device < 0) return COMMVQ_ERR_NO_DEVICE;
    const commvq_config &c = h->cfg;
    const EncodeWhat w = encode_what(c, values);
    const int rows = c.n_kv_heads * w.levels * w.K;
    float *norms = static_cast<float *>(tables), *cross = norms + rows;
    const size_t n = w.paired ? (size_t)rows * w.K : (size_t)rows;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (c.codebook_dtype == COMMVQ_BF16)
        hipLaunchKernelGGL(k_encode_tables<true>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, cb, norms, cross, rows, w.K, w.paired ? 1 : 0);
    else
        hipLaunchKernelGGL(k_encode_tables<false>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, cb, norms, cross, rows, w.K, w.paired ? 1 : 0);
    return hipGetLastError() == hipSuccess ? COMMVQ_OK : COMMVQ_ERR_LAUNCH;
}

commvq_status encode_vectors(commvq_handle *h, bool values, const void *keys, int32_t n_tokens, const void *key_cb, const void *tables,
                             uint8_t *codes_out, int64_t token_stride, int64_t head_stride, void *stream)
{
    if (!h || !keys || !key_cb || !tables || !codes_out) return COMMVQ_ERR_NULL;
    const commvq_config &c = h->cfg;
    const EncodeWhat w = encode_what(c, values);
    const bool paired = w.paired;
    const int levels = w.levels, K = w.K, rec = w.rec;
    if (n_tokens < 1 || (int64_t)n_tokens * c.n_kv_heads > (int64_t)1 << 30) return COMMVQ_ERR_SHAPE;
    if (head_stride < rec || token_stride < rec) return COMMVQ_ERR_SHAPE;  // records must not overlap
    if ((reinterpret_cast<uintptr_t>(tables) | reinterpret_cast<uintptr_t>(keys) | reinterpret_cast<uintptr_t>(key_cb)) & 15u)
        return COMMVQ_ERR_SHAPE;
    EncodeDims d;
    d.Hkv = c.n_kv_heads; d.levels = levels; d.K = K; d.key_bf16 = c.q_dtype == COMMVQ_BF16; d.record_bytes = rec;
    d.token_stride = token_stride; d.head_stride = head_stride;
    const int rows = c.n_kv_heads * levels * K;
    const float *norms = static_cast<const float *>(tables), *cross = norms + rows;
    const dim3 grid((unsigned)(n_tokens * c.n_kv_heads));
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool bf16 = c.codebook_dtype == COMMVQ_BF16;
    if (paired && !bf16) return COMMVQ_ERR_CONFIG;
    if (h->device < 0) return COMMVQ_ERR_NO_DEVICE;
    if (paired && n_tokens >= kEbTokens) {  // many tokens: 64 per workgroup, dot products on the matrix cores
        static std::atomic<uint64_t> lds_ok{0};
        if (allow_dynamic_lds(&k_encode_pair_batch, kEpLds, lds_ok) != hipSuccess) return COMMVQ_ERR_LAUNCH;
        const dim3 bgrid((unsigned)((n_tokens + kEbTokens - 1) / kEbTokens * c.n_kv_heads));
        hipLaunchKernelGGL(k_encode_pair_batch, bgrid, dim3(256), kEpLds, s, keys, static_cast<const uint4 *>(key_cb), norms, cross,
                           codes_out, d, n_tokens);
    } else if (paired) {  // rows, norms and cross terms staged in LDS, next level prefetched
        const int lds = (2 * K * kEncRowDw + 2 * K * K + 2 * K + kD + 256 + 8 + 32) * 4;
        static std::atomic<uint64_t> lds_ok{0};
        if (allow_dynamic_lds(&k_encode_lds<true>, lds, lds_ok) != hipSuccess) return COMMVQ_ERR_LAUNCH;
        hipLaunchKernelGGL(k_encode_lds<true>, grid, dim3(256), lds, s, keys, static_cast<const unsigned *>(key_cb), norms, cross, codes_out, d);
    } else if (bf16 && n_tokens >= kEbTokens) {  // many tokens: rows staged once per 64 tokens, dot products on the matrix cores
        static std::atomic<uint64_t> lds_ok{0};
        if (allow_dynamic_lds(&k_encode_batch, kEbLds, lds_ok) != hipSuccess) return COMMVQ_ERR_LAUNCH;
        const dim3 bgrid((unsigned)((n_tokens + kEbTokens - 1) / kEbTokens * c.n_kv_heads));
        hipLaunchKernelGGL(k_encode_batch, bgrid, dim3(256), kEbLds, s, keys, static_cast<const uint4 *>(key_cb), norms, codes_out, d,
                           n_tokens);
    } else if (bf16) {  // few tokens: next level's rows on their way into LDS while this level is searched
        static std::atomic<uint64_t> lds_ok{0};
        if (allow_dynamic_lds(&k_encode_dma, kEdLds, lds_ok) != hipSuccess) return COMMVQ_ERR_LAUNCH;
        hipLaunchKernelGGL(k_encode_dma, grid, dim3(256), kEdLds, s, keys, static_cast<const uint4 *>(key_cb), norms, codes_out, d);
    } else {
        hipLaunchKernelGGL(k_encode<false>, grid, dim3(256), 0, s, keys, key_cb, norms, codes_out, d);
    }
    return hipGetLastError() == hipSuccess ? COMMVQ_OK : COMMVQ_ERR_LAUNCH;
}

}  // namespace

extern "C" {

commvq_status commvq_encoder_table_bytes(const commvq_handle *h, size_t *bytes) { return encoder_table_bytes(h, false, bytes); }
// a free binary value code has no greedy stand-in here: its only producer is the trained encoder of Sec. 4.1
static bool binary_values(const commvq_handle *h) { return h && h->cfg.value_format == COMMVQ_VALUES_BINARY; }

commvq_status commvq_value_encoder_table_bytes(const commvq_handle *h, size_t *bytes)
{
    if (binary_values(h)) return COMMVQ_ERR_CONFIG;
    return encoder_table_bytes(h, true, bytes);
}

commvq_status commvq_encoder_prepare(commvq_handle *h, const void *key_cb, void *tables, void *stream)
{
    return encoder_prepare(h, false, key_cb, tables, stream);
}
commvq_status commvq_value_encoder_prepare(commvq_handle *h, const void *val_cb, void *tables, void *stream)
{
    if (binary_values(h)) return COMMVQ_ERR_CONFIG;
    return encoder_prepare(h, true, val_cb, tables, stream);
}

commvq_status commvq_encode_keys(commvq_handle *h, const void *keys, int32_t n_tokens, const void *key_cb, const void *tables,
                                 uint8_t *codes_out, int64_t token_stride, int64_t head_stride, void *stream)
{
    return encode_vectors(h, false, keys, n_tokens, key_cb, tables, codes_out, token_stride, head_stride, stream);
}
commvq_status commvq_encode_values(commvq_handle *h, const void *values, int32_t n_tokens, const void *val_cb, const void *tables,
                                   uint8_t *codes_out, int64_t token_stride, int64_t head_stride, void *stream)
{
    if (binary_values(h)) return COMMVQ_ERR_CONFIG;
    return encode_vectors(h, true, values, n_tokens, val_cb, tables, codes_out, token_stride, head_stride, stream);
}

}  // extern "C"
