// Value stage of libcommvq for the paper's own value code (Sec. 4.1): a token's whole value vector -- all KV heads
// side by side -- is encoded as a binary sequence s of N_c bits with any number of ones and decodes to s C_V
// (Eq. vanilla_decode).  Eq. optimized_v evaluates attention as (Softmax(A) S_V) C_V; with a free binary S_V the first
// product is a dense matrix product over the context,
//     bins[h][c] = sum_i w[h][i] * S_V[i][c]        (all query heads h x all N_c code bits c),
// and runs on the matrix cores (k_vbits).  Its result has the same form as the bins of the index-form value stage, so
// the second product (bins x C_V, k_out / k_out_mfma / k_out_final in commvq.hip) is shared.
#include "commvq_internal.hpp"
#include "commvq_vbits.hpp"

namespace {

constexpr int kVbThreads = 512;                // 8 wavefronts: each takes 128 of the workgroup's 1024 code bits
constexpr int kVbStage = 128;                  // tokens per LDS stage = two 64-token steps of the matrix instruction
constexpr int kVbSRows = kVbitsCols / 32;      // record dwords of a workgroup
constexpr int kVbSStride = kVbStage + 4;       // dwords per row of the transposed bit stage (rows 16-byte aligned)
constexpr int kVbAStride = kVbStage / 4 + 8;   // dwords per (digit, head) row of the weight stage: 10 bank columns of 16 bytes, so that
                                               // the lanes a 16-byte LDS read serves together (l % 8, (l / 16) % 2) fall on 16 different columns
typedef int intx4_t __attribute__((ext_vector_type(4)));
typedef float f4u_t __attribute__((ext_vector_type(4), aligned(4)));  // four floats at any 4-byte boundary

// One workgroup = (sequence, token range, 16 query heads, 1024 code bits).
//
// Exactness.  As in the index-form value stage the weights are added in fixed point: w = exp(logit - max) is taken
// as the integer W = round(w 2^S), with S chosen from the known exp-sum of the range so that the sum of all W stays
// below 2^30.  W + 0x80808080 has the bytes u'_k with W = sum_k (u'_k - 128) 256^k: four signed 8-bit digits, which
// is what v_mfma_i32_16x16x64_i8 multiplies.  The code bits enter as the bytes 2^p in pass p (a mask on the record byte
// instead of a shift per bit; 2^7 reads as -128), the four digit sums are integers in 32-bit accumulators (|digit| x 128 x
// tokens of a range <= 2^30), and sum_k (acc_k / +-2^p) 256^k modulo 2^32 is the exact integer sum_i W_i S_V[i][c] whatever
// the order of additions: results are bit-reproducible and carry a rounding error below (tokens of the range) x 2^-30 of
// its weight.
//
// Data flow per stage of 128 tokens: the records' 128 bytes that hold the workgroup's code bits are loaded coalesced and
// written to LDS transposed ([dword of the record][token]); the 16 x 128 logits become digit bytes (one 4 x 4 byte
// transpose per thread: one digit of four consecutive tokens per dword) in LDS [digit][head][token].  A wavefront then
// reads, per 64-token step, one record dword for 16 tokens per lane (lane n of a 16-lane row: dword n / 4 of the
// wavefront's four, byte n % 4), picks its byte with two byte permutes per token quad, and issues 8 passes (one record
// bit each, the same for all lanes: a constant mask) x 4 digits matrix instructions over them.  The global loads run two
// stages ahead.
__global__ __launch_bounds__(kVbThreads) void k_vbits(VbitsArgs a)
{
    __shared__ __attribute__((aligned(16))) unsigned s_lds[2][kVbSRows * kVbSStride];
    __shared__ __attribute__((aligned(16))) unsigned a_lds[2][4 * kVbitsHeads * kVbAStride];
    __shared__ float eoff_s[kVbitsHeads];

    const int ncg = a.Nc / kVbitsCols;
    const int nhg = (a.Hq + kVbitsHeads - 1) / kVbitsHeads;
    // The head groups (and column groups) of one token range read the same records and logits.  Workgroups go to the
    // chip's eight L2 domains round robin by index, so the group is the SLOW index: with a multiple of eight ranges the
    // readers of a range share one L2 and the second read of a line is a hit there.
    const int nrange = (int)gridDim.x / (ncg * nhg);
    const int id = blockIdx.x % nrange, grp = blockIdx.x / nrange;
    const int hg = grp % nhg, cg = grp / nhg;
    const int vs = id % a.nvsplit;
    const int b = id / a.nvsplit;
    const int cu0 = a.cu[b];
    const int L = a.cu[b + 1] - cu0;
    const int v0 = vs * a.vsplit_len;
    if (v0 >= L) return;
    const int v1 = min(v0 + a.vsplit_len, L);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int h0 = hg * kVbitsHeads;

    const int NB = a.Nc / 8;
    const uint8_t *rec = a.val_bits + (size_t)cu0 * NB + cg * (kVbitsCols / 8);
    const float *srow = a.scores + (size_t)cu0 * a.Hq;
    // bit stage: two (token, 16-byte piece of the record part) items per thread; weight stage: one (head, token quad)
    const int wh = tid >> 5, wq = tid & 31;
    // two sets of staging registers: a stage's loads are requested two stages ahead (one compute phase does not cover
    // the latency of memory)
    uint4 sreg2[2][2];
    float wreg2[2][4];
    auto fetch = [&](int t0, int set) {
        uint4(&sreg)[2] = sreg2[set];
        float(&wreg)[4] = wreg2[set];
        if (t0 + kVbStage <= v1 && h0 + kVbitsHeads <= a.Hq) {  // (uniform) a whole stage: no bounds to watch
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int it = tid + kVbThreads * u;
                sreg[u] = *reinterpret_cast<const uint4 *>(rec + (size_t)(t0 + (it >> 3)) * NB + 16 * (it & 7));
            }
            // (a logit row starts wherever the previous one ended: 4-byte alignment is all that is known)
            const f4u_t v = *reinterpret_cast<const f4u_t *>(srow + (size_t)(h0 + wh) * L + t0 + 4 * wq);
            wreg[0] = v.x; wreg[1] = v.y; wreg[2] = v.z; wreg[3] = v.w;
            return;
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int it = tid + kVbThreads * u, t = t0 + (it >> 3);
            sreg[u] = t < v1 ? *reinterpret_cast<const uint4 *>(rec + (size_t)t * NB + 16 * (it & 7)) : make_uint4(0u, 0u, 0u, 0u);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int ti = t0 + 4 * wq + j;
            wreg[j] = (h0 + wh < a.Hq && ti < v1) ? srow[(size_t)(h0 + wh) * L + ti] : -INFINITY;  // exp -> 0: no weight
        }
    };
    fetch(v0, 0);
    if (v0 + kVbStage < v1) fetch(v0 + kVbStage, 1);

    // Statistics, per head as in the index-form stage: the sequence maximum, the exp-sum of the score tiles that the range
    // touches (bounds every bin, fixes the fixed-point unit), and the exp-sum of the tiles that begin inside the range
    // (what it reports towards the softmax denominator).
    constexpr int HPW = kVbitsHeads / (kVbThreads / 64);  // heads per wavefront
    const int ns = min((L + a.split_len - 1) / a.split_len, a.nsplit);
    float2 first[HPW];  // the first 64 tiles' statistics of every head, requested together
#pragma unroll
    for (int u = 0; u < HPW; ++u) {
        const int h = h0 + wave + (kVbThreads / 64) * u;
        first[u] = (h < a.Hq && lane < ns) ? a.sstat[((size_t)b * a.Hq + h) * a.nsplit + lane] : make_float2(-INFINITY, 0.f);
    }
#pragma unroll
    for (int u = 0; u < HPW; ++u) {
        const int hl = wave + (kVbThreads / 64) * u, h = h0 + hl;
        if (h >= a.Hq) {
            if (lane == 0) eoff_s[hl] = 0.f;
            continue;
        }
        const float2 *st = a.sstat + ((size_t)b * a.Hq + h) * a.nsplit;
        float mx = first[u].x;
        for (int s = lane + 64; s < ns; s += 64) mx = fmaxf(mx, st[s].x);
        mx = wave_max(mx);
        const int sa = v0 / a.split_len, sb = min((v1 + a.split_len - 1) / a.split_len, ns);
        float l = 0.f, lown = 0.f;
        if (lane >= sa && lane < sb) {
            l = first[u].y * __builtin_amdgcn_exp2f((first[u].x - mx) * kLog2e);
            if (lane * a.split_len >= v0) lown = l;
        }
        for (int s = lane + 64; s < sb; s += 64)
            if (s >= sa) {
                const float t = st[s].y * __builtin_amdgcn_exp2f((st[s].x - mx) * kLog2e);
                l += t;
                if (s * a.split_len >= v0) lown += t;
            }
        l = wave_sum(l);
        lown = wave_sum(lown);
        int S = 0;
        if (l >= 1e-30f) S = min(29 - ilogbf(l), 120);
        if (lane == 0) {
            eoff_s[hl] = (float)S - mx * kLog2e;
            if (cg == 0) {
                a.vscale[((size_t)b * a.Hq + h) * a.nvsplit + vs] = ldexpf(1.f, -S);
                a.lsum[((size_t)b * a.Hq + h) * a.nvsplit + vs] = lown;
            }
        }
    }
    __syncthreads();

    auto stage_write = [&](int buf, int set) {
        unsigned *sd = s_lds[buf];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int it = tid + kVbThreads * u, tt = it >> 3, jq = it & 7;
            const uint4 sreg = sreg2[set][u];
            sd[(4 * jq + 0) * kVbSStride + tt] = sreg.x;
            sd[(4 * jq + 1) * kVbSStride + tt] = sreg.y;
            sd[(4 * jq + 2) * kVbSStride + tt] = sreg.z;
            sd[(4 * jq + 3) * kVbSStride + tt] = sreg.w;
        }
        unsigned *ad = a_lds[buf];
        const float eo = eoff_s[wh];
        unsigned wp[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const unsigned W = (unsigned)(__builtin_amdgcn_exp2f(wreg2[set][j] * kLog2e + eo) + 0.5f);
            wp[j] = (W + 0x80808080u) ^ 0x80808080u;  // bytes = signed digits
        }
        // 4 x 4 byte transpose: digit k of the four tokens in one dword
        const unsigned lo01 = __builtin_amdgcn_perm(wp[1], wp[0], 0x05010400u), hi01 = __builtin_amdgcn_perm(wp[1], wp[0], 0x07030602u);
        const unsigned lo23 = __builtin_amdgcn_perm(wp[3], wp[2], 0x05010400u), hi23 = __builtin_amdgcn_perm(wp[3], wp[2], 0x07030602u);
        ad[(0 * kVbitsHeads + wh) * kVbAStride + wq] = __builtin_amdgcn_perm(lo23, lo01, 0x05040100u);
        ad[(1 * kVbitsHeads + wh) * kVbAStride + wq] = __builtin_amdgcn_perm(lo23, lo01, 0x07060302u);
        ad[(2 * kVbitsHeads + wh) * kVbAStride + wq] = __builtin_amdgcn_perm(hi23, hi01, 0x05040100u);
        ad[(3 * kVbitsHeads + wh) * kVbAStride + wq] = __builtin_amdgcn_perm(hi23, hi01, 0x07060302u);
    };

    const int n = lane & 15, q = lane >> 4;
    const unsigned bn = (unsigned)n & 3u;
    const unsigned sel01 = 0x0c0c0000u | ((4u + bn) << 8) | bn;           // byte bn of two dwords -> bytes 0, 1
    const unsigned sel23 = ((4u + bn) << 24) | (bn << 16) | 0x00000c0cu;  // ... -> bytes 2, 3
    intx4_t acc[4][8];
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int p = 0; p < 8; ++p) acc[k][p] = intx4_t{0, 0, 0, 0};

    auto compute = [&](int buf) {
        const unsigned *sd = s_lds[buf] + (4 * wave + (n >> 2)) * kVbSStride;
        const unsigned *ad = a_lds[buf];
#pragma unroll
        for (int kb = 0; kb < kVbStage / 64; ++kb) {
            unsigned Y[4];  // byte j = the lane's record byte of token 4 r + j
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const uint4 X = *reinterpret_cast<const uint4 *>(sd + 64 * kb + 16 * q + 4 * r);
                Y[r] = __builtin_amdgcn_perm(X.y, X.x, sel01) | __builtin_amdgcn_perm(X.w, X.z, sel23);
            }
            intx4_t A[4];
#pragma unroll
            for (int k = 0; k < 4; ++k)
                A[k] = *reinterpret_cast<const intx4_t *>(ad + (k * kVbitsHeads + n) * kVbAStride + 16 * kb + 4 * q);
#pragma unroll
            for (int p = 0; p < 8; ++p) {
                const unsigned mask = 0x01010101u << p;
                const intx4_t B = {(int)(Y[0] & mask), (int)(Y[1] & mask), (int)(Y[2] & mask), (int)(Y[3] & mask)};
#pragma unroll
                for (int k = 0; k < 4; ++k) acc[k][p] = __builtin_amdgcn_mfma_i32_16x16x64_i8(A[k], B, acc[k][p], 0, 0, 0);
            }
        }
    };

    stage_write(0, 0);
    __syncthreads();
    // iteration of stage s (buffer and register set s % 2): request stage s + 2, multiply stage s, stage s + 1 to LDS
    auto iteration = [&](int t0, int par) {
        if (t0 + 2 * kVbStage < v1) fetch(t0 + 2 * kVbStage, par);  // (all conditions uniform over the workgroup)
        compute(par);
        if (t0 + kVbStage < v1) stage_write(par ^ 1, par ^ 1);
        __syncthreads();
    };
    for (int t0 = v0; t0 < v1; t0 += 2 * kVbStage) {
        iteration(t0, 0);
        if (t0 + kVbStage < v1) iteration(t0 + kVbStage, 1);
    }

    // digits -> integer bins [Nc rows][G] per (sequence, KV head, range); row 128 W + 16 p + n for the wavefront's W-th
    // run of 128 code bits (vbits_code_bit gives the code bit of a row): the 16 lanes of a pass store 16 consecutive rows
#pragma unroll
    for (int p = 0; p < 8; ++p) {
        const size_t row = (size_t)(128 * (cg * (kVbitsCols / 128) + wave) + 16 * p + n);
        unsigned val[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            // sum_k (acc_k / 2^p) 256^k modulo 2^32; every acc_k is a multiple of 2^p (pass 7 multiplied by -2^7)
            unsigned tot = (unsigned)(acc[0][p][i] >> p);
#pragma unroll
            for (int k = 1; k < 4; ++k) tot += (unsigned)acc[k][p][i] << (8 * k - p);
            val[i] = p == 7 ? 0u - tot : tot;
        }
        const int h = h0 + 4 * q;  // heads h .. h + 3
        if ((a.G & 3) == 0) {
            if (h < a.Hq) {
                const int g = h / a.G, hh = h % a.G;
                unsigned *dst = a.bins + ((size_t)(b * a.Hkv + g) * a.nvsplit + vs) * ((size_t)a.G * a.Nc) + row * a.G + hh;
                *reinterpret_cast<uint4 *>(dst) = make_uint4(val[0], val[1], val[2], val[3]);
            }
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (h + i < a.Hq) {
                    const int g = (h + i) / a.G, hh = (h + i) % a.G;
                    a.bins[((size_t)(b * a.Hkv + g) * a.nvsplit + vs) * ((size_t)a.G * a.Nc) + row * a.G + hh] = val[i];
                }
        }
    }
}

}  // namespace

hipError_t commvq_launch_vbits(const VbitsArgs &a, hipStream_t stream)
{
    const int ncg = a.Nc / kVbitsCols, nhg = (a.Hq + kVbitsHeads - 1) / kVbitsHeads;
    const unsigned grid = (unsigned)a.batch * (unsigned)a.nvsplit * (unsigned)nhg * (unsigned)ncg;
    hipLaunchKernelGGL(k_vbits, dim3(grid), dim3(kVbThreads), 0, stream, a);
    return hipGetLastError();
}
