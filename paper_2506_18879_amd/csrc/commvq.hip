// libcommvq: decode attention over a CommVQ-compressed KV cache, hand-written for gfx950.
//
// Pipeline of one call (all on the caller's stream):
//   score stage Eq. new_attention: per (token, KV head) gather-sum the M_k selected key
//               codewords, rotate once by the RoPE matrix of the relative position, contract
//               with the G query heads of the group -> scaled logits + per-split (max, sum exp).
//               bf16 codebooks with contiguous key positions: k_prep (codebook re-laid in
//               LDS-image order) + k_score_mfma (codebook slices streamed through LDS, tile codes
//               resident in registers, gather-sum and query contraction on the matrix cores), for
//               short contexts with the tiles also cut along the slices + k_score_combine;
//               fp32 codebooks or explicit key positions: k_score (rows gathered through L1).
//   k_bins      Softmax(A) S_V of Eq. optimized_v (unnormalised): exp(logit - max) is
//               scatter-added into LDS bins (one per head, value codebook and codeword; written out
//               as [K][M_v][G]), one bin set per context split.  The
//               bins are 32-bit fixed point (integer LDS atomics run ~20x faster than fp32 ones
//               on gfx950); the scale of each split is chosen from its known exp-sum so that
//               no bin can overflow and the worst-case error is (tokens per split) * 2^-31.
//   k_out       (bins C_V): split reduction + bins x value-codebook product, per chunk of rows.
//   k_out_final sum of the per-chunk products, division by the softmax denominator.
// Key encoding for cache append lives in commvq_encode.hip, the EM codebook learner in commvq_em.hip.
//
// RoPE algebra used by k_score (Sec. 3.2, Eq. rope_ri).  Writing a 2-D sub-vector (x, y) as
// z = x + iy, the paper's row-vector product (x, y) R_m^j is z * exp(-i m theta_j).  The dot
// product of two sub-vectors is Re(a conj(b)), so
//     (q^j R_t^j) . (k^j R_p^j) = Re( q^j conj(k^j) exp(-i (t - p) theta_j) ),
// i.e. only the relative position t - p enters, and the rotation can be applied to the
// gather-summed codewords once per token (commutativity, Property 1).
#include <algorithm>
#include <cstring>

#include "commvq_internal.hpp"
#include "commvq_vbits.hpp"

// Scratch memory of commvq_decode_attn_static: the workspace of a call, held by the library itself so that the
// entry point allocates nothing.  One copy per GPU the library is loaded on, for the life of the process.  In host
// code this name is only a stand-in for the symbol: the device address is looked up once per device in
// commvq_create (hipGetSymbolAddress) and kept in the handle; kernels receive that pointer.
constexpr size_t kStaticScratchBytes = (size_t)48 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

struct Workspace {
    float *scores;    // [T * Hq] scaled logits
    float2 *sstat;    // [B * Hq * score_splits] (max, sum of exp(logit - max)) of each score split
    float *vscale;    // [B * Hq * value_splits] 2^-S: value of one fixed-point unit of that split's bins
    float *lsum;      // [B * Hq * value_splits] sum of exp(logit - sequence max) over the score tiles that begin in that value split
    unsigned *bins;   // [B * Hkv * value_splits][K][Mv][G] fixed-point bins (codeword-major: see k_bins)
    float *partial;   // [B * Hq * out_chunks][d]
    uint4 *packed;    // key codebook re-laid slice-major for k_score_mfma / k_score_pair
    uint8_t *pair_bytes;  // paired-code keys: one byte per index, [T * Hkv][32 * blocks]
    float *lut;           // position-free keys: scale * q . C, [B * Hkv][M_k * K][G]
    float *scores_part;   // [slice groups][T * Hq] partial logits when the score tiles are also cut along the slices
    uint4 *packed_val;    // value codebook re-laid for k_out_mfma (batches; only if the caller has not packed it)
    size_t bytes;
};

// The slice-streaming score kernel (k_score_mfma) serves bf16 codebooks with contiguous positions; everything else
// (fp32 codebooks, explicit key positions) goes through the gather kernel.
bool use_sliced(const commvq_handle *h, bool explicit_positions)
{
    if (h->cfg.position_free) return true;  // scalar look-up table kernel: same tiling, positions play no role
    return h->cfg.codebook_dtype == COMMVQ_BF16 && !explicit_positions;
}

// The batched output kernel (value codebook on the matrix cores) serves bf16 codebooks from 16 output rows
// (sequences x query heads of a KV head) on.
inline bool use_out_mfma(const commvq_handle *h, int batch)
{
    return h->cfg.codebook_dtype == COMMVQ_BF16 && batch * h->G >= kOutMfmaMinRows;
}

// Binary value code: N_c code bits per token for all KV heads, one codebook [N_c][Hkv * d].  Towards the output kernels a
// KV head's N_c bins stand in for N_c / 256 value codebooks of 256 rows; bins row r is code bit vbits_code_bit(r).
inline bool bin_values(const commvq_config &c) { return c.value_format == COMMVQ_VALUES_BINARY; }
inline int val_books(const commvq_config &c) { return bin_values(c) ? c.value_bits / kK : c.m_val; }

// Paired-code key format: blocks of 16 levels, bytes of one packed record, bytes of the unpacked indices of a token.
inline bool pair_keys(const commvq_config &c) { return c.key_format == COMMVQ_KEYS_PAIRED; }
inline int pair_blocks(const commvq_config &c) { return (c.key_levels + 15) / 16; }
inline int pair_record_bytes(const commvq_config &c) { return (12 * c.key_levels + 7) / 8; }
inline size_t packed_key_bytes(const commvq_config &c)
{
    if (pair_keys(c)) return (size_t)c.n_kv_heads * 16 * pair_blocks(c) * 64 * 256;  // 16 planes x blocks x 16 KiB
    return (size_t)c.n_kv_heads * c.m_key * kK * kD * 2;
}

void make_plan(const commvq_handle *h, int B, int max_seqlen, bool sliced, commvq_plan *p)
{
    const int units = B * h->cfg.n_kv_heads;
    int len, groups = 1;
    if (sliced) {
        // Tile = 1024, 2048 or 4096 tokens of one (sequence, KV head); a context too short to fill the 256 compute
        // units with such tiles is also cut along the codebook slices, `groups` workgroups per tile that each stream
        // S / groups slices and leave partial logits for k_score_combine to add.  Cost model of a workgroup, in
        // microseconds as measured on the five configurations: a fixed start (first fetches, write-out), per slice a
        // switch (LDS refill, barriers) and the passes themselves.
        const bool splittable = !pair_keys(h->cfg) && !h->cfg.position_free;
        const int S = pair_keys(h->cfg) ? 4 : h->cfg.m_key / 2;                       // slices per tile
        const double c1024 = h->cfg.m_key == 16 && !pair_keys(h->cfg) ? 2.1 : 1.85;  // passes of 1024 tokens over one slice
        double best = 1e30;
        len = 1024;
        groups = 1;
        for (int tpt = 1; tpt <= kScoreMaxTpt; tpt *= 2) {
            if (tpt == 4 && h->G == 8 && (h->cfg.m_key == 16 || pair_keys(h->cfg))) break;  // those instantiations run out of registers
            for (int e = 1; e <= (splittable ? S : 1); e *= 2) {
                const long wgs = (long)units * ((max_seqlen + 1024 * tpt - 1) / (1024 * tpt)) * e;
                // cut along the slices: every group fetches the tile's codes again, the partial logits take a trip through
                // memory, and k_score_combine is one more launch
                const double t = (double)((wgs + 255) / 256) * (9.0 + (double)(S / e) * (1.3 + tpt * c1024)) + (e > 1 ? 12.0 : 0.0);
                if (t < best * 0.9999) { best = t; len = 1024 * tpt; groups = e; }
            }
        }
    } else {
        len = 1024;
        // down to 4 tokens per wavefront (one iteration of four tokens): a short context still spreads over the chip
        while (len > 16 && (long)units * ((max_seqlen + len - 1) / len) < kScoreMinWgs) len /= 2;
    }
    p->score_split_len = len;
    p->score_splits = (max_seqlen + len - 1) / len;
    int nv = 256 / units;  // about one value workgroup per compute unit
    if (bin_values(h->cfg))  // a workgroup of the binary-code value kernel: 16 query heads x 1024 code bits of one token range
        nv = 256 / (B * ((h->cfg.n_q_heads + kVbitsHeads - 1) / kVbitsHeads) * (h->cfg.value_bits / kVbitsCols));
    if (nv < 1) nv = 1;
    int vlen = (max_seqlen + nv - 1) / nv;
    // a value split is a whole number of statistics tiles (score tiles; 1024 tokens when k_score_combine writes the
    // statistics), or a power-of-two fraction of one (never less than 1024 tokens): k_bins takes its exp-sums from them
    const int slen = groups > 1 ? 1024 : len;
    if (vlen >= slen || slen <= 1024) {
        const int round_to = slen > 1024 ? slen : 1024;
        vlen = (vlen + round_to - 1) / round_to * round_to;
    } else {
        int part = 1024;
        while (part < vlen) part *= 2;
        vlen = part;  // 1024 or 2048 inside a 2048- or 4096-token tile
    }
    // the binary-code value kernel sums signed digit x bit products in 32-bit accumulators: |digit| <= 2^7, |bit byte| <= 2^7,
    // so a range of at most 2^16 tokens stays within 2^30
    if (bin_values(h->cfg) && vlen > (1 << 16)) vlen = 1 << 16;
    p->value_split_len = vlen;
    p->value_splits = (max_seqlen + vlen - 1) / vlen;
    p->out_chunks = val_books(h->cfg) * kK / kOutRows;
    p->score_kernel = sliced ? 1 : 0;
    p->score_slice_groups = groups;
}

// Granularity of the (max, sum of exp) statistics that the score stage leaves for k_bins: the score tile, except that
// k_score_combine (tiles cut along the slices) writes them per 1024 tokens.
inline int stat_len(const commvq_plan &p) { return p.score_kernel && p.score_slice_groups > 1 ? 1024 : p.score_split_len; }
inline int stat_splits(const commvq_plan &p, int max_seqlen) { return (max_seqlen + stat_len(p) - 1) / stat_len(p); }

// Carves the workspace.  Array sizes are the larger of what the two score kernels need, so one
// workspace size serves a batch shape whether or not explicit positions are passed.
void carve(const commvq_handle *h, int B, int64_t T, int max_seqlen, void *base, Workspace *w)
{
    const commvq_config &c = h->cfg;
    commvq_plan pa, pb;
    make_plan(h, B, max_seqlen, true, &pa);
    make_plan(h, B, max_seqlen, false, &pb);
    const size_t ssplits = std::max<size_t>(std::max(pa.score_splits, pb.score_splits), (size_t)stat_splits(pa, max_seqlen));
    const size_t vsplits = pa.value_splits > pb.value_splits ? pa.value_splits : pb.value_splits;
    size_t off = 0;
    auto take = [&](size_t n_floats) {
        float *ptr = base ? reinterpret_cast<float *>(static_cast<char *>(base) + off) : nullptr;
        off += align_up(n_floats * sizeof(float), 256);
        return ptr;
    };
    w->scores = take((size_t)T * c.n_q_heads);
    w->sstat = reinterpret_cast<float2 *>(take((size_t)B * c.n_q_heads * ssplits * 2));
    w->vscale = take((size_t)B * c.n_q_heads * vsplits);
    w->lsum = take((size_t)B * c.n_q_heads * vsplits);
    w->bins = reinterpret_cast<unsigned *>(take((size_t)B * c.n_kv_heads * vsplits * h->G * val_books(c) * kK));
    w->partial = take((size_t)B * c.n_q_heads * pa.out_chunks * kD);
    w->packed = reinterpret_cast<uint4 *>(take(packed_key_bytes(c) / 4));
    w->pair_bytes = pair_keys(c) ? reinterpret_cast<uint8_t *>(take((size_t)T * c.n_kv_heads * 8 * pair_blocks(c))) : nullptr;
    w->lut = c.position_free ? take((size_t)B * c.n_q_heads * c.m_key * kK) : nullptr;
    w->scores_part = pa.score_slice_groups > 1 ? take((size_t)pa.score_slice_groups * T * c.n_q_heads) : nullptr;
    w->packed_val = use_out_mfma(h, B) ? reinterpret_cast<uint4 *>(take((size_t)c.n_kv_heads * val_books(c) * kK * kD * 2 / 4)) : nullptr;
    w->bytes = off;
}

// ------------------------------------------------------------------ k_score
struct ScoreDims {
    int Hq, Hkv, nsplit, split_len, n_hi, q_bf16;
    float scale;
};


// Raw buffer descriptor over [base, base + bytes): loads take a per-lane byte offset plus a
// wave-uniform (scalar) byte offset, and reads past the end return zero instead of faulting.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *base, unsigned bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00020000);
}

__device__ __forceinline__ float row_max16(float v)
{
    v = fmaxf(v, dpp_mov<0xB1>(v));
    v = fmaxf(v, dpp_mov<0x4E>(v));
    v = fmaxf(v, dpp_mov<0x141>(v));
    return fmaxf(v, dpp_mov<0x140>(v));
}

// Sum over each 16-lane row; every lane of the row receives the row total.
__device__ __forceinline__ float row_sum16(float v)
{
    v += dpp_mov<0xB1>(v);
    v += dpp_mov<0x4E>(v);
    v += dpp_mov<0x141>(v);
    return v + dpp_mov<0x140>(v);
}


// Score kernel.  A wavefront handles FOUR tokens per iteration, one per 16-lane row; lane
// `sub` of a row owns sub-spaces 4*sub .. 4*sub+3 (elements 8*sub .. 8*sub+7), i.e. 16 bytes of
// a bf16 codeword row, so one 16-byte-per-lane buffer load fetches four different codeword
// rows (1 KiB) per instruction: measured ~1.7x the bytes per clock of the one-row-per-
// instruction form, whose rate is bound by the L1's per-instruction cost.  The per-lane byte
// offset (code << 8 | sub * 16) is built by a single byte permute; the codebook index is the
// load's scalar offset.  The relative-position phase is split as 64 * hi + lo: E_hi is folded
// into the query registers (recomputed only when some lane's hi changes, every 64 tokens for
// contiguous positions), E_lo comes from a 32 KiB LDS table.  The dot products are reduced
// inside the 16-lane rows (4 DPP steps per head), parked for 16 iterations and written as
// one 256-byte run per head.  blockIdx.x % Hkv selects the KV head: consecutive workgroups
// go to consecutive XCDs, so with 8 KV heads each XCD's L2 serves one head's codebook.

template <int M, int G, bool BF16>
__global__ __launch_bounds__(kScoreThreads) void k_score(
    const void *__restrict__ q, const uint8_t *__restrict__ key_codes, const void *__restrict__ key_cb,
    const int32_t *__restrict__ cu, const int32_t *__restrict__ q_pos, const int32_t *__restrict__ key_pos,
    const float2 *__restrict__ tbl_hi, const float2 *__restrict__ tbl_lo, float *__restrict__ scores,
    float2 *__restrict__ sstat, const ScoreDims a)
{
    constexpr int CW = M / 4;
    constexpr unsigned ROWB = BF16 ? kD * 2 : kD * 4;
    // E_lo as two planes of float4: plane h, entry [lo][sub] = sub-spaces 4*sub+2h, 4*sub+2h+1
    __shared__ float4 lo_lds[2][kLo][16];
    __shared__ float2 wstat[kScoreThreads / 64][G];

    int id = blockIdx.x;
    const int g = id % a.Hkv;
    id /= a.Hkv;
    const int split = id % a.nsplit;
    const int b = id / a.nsplit;
    const int cu0 = cu[b];
    const int L = cu[b + 1] - cu0;
    const int s0 = split * a.split_len;
    if (s0 >= L) return;
    for (int x = threadIdx.x; x < 2 * kLo * 16; x += kScoreThreads) {
        const int h = x / (kLo * 16), lo = (x / 16) % kLo, sb = x % 16;
        const float2 e0 = tbl_lo[lo * kJ + 4 * sb + 2 * h], e1 = tbl_lo[lo * kJ + 4 * sb + 2 * h + 1];
        lo_lds[h][lo][sb] = make_float4(e0.x, e0.y, e1.x, e1.y);
    }
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int r = lane >> 4, sub = lane & 15;
    const int wlen = a.split_len / (kScoreThreads / 64);  // 4, 8, 16, 32 or a multiple of 64 tokens per wavefront
    const int t0 = s0 + wave * wlen;
    const int t1 = min(min(t0 + wlen, s0 + a.split_len), L);
    const int n_it = t1 > t0 ? (t1 - t0 + 3) / 4 : 0;
    const int qpos = q_pos[b];
    __syncthreads();

    const uint8_t *codes = key_codes + ((size_t)cu0 * a.Hkv + (size_t)g * L) * M;
    const __amdgpu_buffer_rsrc_t cb_rs =
        make_rsrc(static_cast<const char *>(key_cb) + (size_t)g * M * kK * ROWB, (unsigned)(M * kK) * ROWB);
    const __amdgpu_buffer_rsrc_t hi_rs = make_rsrc(tbl_hi, (unsigned)a.n_hi * kJ * 8u);
    float *srow = scores + (size_t)cu0 * a.Hq + (size_t)g * G * L;
    const size_t q_off = ((size_t)b * a.Hq + (size_t)g * G) * kD + 8 * sub;
    const unsigned sel_lo = opaque_sgpr(0x00003f80u), sel_hi = opaque_sgpr(0x3f800000u);
    const unsigned lane_off = BF16 ? sub * 16u : sub * 32u;

    float qr[G][8];  // queries of the group with E_hi folded in: (x, y) of this lane's 4 sub-spaces
#pragma unroll
    for (int hh = 0; hh < G; ++hh)
#pragma unroll
        for (int e = 0; e < 8; ++e) qr[hh][e] = 0.f;
    int cur_key = -1;  // per lane: (hi << 1 | negative) whose phase is folded into qr
    float keep[G], vmax[G], vsum[G];
#pragma unroll
    for (int hh = 0; hh < G; ++hh) { keep[hh] = 0.f; vmax[hh] = -INFINITY; vsum[hh] = 0.f; }

    // Codeword loads are issued in chunks of CH codebooks into two register buffers; the chunk
    // after the one being summed is always in flight (across iterations too), and the codes
    // are fetched two iterations ahead.
    constexpr int CH = BF16 ? 4 : 2;  // codebooks per chunk
    constexpr int LPC = BF16 ? CH : 2 * CH;                                  // 16-byte loads per chunk
    constexpr int NC = M / CH;
    static_assert(NC % 2 == 0, "buffer parity must repeat every iteration");
    uint4_t buf[2][LPC];
    unsigned cw[CW], cwn[CW];
    auto load_codes = [&](int i, unsigned(&dst)[CW]) {
        const uint4 *cp = reinterpret_cast<const uint4 *>(codes + (size_t)min(i + r, L - 1) * M);
#pragma unroll
        for (int v = 0; v < M / 16; ++v) {
            const uint4 c4 = cp[v];
            dst[4 * v + 0] = c4.x; dst[4 * v + 1] = c4.y; dst[4 * v + 2] = c4.z; dst[4 * v + 3] = c4.w;
        }
    };
    auto issue = [&](const unsigned(&c)[CW], int chunk, uint4_t(&dst)[LPC]) {
#pragma unroll
        for (int k = 0; k < CH; ++k) {
            const int m = chunk * CH + k;
            if (BF16) {
                // byte 1 <- code m, byte 0 <- sub * 16: (code << 8) | (sub * 16)
                const unsigned voff = __builtin_amdgcn_perm(c[m / 4], lane_off, 0x0c0c0000u | ((4u + (m % 4)) << 8));
                dst[k] = __builtin_amdgcn_raw_buffer_load_b128(cb_rs, voff, (unsigned)m * kK * ROWB, 0);
            } else {
                const unsigned voff = ((c[m / 4] >> (8 * (m % 4))) & 0xffu) * ROWB + lane_off;
                dst[2 * k] = __builtin_amdgcn_raw_buffer_load_b128(cb_rs, voff, (unsigned)m * kK * ROWB, 0);
                dst[2 * k + 1] = __builtin_amdgcn_raw_buffer_load_b128(cb_rs, voff + 16u, (unsigned)m * kK * ROWB, 0);
            }
        }
    };
    float A[8];
    auto consume = [&](const uint4_t(&src)[LPC]) {
#pragma unroll
        for (int k = 0; k < LPC; ++k)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const unsigned ve = src[k][e];
                if (BF16) {
                    A[2 * e] = add_bf16_sel(ve, sel_lo, A[2 * e]);
                    A[2 * e + 1] = add_bf16_sel(ve, sel_hi, A[2 * e + 1]);
                } else {
                    A[4 * (k & 1) + e] += __builtin_bit_cast(float, ve);
                }
            }
    };
    if (n_it > 0) {
        load_codes(t0, cw);
        issue(cw, 0, buf[0]);
        load_codes(t0 + 4, cwn);
    }

    for (int it = 0; it < n_it; ++it) {
        const int i = t0 + it * 4;
        // relative position of this row's token
        const int tok = min(i + r, L - 1);
        const int pos = key_pos ? key_pos[cu0 + tok] : tok;
        const int dl = qpos - pos;
        const int neg = dl < 0;
        const int ad = neg ? -dl : dl;
        const int hi = min(ad >> kLoBits, a.n_hi - 1);
        const int lo = ad & (kLo - 1);
        const int key = (hi << 1) | neg;
        if (__builtin_amdgcn_ballot_w64(key != cur_key) != 0) {
            // fold the coarse phase into the queries: q' = q conj(E_hi) for t >= p, q E_hi otherwise
            cur_key = key;
            float eh[8];
#pragma unroll
            for (int hf = 0; hf < 2; ++hf) {
                const uint4_t v = __builtin_amdgcn_raw_buffer_load_b128(hi_rs, (unsigned)hi * (kJ * 8u) + sub * 32u + 16u * hf, 0, 0);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const unsigned ve = v[e];
                    eh[4 * hf + e] = __builtin_bit_cast(float, ve);
                }
            }
#pragma unroll
            for (int hh = 0; hh < G; ++hh) {
                float qx[4], qy[4];
                if (a.q_bf16) {
                    const uint4 v = *reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(q) + q_off + (size_t)hh * kD);
                    const unsigned w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) { qx[e] = bf16_lo(w[e]) * a.scale; qy[e] = bf16_hi(w[e]) * a.scale; }
                } else {
                    const float4 *qp = reinterpret_cast<const float4 *>(static_cast<const float *>(q) + q_off + (size_t)hh * kD);
                    const float4 v0 = qp[0], v1 = qp[1];
                    qx[0] = v0.x * a.scale; qy[0] = v0.y * a.scale; qx[1] = v0.z * a.scale; qy[1] = v0.w * a.scale;
                    qx[2] = v1.x * a.scale; qy[2] = v1.y * a.scale; qx[3] = v1.z * a.scale; qy[3] = v1.w * a.scale;
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float hc = eh[2 * e], hs = neg ? -eh[2 * e + 1] : eh[2 * e + 1];
                    qr[hh][2 * e] = qx[e] * hc + qy[e] * hs;
                    qr[hh][2 * e + 1] = qy[e] * hc - qx[e] * hs;
                }
            }
        }
        // A = sum of the M selected codeword rows (Eq. commute_decode), this lane's 4 sub-spaces
#pragma unroll
        for (int e = 0; e < 8; ++e) A[e] = 0.f;
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            // (the last iteration issues one redundant, in-range chunk rather than branch)
            if (c + 1 < NC) issue(cw, c + 1, buf[(c + 1) & 1]);
            else issue(cwn, 0, buf[0]);
            __builtin_amdgcn_sched_barrier(0);
            consume(buf[c & 1]);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int v = 0; v < CW; ++v) cw[v] = cwn[v];
        load_codes(i + 8, cwn);  // token index is clamped to the sequence

        // B = A E_lo (conjugated for negative distances); score_h = sum_j Re(q'_h conj(B))
        const float4 l0 = lo_lds[0][lo][sub], l1 = lo_lds[1][lo][sub];
        const float ec[4] = {l0.x, l0.z, l1.x, l1.z};
        const float es[4] = {neg ? -l0.y : l0.y, neg ? -l0.w : l0.w, neg ? -l1.y : l1.y, neg ? -l1.w : l1.w};
        float Bx[4], By[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            Bx[e] = A[2 * e] * ec[e] - A[2 * e + 1] * es[e];
            By[e] = A[2 * e] * es[e] + A[2 * e + 1] * ec[e];
        }
        const bool mine = sub == (it & 15);
#pragma unroll
        for (int hh = 0; hh < G; ++hh) {
            float v = 0.f;
#pragma unroll
            for (int e = 0; e < 4; ++e) v += qr[hh][2 * e] * Bx[e] + qr[hh][2 * e + 1] * By[e];
            v = row_sum16(v);
            keep[hh] = mine ? v : keep[hh];
        }
        if ((it & 15) == 15 || it == n_it - 1) {  // flush: lane (r, sub) holds token 4 * sub + r of this 64-token block
            const int itc = (it & ~15) + sub;
            const int tk = t0 + itc * 4 + r;
            if (itc <= it && tk < t1) {
#pragma unroll
                for (int hh = 0; hh < G; ++hh) {
                    srow[(size_t)hh * L + tk] = keep[hh];
                    const float mn = fmaxf(vmax[hh], keep[hh]);
                    vsum[hh] = vsum[hh] * __builtin_amdgcn_exp2f((vmax[hh] - mn) * kLog2e) +
                               __builtin_amdgcn_exp2f((keep[hh] - mn) * kLog2e);
                    vmax[hh] = mn;
                }
            }
        }
    }

    // (max, sum exp) of the split: lanes -> waves -> one pair per head
#pragma unroll
    for (int hh = 0; hh < G; ++hh) {
        const float m = wave_max(vmax[hh]);
        const float l = wave_sum(vmax[hh] == -INFINITY ? 0.f : vsum[hh] * __builtin_amdgcn_exp2f((vmax[hh] - m) * kLog2e));
        if (lane == 0) wstat[wave][hh] = make_float2(m, l);
    }
    __syncthreads();
    if (threadIdx.x < G) {
        float m = -INFINITY;
        for (int w = 0; w < kScoreThreads / 64; ++w) m = fmaxf(m, wstat[w][threadIdx.x].x);
        float l = 0.f;
        for (int w = 0; w < kScoreThreads / 64; ++w) {
            const float2 st = wstat[w][threadIdx.x];
            if (st.x != -INFINITY) l += st.y * __builtin_amdgcn_exp2f((st.x - m) * kLog2e);
        }
        sstat[((size_t)b * a.Hq + (size_t)g * G + threadIdx.x) * a.nsplit + split] = make_float2(m, l);
    }
}

// ------------------------------------------------------------------ k_prep
constexpr int kSliceThreads = 1024;              // one workgroup per compute unit
constexpr int kSliceBytes = 128 * 1024;          // LDS bytes of one codebook slice
constexpr int kPhaseBytes = (4 * 64 + 4 * 65) * 16;  // LDS bytes of the slice's phase factors (at most)
constexpr int kStatBytes = (kSliceThreads / 64) * 8 * 8;  // per-wavefront (max, sum) of up to 8 heads
constexpr int kScoreLds = kSliceBytes + 2 * kPhaseBytes + kStatBytes;  // the phase factors are double-buffered

// Key codebook re-laid for k_score_mfma.
//   packed[g][s][blk][c][col] : 16-byte pieces (8 bf16).  Slice s holds elements DS*s .. DS*s + DS-1 of
//                        every codeword (DS = 256 / M, S = 128 / DS slices) as one contiguous 128 KiB
//                        image of two 64 KiB blocks of 256 rows (one per code value c) x 16 pieces:
//                        piece x = 16 blk + col with x = 16 * plane + m for M = 16 (plane = which 8 of
//                        the 16 elements) and x = m for M = 32.  A 256-byte row spans all 64 LDS banks,
//                        so a piece lives in bank column col whatever its code: lanes that read
//                        different columns never conflict.
// One thread per 16-byte piece of the source (coalesced reads).
__global__ __launch_bounds__(256) void k_prep(const uint4 *__restrict__ key_cb, uint4 *__restrict__ packed, int Hkv, int M)
{
    const int P = 32 / M;                       // planes: DS / 8 = (256 / M) / 8
    const size_t n_pieces = (size_t)Hkv * M * kK * 16;
    const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= n_pieces) return;
    const int piece = (int)(t & 15);            // 16 pieces of 8 elements per row
    const size_t row = t >> 4;                  // (g * M + m) * K + c
    const int g = (int)(row / ((size_t)M * kK));
    const int mc = (int)(row % ((size_t)M * kK));
    const int m = mc / kK, c = mc % kK;
    const int sl = piece / P, pl = piece % P;
    const int S = 16 / P;
    const int x = pl * 16 + m;                  // 0..31: block x / 16, bank column x % 16
    packed[((((size_t)g * S + sl) * 2 + x / 16) * kK + c) * 16 + x % 16] = key_cb[t];
}

struct SliceDims {
    int Hq, Hkv, nsplit, n_hi, q_bf16;
    float scale;
    int groups;            // workgroups per tile, each with S / groups of the codebook slices (k_score_mfma)
    long long part_stride; // floats between the partial logit arrays of two slice groups
};

// ------------------------------------------------------------------ k_score_mfma

// 16-byte LDS read at an absolute LDS byte address.  The score kernels keep their dynamic LDS at address 0
// (no static LDS), but the compiler only learns that after instruction selection: a read through the array's
// base costs one "add 0" per read.
typedef __attribute__((address_space(3))) const uint4_t *lds_u4_ptr;
__device__ __forceinline__ uint4_t lds_read_b128(unsigned byte_addr) { return *reinterpret_cast<lds_u4_ptr>(byte_addr); }

// Max / sum over the lanes of a wavefront that hold logits of the same query head in k_score_mfma:
// one 16-lane row (M = 16), or the two rows r and r + 2 (M = 32).
template <int M>
__device__ __forceinline__ float head_lanes_max(float v)
{
    v = row_max16(v);
    if (M == 16) return v;
    const unsigned u = __builtin_bit_cast(unsigned, v);
    auto r32 = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return fmaxf(__builtin_bit_cast(float, (unsigned)r32[0]), __builtin_bit_cast(float, (unsigned)r32[1]));
}
template <int M>
__device__ __forceinline__ float head_lanes_sum(float v)
{
    v = row_sum16(v);
    if (M == 16) return v;
    const unsigned u = __builtin_bit_cast(unsigned, v);
    auto r32 = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __builtin_bit_cast(float, (unsigned)r32[0]) + __builtin_bit_cast(float, (unsigned)r32[1]);
}
// x + y after exchanging the odd 16-lane rows of x with the even rows of y (row r of the result:
// r even: x[r] + x[r+1], r odd: y[r-1] + y[r]), and the same with 32-lane halves.
__device__ __forceinline__ float swap16_add(float x, float y)
{
    auto r = __builtin_amdgcn_permlane16_swap(__builtin_bit_cast(unsigned, x), __builtin_bit_cast(unsigned, y), false, false);
    return __builtin_bit_cast(float, (unsigned)r[0]) + __builtin_bit_cast(float, (unsigned)r[1]);
}
__device__ __forceinline__ float swap32_add(float x, float y)
{
    auto r = __builtin_amdgcn_permlane32_swap(__builtin_bit_cast(unsigned, x), __builtin_bit_cast(unsigned, y), false, false);
    return __builtin_bit_cast(float, (unsigned)r[0]) + __builtin_bit_cast(float, (unsigned)r[1]);
}

// The tile's (max, sum of exp) per head, and the logits to memory, for the slice-streaming score kernels.
// sc[p][x][o] of lane (n, gk) is the logit of head 4 x + gk (M = 16) or 4 x + 2 o + par (M = 32) for the lane's token
// of pass p, tb + p * 4 * 64 * (sets of the pass).  The tokens of a wavefront are scattered over the tile (4 fine
// positions x 4 coarse rows per pass), so the logits of four heads at a time are transposed through the now idle
// slice area of LDS (stg), [head][coarse row][68] floats (rows padded from 64, heads offset by 16 banks: the writes
// of a wavefront fall on 32 different banks), and leave as runs of 256 consecutive tokens per wavefront.
// stat_dst: where the tile's statistics of head 0 go (stride nsplit per head), or null.
template <int M, int G, int TPT, int NPASS, int NGRP, int NOUT>
__device__ __forceinline__ void write_tile_logits(const float (&sc)[NPASS][NGRP][NOUT], float *stg, float2 (*wstat)[G],
                                                  float *srow, float2 *stat_dst, int nsplit, int tb, int t0, int L)
{
    constexpr int TILE = TPT * kSliceThreads, NW = kSliceThreads / 64;
    constexpr int PSTRIDE = 4 * kLo * (M == 16 ? 1 : 2);
    constexpr int SROW = 68, SHEAD = (TILE / kLo) * SROW + 16;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, gk = lane >> 4, par = gk & 1, set = gk >> 1;
    const int rel0 = tb - t0;
#pragma unroll
    for (int x = 0; x < NGRP; ++x) {
#pragma unroll
        for (int o = 0; o < NOUT; ++o) {
            const int head = 4 * x + (M == 16 ? gk : 2 * o + par);
            float mx = -INFINITY;
#pragma unroll
            for (int p = 0; p < NPASS; ++p) {
                const int tok = tb + p * PSTRIDE;
                if (head < G && tok < L) mx = fmaxf(mx, sc[p][x][o]);
            }
            const float wm = head_lanes_max<M>(mx);
            float l = 0.f;
#pragma unroll
            for (int p = 0; p < NPASS; ++p) {
                const int tok = tb + p * PSTRIDE;
                if (head < G && tok < L) l += __builtin_amdgcn_exp2f((sc[p][x][o] - wm) * kLog2e);
            }
            l = head_lanes_sum<M>(l);
            if (n == 0 && head < G && (M == 16 || set == 0)) wstat[wave][head] = make_float2(wm, l);
        }
        __syncthreads();  // the last slice (x = 0) or the previous group's logits have been read by everyone
#pragma unroll
        for (int o = 0; o < NOUT; ++o) {
            const int hl = M == 16 ? gk : 2 * o + par;
#pragma unroll
            for (int p = 0; p < NPASS; ++p) {
                const int rel = rel0 + p * PSTRIDE;
                stg[hl * SHEAD + (rel >> kLoBits) * SROW + (rel & (kLo - 1))] = sc[p][x][o];
            }
        }
        __syncthreads();
#pragma unroll
        for (int it = 0; it < TPT; ++it) {
            const int idx = it * kSliceThreads + tid;
            const int hl = idx / (TILE / 4), rel = 4 * (idx % (TILE / 4));
            const int head = 4 * x + hl, tok = t0 + rel;
            if (head < G && tok < L) {
                const float4 v = *reinterpret_cast<const float4 *>(stg + hl * SHEAD + (rel >> kLoBits) * SROW + (rel & (kLo - 1)));
                float *dst = srow + (size_t)head * L + tok;
                if (tok + 3 < L) {
                    typedef float f4u __attribute__((ext_vector_type(4), aligned(4)));  // L need not be a multiple of 4
                    const f4u vv = {v.x, v.y, v.z, v.w};
                    *reinterpret_cast<f4u *>(dst) = vv;
                } else {
                    dst[0] = v.x;
                    if (tok + 1 < L) dst[1] = v.y;
                    if (tok + 2 < L) dst[2] = v.z;
                }
            }
        }
    }
    __syncthreads();
    if (tid < G && stat_dst) {
        float m = -INFINITY;
        for (int w = 0; w < NW; ++w) m = fmaxf(m, wstat[w][tid].x);
        float l = 0.f;
        for (int w = 0; w < NW; ++w) {
            const float2 st = wstat[w][tid];
            if (st.x != -INFINITY) l += st.y * __builtin_amdgcn_exp2f((st.x - m) * kLog2e);
        }
        stat_dst[(size_t)tid * nsplit] = make_float2(m, l);
    }
}

// Slice-streaming score kernel with both contractions on the matrix cores (Eq. new_attention,
// re-bracketed: gather-sum the codeword blocks first, rotate once, contract with the G queries).
// Works on the key codebook repacked by k_prep: slice sl (DS = 256 / M consecutive elements of
// every codeword) sits in LDS as tab[P][M][K] 16-byte pieces while all tokens of the tile pass by.
//
// Tokens.  A tile of TILE = 1024 TPT tokens is 64 fine positions (token mod 64) x TILE / 64 coarse rows.  A
// wavefront owns 4 fine positions; in a pass, lane n of its 16 token lanes takes fine position n / 4 and
// coarse row n % 4 of the pass's block of rows (M = 32: a second set of 16 tokens, 4 rows further on).
// So the 4 lanes of a 4-lane block, and all passes of a lane, are whole coarse rows apart: they share the
// fine phase factor E_lo of the relative position 64 H + lo, which is therefore folded into the block's
// query operand once per slice, and a pass only rotates by the coarse factor E_hi.
//
// Codes.  The tile's codes are read once and stay in registers for all slices, already in the byte order
// of the lane's gather steps (M = 16: streamed in during the first slice; see STREAM0).
//
// Per slice and pass:
//  1. Gather-sum: v_smfmac_f32_16x16x64_bf16 (structured-sparse first operand) with a constant 0/1
//     selection matrix as first operand and 128 gathered pieces as second: lane n + 16 g supplies two
//     pieces, A and B, for column n.  Products with 1.0 are exact, so this is the plain fp32 sum of the
//     M codeword slices.  Rows 0..7 of the result are the elements of the four lanes' A pieces added up,
//     rows 8..15 those of their B pieces:
//       M = 16 (two planes): a pass covers 16 tokens; A / B = plane 0 / plane 1 of one codebook;
//               lane (n, g) receives elements 4g .. 4g+3 of the slice for its token;
//       M = 32 (one plane):  a pass covers 32 tokens in two sets; A / B = the same codebook for the
//               lane's token of set 0 and of set 1; lane (n, g) receives elements 4 (g & 1) .. +3 for
//               its token of set g >> 1.
//     The LDS reads of a group of steps are issued right after the matrix instructions that consumed the
//     group's registers, so the first reads of the next pass travel while this pass is finished.
//  2. Each lane rotates its two (x, y) sub-spaces by the coarse phase factor of its token.
//  3. Contraction with the queries: four v_mfma_f32_4x4x1_16b_f32 per group of 4 heads.  In each
//     block of 4 lanes, lane i supplies q'[head i][the block's r-th element] (q' = q conj(E_lo)) and every
//     lane its own rotated r-th element, so register i of a lane receives the partial logit of head i for
//     the lane's own token over the lane's 4 elements.  The 4 (M = 16) or 2 (M = 32) lanes of a token
//     are then combined with row / half swaps so that each keeps the total of one (two) heads:
//     lane (n, g) holds head g of its token (M = 16), heads g & 1 and 2 + (g & 1) (M = 32).
// On gfx950 the vector and matrix instructions of a SIMD do not overlap (measured again on this kernel:
// interleaving the next pass's gather-sum with this pass's vector work changes nothing), so a pass costs the
// sum of its instruction issue: 4 (8) sparse MFMA of 16 clk, 4 small ones of 8 per head group, ~28 vector
// instructions.
//
// Short contexts: a launch may cut every tile along the slices as well (SliceDims::groups workgroups per
// tile); each then writes partial logits, which k_score_combine adds.
template <int M, int G, int TPT>
__global__ __launch_bounds__(kSliceThreads) void k_score_mfma(
    const void *__restrict__ q, const uint8_t *__restrict__ key_codes, const uint4 *__restrict__ packed,
    const int32_t *__restrict__ cu, const int32_t *__restrict__ q_pos, const float2 *__restrict__ tbl_hi,
    const float2 *__restrict__ tbl_lo, float *__restrict__ scores, float2 *__restrict__ sstat, const SliceDims a)
{
    constexpr int DS = 256 / M;          // elements per slice (16 or 8)
    constexpr int NJ = DS / 2;           // sub-spaces per slice
    constexpr int P = DS / 8;            // 16-byte planes per slice
    constexpr int S = kD / DS;           // slices
    constexpr int TILE = TPT * kSliceThreads;
    constexpr int NW = kSliceThreads / 64;
    constexpr int SETS = M == 16 ? 1 : 2;                     // 16-token sets per wavefront pass
    constexpr int NPASS = TILE / (16 * SETS * NW);
    constexpr int PARTS = NJ / 2;                             // 16-byte (two sub-space) parts of a slice's phase rows
    constexpr int NHR = TILE / kLo + 1;                       // coarse phase rows a tile can touch
    constexpr int NGRP = (G + 3) / 4;                         // groups of 4 heads (padded with zero queries)
    constexpr int NOUT = M == 16 ? 1 : 2;                     // heads per group whose totals a lane keeps
    constexpr int CW = M / 8;                                 // code dwords a lane needs per token
    static_assert(NPASS % 2 == 0, "code double-buffer parity assumes an even number of passes");
    extern __shared__ __attribute__((aligned(16))) uint4 tab[];  // [2][K][16] 16-byte pieces, then the phase factors
    float4 *elo = reinterpret_cast<float4 *>(tab + kSliceBytes / 16);  // [PARTS][64]  exp(i theta_j lo), this slice's j
    float4 *ehi = elo + PARTS * kLo;                                   // [NHR][PARTS] exp(i theta_j 64 H), H = Hmin + row
    // the slice sits at LDS address 0 (no static LDS in this kernel), so gather addresses need no base added
    float2(*wstat)[G] = reinterpret_cast<float2(*)[G]>(reinterpret_cast<char *>(tab) + kSliceBytes + 2 * kPhaseBytes);  // [NW][G]

    int id = blockIdx.x;
    const int g = id % a.Hkv;
    id /= a.Hkv;
    const int tile = id % a.nsplit;
    id /= a.nsplit;
    const int eg = id % a.groups;                             // which group of slices (0 when tiles are not cut along them)
    const int b = id / a.groups;
    const int s_begin = eg * (S / a.groups), s_end = s_begin + S / a.groups;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // The first slice of the head's codebook depends on nothing but the workgroup index: it is requested before the
    // sequence's bounds are even known, so that its (cold) fetch, that of the bounds and that of the tile's codes
    // overlap.  Later slices are fetched into the same registers while the last pass of the current one finishes (its
    // gather registers are dead by then).
    constexpr int PIECES = P * M * kK;
    constexpr int PPT = PIECES / kSliceThreads;
    const uint4 *src = packed + (size_t)g * S * P * M * kK;
    const __amdgpu_buffer_rsrc_t src_rs = make_rsrc(src, (unsigned)S * PIECES * 16u);
    uint4_t stage[PPT];
    auto fetch_slice = [&](int sl) {
        // the slice index is the same in every lane; said so explicitly, or the loads may be wrapped in a loop over
        // the distinct values of what the compiler holds in a vector register
        const unsigned soff = __builtin_amdgcn_readfirstlane((unsigned)sl * (PIECES * 16u));
#pragma unroll
        for (int x = 0; x < PPT; ++x)
            stage[x] = __builtin_amdgcn_raw_buffer_load_b128(src_rs, (unsigned)(x * kSliceThreads + tid) * 16u, soff, 0);
    };
    constexpr bool PREFETCH = !(M == 32 && G == 8 && TPT == 4);  // that instantiation has no registers to spare
    if (PREFETCH) fetch_slice(s_begin);
    const int cu0 = cu[b];
    const int L = cu[b + 1] - cu0;
    const int t0 = tile * TILE;
    if (t0 >= L) return;
    const int n = lane & 15, gk = lane >> 4;
    const int par = gk & 1;                                   // odd / even codebook of a gather step
    const int set = gk >> 1;                                  // M = 32: which 16-token set the lane gathers for
    const int el = M == 16 ? 4 * gk : 4 * par;                // first of the lane's 4 slice elements
    const int qpos = q_pos[b];
    const uint8_t *codes = key_codes + ((size_t)cu0 * a.Hkv + (size_t)g * L) * M;
    const __amdgpu_buffer_rsrc_t cd_rs = make_rsrc(codes, (unsigned)L * M);
    const unsigned qesz = a.q_bf16 ? 2u : 4u;
    const __amdgpu_buffer_rsrc_t q_rs =
        make_rsrc(static_cast<const char *>(q) + ((size_t)b * a.Hq + (size_t)g * G) * kD * qesz, (unsigned)G * kD * qesz);

    // Selection operand of v_smfmac_f32_16x16x64_bf16 (first operand structured-sparse: two of every four
    // consecutive k kept, 2-bit positions in an index register).  Its second operand takes two 16-byte pieces per
    // lane, A (elements 0..7) and B (8..15); measured layout (micro-benchmark smfmac_layouts): logical k =
    // 32 * (A | B) + 8 * (lane / 16) + element, and first-operand lane (row i, block q) covers k = 16 q .. 16 q + 15
    // with stored slots 2 t, 2 t + 1 for its t-th group of four.  Rows 0..7 must add element i of the four lanes'
    // A pieces, rows 8..15 element i - 8 of their B pieces: lane (i, q) is active when (i < 8) == (q < 2) and then
    // keeps 1.0 at position e % 4 of groups e / 4 and 2 + e / 4 (e = i % 8); every other stored value is 0.0.
    uint4_t sel = {0u, 0u, 0u, 0u};
    unsigned sidx = 0x44444444u;  // default positions (0, 1) of every stored pair
    {
        const int e = n & 7;
        if ((n < 8) == (gk < 2)) {
            const int t = e >> 2, pos = e & 3, other = pos == 0 ? 1 : 0;
            sel[t] = 0x00003f80u;        // slot 2 t      = 1.0, slot 2 t + 1 = 0.0
            sel[2 + t] = 0x00003f80u;    // slot 4 + 2 t  = 1.0
            const unsigned pair = (unsigned)pos | (unsigned)other << 2;
            sidx = (sidx & ~(0xfu << (4 * t)) & ~(0xfu << (4 * (2 + t)))) | pair << (4 * t) | pair << (4 * (2 + t));
            sidx = (sidx & 0xffffu) | sidx << 16;
        }
    }
    const bf16x8_t selv = __builtin_bit_cast(bf16x8_t, sel);
    // as first operand of the query contraction the lane supplies head 4 grp + n % 4; rows past the last
    // head read beyond the end of the buffer, i.e. zero
    const unsigned q_off = (unsigned)(n & 3) * kD + (unsigned)el;  // in elements

    float sc[NPASS][NGRP][NOUT];
#pragma unroll
    for (int p = 0; p < NPASS; ++p)
#pragma unroll
        for (int x = 0; x < NGRP; ++x)
#pragma unroll
            for (int o = 0; o < NOUT; ++o) sc[p][x][o] = 0.f;

    // What a lane gathers (gk = (hi, par)):
    //   M = 16: for its own token the 4 codebooks 8 par + (n + 4 hi + st) mod 8, st = 0..3, piece A from plane 0 and
    //           piece B from plane 1 of each: the four lanes of a token cover its 16 codebooks in 4 instructions;
    //   M = 32: for tokens n (piece A) and n + 16 (piece B) of the pass the 8 codebooks 16 hi + 8 par + (n + st) mod 8.
    // In every group of lanes that the LDS checks against each other for bank conflicts the 16 pieces of one read
    // then come from 16 different bank columns, whatever the codes.  xreg[st]: byte 0 = 16 * column read at step
    // st, byte 2 = 64 KiB block (M = 16: 0, and byte 3 = 1 for plane 1; M = 32: hi); a byte permute splices the code
    // in as byte 1, which yields the LDS byte address 65536 blk + 256 c + 16 col in one instruction.
    const int hi = gk >> 1;
    constexpr int NST = M == 16 ? 4 : 8;  // gather steps = sparse matrix instructions per pass
    unsigned xreg[NST];
#pragma unroll
    for (int st = 0; st < NST; ++st)
        xreg[st] = (unsigned)(8 * par + ((n + st + (M == 16 ? 4 * hi : 0)) & 7)) * 16u | (M == 16 ? 1u << 24 : (unsigned)hi << 16);
    // byte selectors that rotate 8 code bytes so that step st finds its code at byte st
    unsigned rsel_lo = 0u, rsel_hi = 0u;
#pragma unroll
    for (int x = 0; x < 4; ++x) {
        rsel_lo |= (unsigned)((x + n + (M == 16 ? 4 * hi : 0)) & 7) << (8 * x);
        rsel_hi |= (unsigned)((x + 4 + n) & 7) << (8 * x);
    }

    // tb is the lane's token of pass 0 (the one whose logits it ends up with; pass p: tb + p PSTRIDE); it is re-read
    // through an opaque copy in every slice so that nothing that depends on a token index (table offsets) is hoisted
    // out of the slice loop.  M = 32: the lane gathers for the set-0 token tb - 256 set and the set-1 token 256 further.
    int tb = t0 + 4 * wave + (n >> 2) + kLo * ((n & 3) + (M == 16 ? 0 : 4 * set));
    constexpr int PSTRIDE = 4 * kLo * SETS;  // tokens between two passes of a lane: a whole number of coarse rows
    // byte offset of the codes the lane gathers in pass 0 (M = 32: of the first of its two tokens, the second is
    // 4 coarse rows further on); refreshed with tb in every slice
    unsigned code_off = (unsigned)(tb - (M == 16 ? 0 : 4 * kLo * set)) * M + (M == 16 ? 8u * par : 16u * hi + 8u * par);
    auto fetch_codes = [&](int p, unsigned(&dst)[CW]) {
        // tokens past the end of the sequence read zeros (the descriptor ends with the sequence): code 0, a valid row
        if (M == 16) {  // bytes 8 par .. + 7 of the token's codes
            const uint2_t c2 = __builtin_amdgcn_raw_buffer_load_b64(cd_rs, code_off + (unsigned)(p * PSTRIDE * M), 0, 0);
            dst[0] = c2[0]; dst[1] = c2[1];
        } else {        // bytes 16 hi + 8 par .. + 7 of both tokens
#pragma unroll
            for (int v = 0; v < 2; ++v) {
                const uint2_t c2 = __builtin_amdgcn_raw_buffer_load_b64(cd_rs, code_off + (unsigned)((p * PSTRIDE + 4 * kLo * v) * M), 0, 0);
                dst[2 * v + 0] = c2[0]; dst[2 * v + 1] = c2[1];
            }
        }
    };
    // cc[v][h]: rotated code bytes 4 h .. 4 h + 3 of token v (M = 16: one token, steps 0..3 only): what the gather
    // addresses of a pass are made from.
    constexpr int CV = M == 16 ? 1 : 2;
    auto make_cc = [&](const unsigned(&c)[CW], unsigned(&cc)[CV][CV]) {
        if (M == 16) {
            cc[0][0] = __builtin_amdgcn_perm(c[1], c[0], rsel_lo);
        } else {
#pragma unroll
            for (int v = 0; v < 2; ++v) {
                cc[v][0] = __builtin_amdgcn_perm(c[2 * v + 1], c[2 * v], rsel_lo);
                cc[v][CV - 1] = __builtin_amdgcn_perm(c[2 * v + 1], c[2 * v], rsel_hi);
            }
        }
    };
    // The codes of the whole tile are read ONCE and stay in registers, in gather order (ccall[p] = cc of pass p), for
    // all slices: a per-pass fetch has to cover the latency of a load that misses L1 in every slice (the tile's codes
    // are 64 KiB or more), which a look-ahead of two passes does not, and it re-reads the tile's codes once per slice.
    // Only the first slice streams them (STREAM0): its pass p turns the codes of pass p + 1 into ccall[p + 1] and
    // requests those of pass p + 3, so that the cold fetch of the codes hides behind the first slice's arithmetic.
    // Raw codes in flight: those of passes 0 and 1 (requested here) wait in the ccall slots of the LAST passes, which
    // are not written until the raw values have long been used; later ones in the first registers of the slice
    // staging buffer, idle between the slice's LDS write and the last pass.
    constexpr bool STREAM0 = M == 16 && NPASS >= 4;  // (with 32 codebooks the stream's two loads per pass do not hide)
    constexpr int RAWS = NPASS * CV * CV / CW;                // ccall slots that one pass's raw codes take (2 or 1)
    unsigned ccall[NPASS][CV][CV];
    auto raw_slot = [&](int k, unsigned(&dst)[CW]) {          // raw codes of pass k (0 or 1): copy out of their parking slots
#pragma unroll
        for (int i = 0; i < CW; ++i) {
            const int flat = (NPASS * CV * CV - 2 * CW) + k * CW + i;
            dst[i] = ccall[flat / (CV * CV)][(flat / CV) % CV][flat % CV];
        }
    };
    if (STREAM0) {
        unsigned r0[CW], r1[CW];
        fetch_codes(0, r0);
        fetch_codes(1, r1);
#pragma unroll
        for (int i = 0; i < CW; ++i) {
            const int f0 = (NPASS * CV * CV - 2 * CW) + i, f1 = f0 + CW;
            ccall[f0 / (CV * CV)][(f0 / CV) % CV][f0 % CV] = r0[i];
            ccall[f1 / (CV * CV)][(f1 / CV) % CV][f1 % CV] = r1[i];
        }
    } else {
        unsigned craw[NPASS][CW];
#pragma unroll
        for (int p = 0; p < NPASS; ++p) fetch_codes(p, craw[p]);
#pragma unroll
        for (int p = 0; p < NPASS; ++p) make_cc(craw[p], ccall[p]);
    }
    (void)RAWS;
    const int hmin = (qpos - (t0 + TILE - 1)) >> kLoBits;     // coarse row of the tile's last token (arithmetic shift)
    const unsigned elo_base = (unsigned)kSliceBytes + (unsigned)(M == 16 ? gk : par) * (kLo * 16u);
    const unsigned ehi_base = (unsigned)kSliceBytes + (unsigned)(PARTS * kLo) * 16u + (unsigned)(M == 16 ? gk : par) * 16u;

    // Phase factors of a slice's sub-spaces, two buffers of [PARTS * 64 fine entries][NHR * PARTS coarse entries]:
    // the fine table as it is, and the rows of the coarse table that the tile's distances q_pos - token can reach,
    // row-major, so that the four coarse rows and the parts that the lanes of a read touch are 16 consecutive 16-byte
    // pieces (no bank conflicts).  Thread t < PARTS * 64 moves fine entry t, the next PARTS * NHR threads one coarse
    // entry each.  Where no distance of the tile is negative the entries go from memory straight into LDS, a whole
    // slice ahead; a negative distance takes the conjugate of the row of its absolute value, which needs a register.
    const bool DMA_OK = hmin >= 0;
    auto phase_src = [&](int sl, bool &neg) -> const float2 * {
        neg = false;
        if (tid < PARTS * kLo) {
            const int part = tid / kLo, lo = tid % kLo;
            return tbl_lo + (size_t)lo * kJ + sl * NJ + 2 * part;
        }
        const int x = tid - PARTS * kLo;
        const int part = x % PARTS, H = hmin + x / PARTS;
        neg = H < 0;
        return tbl_hi + (size_t)min(H < 0 ? -H : H, a.n_hi - 1) * kJ + sl * NJ + 2 * part;
    };
    static_assert(PARTS * kLo + PARTS * NHR <= kSliceThreads && (PARTS * kLo) % 64 == 0, "one phase entry per thread");
    auto dma_phase = [&](int sl, int buf) {
        if (tid < PARTS * kLo + PARTS * NHR) {
            bool neg;
            const float2 *srcp = phase_src(sl, neg);
            lds_dma16(srcp, __builtin_amdgcn_readfirstlane((unsigned)kSliceBytes + (unsigned)buf * kPhaseBytes + (unsigned)wave * 1024u));
        }
    };
    auto stage_phase = [&](int sl, int buf) {
        if (tid < PARTS * kLo + PARTS * NHR) {
            bool neg;
            float4 e = *reinterpret_cast<const float4 *>(phase_src(sl, neg));
            if (neg) { e.y = -e.y; e.w = -e.w; }
            elo[(size_t)buf * (kPhaseBytes / 16) + tid] = e;
        }
    };
    if (DMA_OK) dma_phase(s_begin, s_begin & 1);

    for (int si = 0; si < s_end - s_begin; ++si) {  // (counted from 0, so that the first slice's extra work can be peeled off)
        const int sl = s_begin + si;
        if (!PREFETCH) fetch_slice(sl);
        // queries of this slice (head 4 grp + n % 4, the lane's 4 elements): requested before the barriers, so
        // that they have arrived when the first pass needs them
        uint4_t qraw[NGRP];
#pragma unroll
        for (int x = 0; x < NGRP; ++x) {
            const unsigned off = q_off + (unsigned)x * (4u * kD);
            if (a.q_bf16) {
                const uint2_t q2 = __builtin_amdgcn_raw_buffer_load_b64(q_rs, off * 2u, (unsigned)sl * DS * 2u, 0);
                qraw[x][0] = q2[0]; qraw[x][1] = q2[1]; qraw[x][2] = 0u; qraw[x][3] = 0u;
            } else {
                qraw[x] = __builtin_amdgcn_raw_buffer_load_b128(q_rs, off * 4u, (unsigned)sl * DS * 4u, 0);
            }
        }
        __syncthreads();  // everyone is done reading the previous slice
#pragma unroll
        for (int x = 0; x < PPT; ++x) reinterpret_cast<uint4_t *>(tab)[x * kSliceThreads + tid] = stage[x];
        if (!DMA_OK) stage_phase(sl, sl & 1);
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this slice's phase factors (sent a slice ago) are in LDS
        __syncthreads();
        // the phase factors of the next slice travel into the other phase buffer while this slice is worked on
        if (DMA_OK) dma_phase(min(sl + 1, S - 1), (sl + 1) & 1);
        const unsigned ph_off = (unsigned)(sl & 1) * kPhaseBytes;
        asm volatile("" : "+v"(tb));
        code_off = (unsigned)(tb - (M == 16 ? 0 : 4 * kLo * set)) * M + (M == 16 ? 8u * par : 16u * hi + 8u * par);
        // byte offsets (in the LDS phase tables) of the lane's part, and its distance to the query, times 16
        const int dist16 = (qpos - tb) * 16;
        // scaled queries of this slice
        float qrow[NGRP][4];
#pragma unroll
        for (int x = 0; x < NGRP; ++x) {
            if (a.q_bf16) {
                qrow[x][0] = bf16_lo(qraw[x][0]) * a.scale; qrow[x][1] = bf16_hi(qraw[x][0]) * a.scale;
                qrow[x][2] = bf16_lo(qraw[x][1]) * a.scale; qrow[x][3] = bf16_hi(qraw[x][1]) * a.scale;
            } else {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const unsigned u = qraw[x][r];
                    qrow[x][r] = __builtin_bit_cast(float, u) * a.scale;
                }
            }
        }
        // The tokens of a lane (one per pass) and of the four lanes of a 4-lane block are whole coarse rows (64
        // tokens) apart: they share the fine phase factor E_lo, so it is folded into the block's query operand
        // once per slice, q' = q conj(E_lo) (Re(conj(q) a E_hi E_lo) = Re(conj(q') a E_hi)), and a pass only rotates
        // by the coarse factor, whose row steps down by a constant from pass to pass.
        static_assert(PSTRIDE % kLo == 0, "pass stride in whole coarse rows");
        {
            const uint4_t elr = lds_read_b128(elo_base + ph_off + (unsigned)(dist16 & ((kLo - 1) * 16)));
#pragma unroll
            for (int x = 0; x < NGRP; ++x)
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const unsigned lxr = elr[2 * u], lyr = elr[2 * u + 1];
                    const float lx = __builtin_bit_cast(float, lxr), ly = __builtin_bit_cast(float, lyr);
                    const float qx = qrow[x][2 * u], qy = qrow[x][2 * u + 1];
                    qrow[x][2 * u] = qx * lx + qy * ly;
                    qrow[x][2 * u + 1] = qy * lx - qx * ly;
                }
        }
        const unsigned ehi_last = ehi_base + ph_off + (unsigned)(((dist16 >> (kLoBits + 4)) - hmin - (NPASS - 1) * (PSTRIDE / kLo)) * (16 * PARTS));
        // per step two LDS reads (pieces A and B) and one sparse MFMA; reads in groups of RG steps, two groups in flight
        constexpr int RG = (G == 8 && TPT == 4) ? 1 : 2, NG = NST / RG;  // fewer reads in flight where registers are short
        uint4_t v[2][RG][2];
        auto issue = [&](int grp, const unsigned(&cc)[CV][CV], uint4_t(&dst)[RG][2]) {
#pragma unroll
            for (int r = 0; r < RG; ++r) {
                const int st = grp * RG + r;
#pragma unroll
                for (int ab = 0; ab < 2; ++ab) {
                    // address bytes: [0] column, [1] code byte st % 4 of its dword, [2] block, [3] zero.  M = 16: block =
                    // plane = ab (xreg bytes 2, 3 hold 0, 1); M = 32: block = hi (xreg byte 2), the code is token ab's
                    const unsigned sel = 0x0c000000u | (unsigned)(M == 16 ? 2 + ab : 2) << 16 | (unsigned)(4 + st % 4) << 8;
                    const unsigned addr = __builtin_amdgcn_perm(cc[M == 16 ? 0 : ab][M == 16 ? 0 : st / 4], xreg[st], sel);
                    dst[r][ab] = lds_read_b128(addr);
                }
            }
        };
        // The passes are software-pipelined: the LDS reads of a group of steps are issued as soon as the matrix
        // instructions that consumed the group's registers have been issued -- for the last groups of a pass these are
        // the first reads of the NEXT pass, which then travel while this pass is rotated and contracted with the queries.
        unsigned cc[CV][CV];
        if (STREAM0 && si == 0) {
            unsigned r[CW];
            raw_slot(0, r);
            make_cc(r, ccall[0]);
            if (2 < NPASS) {
                unsigned f[CW];
                fetch_codes(2, f);
#pragma unroll
                for (int i = 0; i < CW; ++i) stage[0][i] = f[i];
            }
        }
        // an opaque copy per slice: the gather addresses made from these must not be hoisted out of the slice loop
        // (they would need eight registers per pass instead of one)
#pragma unroll
        for (int pp = 0; pp < NPASS; ++pp)
#pragma unroll
            for (int i = 0; i < CV; ++i)
#pragma unroll
                for (int j = 0; j < CV; ++j) asm volatile("" : "+v"(ccall[pp][i][j]));
#pragma unroll
        for (int i = 0; i < CV; ++i)
#pragma unroll
            for (int j = 0; j < CV; ++j) cc[i][j] = ccall[0][i][j];
        issue(0, cc, v[0]);
        if (NG > 1) issue(1, cc, v[1]);
#pragma unroll
        for (int p = 0; p < NPASS; ++p) {
            __builtin_amdgcn_sched_barrier(0);  // one pass at a time: keeps register pressure flat
            // coarse phase factor of the lane's token and part, from LDS: a pass is a whole number of coarse rows
            // further on
            const uint4_t ehr = lds_read_b128(ehi_last + (unsigned)((NPASS - 1 - p) * (PSTRIDE / kLo) * (16 * PARTS)));
            unsigned ccn[CV][CV];
            if (p + 1 < NPASS) {
                if (STREAM0 && si == 0) {
                    // first slice: the codes of pass p + 1 have arrived (raw, requested two passes ago); keep them in
                    // gather order and request those of pass p + 3 into the buffer they leave
                    unsigned r[CW];
                    if (p == 0) {
                        raw_slot(1, r);
                    } else {
#pragma unroll
                        for (int i = 0; i < CW; ++i) r[i] = stage[(p + 1) & 1][i];
                    }
                    make_cc(r, ccall[p + 1]);
                    if (p + 3 < NPASS) {
                        unsigned f[CW];
                        fetch_codes(p + 3, f);
#pragma unroll
                        for (int i = 0; i < CW; ++i) stage[(p + 1) & 1][i] = f[i];
                    }
                }
#pragma unroll
                for (int i = 0; i < CV; ++i)
#pragma unroll
                    for (int j = 0; j < CV; ++j) ccn[i][j] = ccall[p + 1][i][j];
            }
            __builtin_amdgcn_sched_barrier(0);
            // 1. gather-sum on the matrix cores
            floatx4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int grp = 0; grp < NG; ++grp) {
#pragma unroll
                for (int r = 0; r < RG; ++r) {
                    const uint4_t pa = v[grp & 1][r][0], pb = v[grp & 1][r][1];
                    const uint8v_t both = {pa[0], pa[1], pa[2], pa[3], pb[0], pb[1], pb[2], pb[3]};
                    acc = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(selv, __builtin_bit_cast(bf16x16_t, both), acc, (int)sidx, 0, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
                if (grp + 2 < NG) issue(grp + 2, cc, v[grp & 1]);
                else if (p + 1 < NPASS) issue(grp + 2 - NG, ccn, v[grp & 1]);
                __builtin_amdgcn_sched_barrier(0);
            }
            if (PREFETCH && p == NPASS - 1) fetch_slice(min(sl + 1, S - 1));  // after the last slice: a harmless re-read
            if (p + 1 < NPASS) {
#pragma unroll
                for (int i = 0; i < CV; ++i)
#pragma unroll
                    for (int j = 0; j < CV; ++j) cc[i][j] = ccn[i][j];
            }
            // 2. the lane's two sub-spaces rotated by the coarse phase factor: A E_hi
            float val[4];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const unsigned hxr = ehr[2 * u], hyr = ehr[2 * u + 1];
                const float ex = __builtin_bit_cast(float, hxr);
                const float ey = __builtin_bit_cast(float, hyr);
                const float ax = acc[2 * u], ay = acc[2 * u + 1];
                val[2 * u] = ax * ex - ay * ey;
                val[2 * u + 1] = ax * ey + ay * ex;
            }
            // 3. per-lane partial logits of 4 heads at a time, then totals over the lanes of the token
#pragma unroll
            for (int x = 0; x < NGRP; ++x) {
                floatx4_t t = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int r = 0; r < 4; ++r) t = __builtin_amdgcn_mfma_f32_4x4x1f32(qrow[x][r], val[r], t, 0, 0, 0);
                if (M == 16) {
                    sc[p][x][0] += swap16_add(swap32_add(t[0], t[2]), swap32_add(t[1], t[3]));
                } else {
                    sc[p][x][0] += swap16_add(t[0], t[1]);
                    sc[p][x][NOUT - 1] += swap16_add(t[2], t[3]);
                }
            }
        }
    }

    // a slice group leaves partial logits in its own array; the tile statistics then come from k_score_combine
    float *srow = scores + (size_t)eg * a.part_stride + (size_t)cu0 * a.Hq + (size_t)g * G * L;
    float2 *stat_dst = a.groups == 1 ? sstat + ((size_t)b * a.Hq + (size_t)g * G) * a.nsplit + tile : nullptr;
    write_tile_logits<M, G, TPT, NPASS, NGRP, NOUT>(sc, reinterpret_cast<float *>(tab), wstat, srow, stat_dst, a.nsplit, tb, t0, L);
}

// ------------------------------------------------------------------ k_score_combine
// Score tiles that were also cut along the codebook slices (short contexts): the logit of a token is the sum of the
// partial logits of the slice groups (Eq. new_attention's sum over the sub-spaces, split in `groups` parts).  One
// workgroup per (sequence, query head, 1024 tokens): adds the parts in a fixed order, writes the logits and the
// (max, sum of exp) of its 1024 tokens.
constexpr int kCombineThreads = 256;
__global__ __launch_bounds__(kCombineThreads) void k_score_combine(const float *__restrict__ part, float *__restrict__ scores,
                                                                  float2 *__restrict__ sstat, const int32_t *__restrict__ cu,
                                                                  int Hq, int nsplit, int tile_len, int groups, long long part_stride)
{
    __shared__ float red[kCombineThreads / 64];
    int id = blockIdx.x;
    const int tile = id % nsplit;
    id /= nsplit;
    const int h = id % Hq, b = id / Hq;
    const int cu0 = cu[b], L = cu[b + 1] - cu0;
    const int t0 = tile * tile_len;
    if (t0 >= L) return;
    const int t1 = min(t0 + tile_len, L);
    const size_t row = (size_t)cu0 * Hq + (size_t)h * L;
    constexpr int MAXV = 1024 / kCombineThreads;  // statistics tiles of 1024 tokens
    float v[MAXV];
    float mx = -INFINITY;
#pragma unroll
    for (int k = 0; k < MAXV; ++k) {
        const int tok = t0 + k * kCombineThreads + (int)threadIdx.x;
        v[k] = -INFINITY;
        if (k * kCombineThreads < tile_len && tok < t1) {
            // all parts requested at once (at most 16 slice groups), added in a fixed order
            float pv[16];
#pragma unroll
            for (int e = 0; e < 16; ++e) pv[e] = e < groups ? part[(size_t)e * part_stride + row + tok] : 0.f;
            float acc = pv[0];
#pragma unroll
            for (int e = 1; e < 16; ++e) acc += pv[e];
            scores[row + tok] = acc;
            v[k] = acc;
            mx = fmaxf(mx, acc);
        }
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    mx = wave_max(mx);
    if (lane == 0) red[wave] = mx;
    __syncthreads();
    {
        float m2 = red[0];
        for (int w = 1; w < kCombineThreads / 64; ++w) m2 = fmaxf(m2, red[w]);
        mx = m2;
    }
    __syncthreads();
    float l = 0.f;
#pragma unroll
    for (int k = 0; k < MAXV; ++k)
        if (v[k] != -INFINITY) l += __builtin_amdgcn_exp2f((v[k] - mx) * kLog2e);
    l = wave_sum(l);
    if (lane == 0) red[wave] = l;
    __syncthreads();
    if (threadIdx.x == 0) {
        float lt = 0.f;
        for (int w = 0; w < kCombineThreads / 64; ++w) lt += red[w];  // fixed order
        sstat[((size_t)b * Hq + h) * nsplit + tile] = make_float2(mx, lt);
    }
}

// ------------------------------------------------------------------ position-free keys: scalar look-up table
// The case the paper sets aside in Sec. 4.2: if the rotation did not depend on the token (keys quantized
// after RoPE, or no positional rotation at all), (q C^T) could be computed once and every token's
// score would be M scalar look-ups:  s_i = sum_m T[m][code_i,m],  T[m][c] = scale * q . C[m][c].
//
// k_lut_build: T[b][g][m][c][G] fp32 (G < 4; for G >= 4 in the LDS-image order of k_score_lut, see below), one thread
// per (b, g, m, c) row; the G queries sit in LDS.
template <int G, bool BF16>
__global__ __launch_bounds__(256) void k_lut_build(const void *__restrict__ q, const void *__restrict__ cb,
                                                   float *__restrict__ lut, int Hkv, int M, int q_bf16, float scale)
{
    __shared__ float qs[G][kD];
    const int rows_per_head = M * kK;                       // rows of one KV head
    const int blocks_per_head = rows_per_head / 256;
    const int bg = blockIdx.x / blocks_per_head;            // b * Hkv + g
    const int g = bg % Hkv, b = bg / Hkv;
    const int row = (blockIdx.x % blocks_per_head) * 256 + threadIdx.x;  // m * K + c
    for (int x = threadIdx.x; x < G * kD; x += 256) {
        const size_t i = ((size_t)b * Hkv * G + (size_t)g * G) * kD + x;
        const float v = q_bf16 ? __builtin_bit_cast(float, (unsigned)static_cast<const uint16_t *>(q)[i] << 16)
                               : static_cast<const float *>(q)[i];
        qs[x / kD][x % kD] = v * scale;
    }
    __syncthreads();
    float acc[G];
#pragma unroll
    for (int h = 0; h < G; ++h) acc[h] = 0.f;
    const size_t base = ((size_t)g * rows_per_head + row) * kD;
#pragma unroll 8
    for (int e = 0; e < kD; ++e) {
        const float v = cb_elem<BF16>(cb, base + e);
#pragma unroll
        for (int h = 0; h < G; ++h) acc[h] = __builtin_fmaf(qs[h][e], v, acc[h]);
    }
    if (G >= 4) {
        // groups of four heads: the table leaves in the order k_score_lut keeps it in LDS, [b][g][head group][block of 16
        // codebooks][codeword][codebook of the block][4 heads] -- one 16-byte bank column per codebook
        const int m = row / kK, c = row % kK;
#pragma unroll
        for (int grp = 0; grp < G / 4; ++grp) {
            float4 *dst = reinterpret_cast<float4 *>(lut) +
                          (((size_t)bg * (G / 4) + grp) * (M / 16) + m / 16) * (kK * 16) + (size_t)c * 16 + (m & 15);
            *dst = make_float4(acc[(4 * grp + 0) % G], acc[(4 * grp + 1) % G], acc[(4 * grp + 2) % G], acc[(4 * grp + 3) % G]);
        }
    } else {
        float *dst = lut + ((size_t)bg * rows_per_head + row) * G;
#pragma unroll
        for (int h = 0; h < G; ++h) dst[h] = acc[h];
    }
}

// k_lut_build_mfma: the same table for bf16 codebooks and four or eight heads per KV head, where T = scale q C^T is the
// one dense (heads x M K x d) contraction of these paths: a wavefront takes 16 codebook rows, v_mfma_f32_16x16x32_bf16 with
// the queries as first operand (row = head; a bf16 query as it is, an fp32 query split exactly into three bf16 parts)
// and 16 bytes of a codebook row per lane as second.  Result lane (n, rg) holds heads 4 rg .. 4 rg + 3 of row n: one
// 16-byte entry of head group rg, stored in the LDS-image order of k_score_lut.
template <int G>
__global__ __launch_bounds__(256) void k_lut_build_mfma(const void *__restrict__ q, const uint16_t *__restrict__ cb,
                                                        float *__restrict__ lut, int Hkv, int M, int q_bf16, float scale)
{
    const int rows_per_head = M * kK;
    const int blocks_per_head = rows_per_head / 64;          // 4 wavefronts x 16 rows per workgroup
    const int bg = blockIdx.x / blocks_per_head;             // b * Hkv + g
    const int g = bg % Hkv;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 15, kg = lane >> 4;
    const int row = (blockIdx.x % blocks_per_head) * 64 + 16 * wave + n;  // m * K + c
    floatx4_t acc = {0.f, 0.f, 0.f, 0.f};
    const uint16_t *crow = cb + ((size_t)g * rows_per_head + row) * kD + 8 * kg;
    const size_t qbase = ((size_t)bg * G + (size_t)n) * kD + 8 * kg;  // head n of the group (rows G .. 15: zero)
#pragma unroll
    for (int ks = 0; ks < kD / 32; ++ks) {
        const uint4 B = *reinterpret_cast<const uint4 *>(crow + 32 * ks);
        if (q_bf16) {
            uint4 A = make_uint4(0u, 0u, 0u, 0u);
            if (n < G) A = *reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(q) + qbase + 32 * ks);
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, A), __builtin_bit_cast(bf16x8_t, B), acc, 0, 0, 0);
        } else {
            float qf[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) qf[e] = n < G ? static_cast<const float *>(q)[qbase + 32 * ks + e] : 0.f;
            unsigned part[3][4];
#pragma unroll
            for (int e = 0; e < 8; ++e) {  // top 16 bits, top 16 bits of the rest, the rest: 8 + 8 + 8 mantissa bits, exact
                const unsigned u0 = __builtin_bit_cast(unsigned, qf[e]) & 0xffff0000u;
                const float r1 = qf[e] - __builtin_bit_cast(float, u0);
                const unsigned u1 = __builtin_bit_cast(unsigned, r1) & 0xffff0000u;
                const float r2 = r1 - __builtin_bit_cast(float, u1);
                const unsigned u2 = __builtin_bit_cast(unsigned, r2) & 0xffff0000u;
                if (e & 1) { part[0][e / 2] |= u0; part[1][e / 2] |= u1; part[2][e / 2] |= u2; }
                else { part[0][e / 2] = u0 >> 16; part[1][e / 2] = u1 >> 16; part[2][e / 2] = u2 >> 16; }
            }
#pragma unroll
            for (int pc = 0; pc < 3; ++pc) {
                const uint4 A = make_uint4(part[pc][0], part[pc][1], part[pc][2], part[pc][3]);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, A), __builtin_bit_cast(bf16x8_t, B), acc, 0, 0, 0);
            }
        }
    }
    if (4 * kg < G) {
        const int m = row / kK, c = row % kK;
        float4 *dst = reinterpret_cast<float4 *>(lut) + (((size_t)bg * (G / 4) + kg) * (M / 16) + m / 16) * (kK * 16) + (size_t)c * 16 + (m & 15);
        *dst = make_float4(acc[0] * scale, acc[1] * scale, acc[2] * scale, acc[3] * scale);
    }
}

// k_score_lut: one workgroup per (sequence, KV head, group of HG = min(G, 4) heads, tile of TPT * 1024 tokens); the
// head group's table (M * 256 * HG floats) sits in LDS, a lane owns TPT tokens: M code bytes
// in, M look-ups of HG floats, HG logits out.  Bound by the code stream and the logit writes (HBM).
template <int M, int G, int TPT>
__global__ __launch_bounds__(kSliceThreads) void k_score_lut(const float *__restrict__ lut, const uint8_t *__restrict__ key_codes,
                                                             const int32_t *__restrict__ cu, float *__restrict__ scores,
                                                             float2 *__restrict__ sstat, const SliceDims a)
{
    constexpr int HG = G < 4 ? G : 4;
    constexpr int NGRP = G / HG;
    constexpr int TILE = TPT * kSliceThreads;
    constexpr int NW = kSliceThreads / 64;
    // the table at LDS address 0 (no static LDS in this kernel), the per-wavefront statistics behind it
    extern __shared__ __attribute__((aligned(16))) float tabf[];  // HG < 4: [M * 256][HG]; HG == 4: [M / 16][256][16][4]
    float2(*wstat)[HG] = reinterpret_cast<float2(*)[HG]>(tabf + M * kK * HG);  // [NW][HG]
    int id = blockIdx.x;
    const int g = id % a.Hkv;
    id /= a.Hkv;
    const int grp = id % NGRP;  // a workgroup takes one group of HG heads (eight heads: two workgroups per tile, each with its own table)
    id /= NGRP;
    const int tile = id % a.nsplit;
    const int b = id / a.nsplit;
    const int cu0 = cu[b];
    const int L = cu[b + 1] - cu0;
    const int t0 = tile * TILE;
    if (t0 >= L) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint8_t *codes = key_codes + ((size_t)cu0 * a.Hkv + (size_t)g * L) * M;
    float *srow = scores + (size_t)cu0 * a.Hq + (size_t)g * G * L;
    if (HG == 4) {  // the group's table is contiguous in memory, already in LDS order
        const float4 *src4 = reinterpret_cast<const float4 *>(lut) + (((size_t)b * a.Hkv + g) * NGRP + grp) * (M * kK);
        for (int x = tid; x < M * kK; x += kSliceThreads) reinterpret_cast<float4 *>(tabf)[x] = src4[x];
    } else {
        const float *src = lut + ((size_t)b * a.Hkv + g) * (M * kK) * G;
        for (int x = tid; x < M * kK; x += kSliceThreads)
#pragma unroll
            for (int h = 0; h < HG; ++h) tabf[x * HG + h] = src[(size_t)x * G + grp * HG + h];
    }
    __syncthreads();
    // HG == 4: every codebook of a block of 16 owns one 16-byte bank column (row = codeword), and lane l walks the
    // codebooks of a block in the order (rot + k) mod 16 with rot = l % 8 + 8 ((l / 16) % 2): the 16 lanes that a 16-byte
    // LDS read serves together then fall on 16 different columns whatever their codes (a [codebook][codeword] table
    // lets random codes collide: 12 clk per wavefront read against 6).  The token's 16 code bytes of the block are rotated
    // by rot bytes once, so that step k finds its code at byte k; xreg[k]: byte 0 = 16 x column, byte 3 = 1 (the second
    // 64 KiB block); one byte permute splices the code in as byte 1: address = 65536 block + 256 code + 16 column.
    const unsigned rot = ((unsigned)lane & 7u) + 8u * (((unsigned)lane >> 4) & 1u);
    unsigned xreg[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) xreg[k] = (((unsigned)k + rot) & 15u) * 16u | 1u << 24;
    float mx[HG], sc[TPT][HG];
#pragma unroll
    for (int h = 0; h < HG; ++h) mx[h] = -INFINITY;
    const int tfirst = t0 + tid;
#pragma unroll
    for (int k = 0; k < TPT; ++k) {
        const int tok = tfirst + k * kSliceThreads;
        const int tc = min(tok, L - 1);
        float acc[HG];
        floatx4_t accv = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int h = 0; h < HG; ++h) acc[h] = 0.f;
#pragma unroll
        for (int v = 0; v < M / 16; ++v) {  // 16 codes at a time, 8 look-ups in flight: keeps registers flat
            const uint4 c4 = reinterpret_cast<const uint4 *>(codes + (size_t)tc * M)[v];
            unsigned cw[4] = {c4.x, c4.y, c4.z, c4.w};
            if (HG == 4) {  // rotate the 16 bytes by rot: dword selects, then a byte-granular funnel shift
#pragma unroll
                for (int st = 1; st < 4; st <<= 1) {
                    unsigned t[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) t[j] = ((rot >> 2) & (unsigned)st) ? cw[(j + st) % 4] : cw[j];
#pragma unroll
                    for (int j = 0; j < 4; ++j) cw[j] = t[j];
                }
                unsigned rv[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) rv[j] = __builtin_amdgcn_alignbyte(cw[(j + 1) % 4], cw[j], rot & 3u);
#pragma unroll
                for (int j = 0; j < 4; ++j) cw[j] = rv[j];
            }
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int x = 0; x < 8; ++x) {
                    const int kk = 8 * half + x;
                    if (HG == 4) {  // one 16-byte read, added as a vector right away
                        const unsigned sel = 0x0c000000u | (unsigned)(2 + v) << 16 | (unsigned)(4 + kk % 4) << 8;
                        const unsigned addr = __builtin_amdgcn_perm(cw[kk / 4], xreg[kk], sel);
                        const uint4_t e = lds_read_b128(addr);
                        accv += __builtin_bit_cast(floatx4_t, e);
                    } else {
                        const int m = 16 * v + kk;
                        const unsigned c = (cw[kk / 4] >> (8 * (kk % 4))) & 0xffu;
                        const float *e = tabf + ((size_t)m * kK + c) * HG;
#pragma unroll
                        for (int h = 0; h < HG; ++h) acc[h] += e[h];
                    }
                }
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        if (HG == 4) {
#pragma unroll
            for (int h = 0; h < HG; ++h) acc[h] = accv[h];
        }
#pragma unroll
        for (int h = 0; h < HG; ++h) {
            sc[k][h] = acc[h];
            if (tok < L) {
                srow[(size_t)(grp * HG + h) * L + tok] = acc[h];
                mx[h] = fmaxf(mx[h], acc[h]);
            }
        }
    }
#pragma unroll
    for (int h = 0; h < HG; ++h) {
        const float wm = wave_max(mx[h]);
        float l = 0.f;
#pragma unroll
        for (int k = 0; k < TPT; ++k)
            if (tfirst + k * kSliceThreads < L) l += __builtin_amdgcn_exp2f((sc[k][h] - wm) * kLog2e);
        l = wave_sum(l);
        if (lane == 0) wstat[wave][h] = make_float2(wm, l);
    }
    __syncthreads();
    if (tid < HG) {
        float m = -INFINITY;
        for (int w = 0; w < NW; ++w) m = fmaxf(m, wstat[w][tid].x);
        float l = 0.f;
        for (int w = 0; w < NW; ++w) {
            const float2 st = wstat[w][tid];
            if (st.x != -INFINITY) l += st.y * __builtin_amdgcn_exp2f((st.x - m) * kLog2e);
        }
        sstat[((size_t)b * a.Hq + (size_t)g * G + grp * HG + tid) * a.nsplit + tile] = make_float2(m, l);
    }
}

// ------------------------------------------------------------------ paired-code keys (App. A.1)
// The paper's own key format: per token and KV head R residual levels, each a pair (a, b) of 6-bit
// indices into ONE table of N_c' = 64 centres per level; level r contributes C[r][a] + i C[r][b]
// (Eq. def_center: per 2-D sub-space (x_a - y_b, y_a + x_b)), i.e. index form with 2R tied codebooks.
constexpr int kPairK = 64;       // centres per level
constexpr int kPairPlanes = 4;   // 8-element planes per LDS slice (4 slices cover the 16 planes of d = 128)
constexpr int kPairBlock = kPairK * 256;  // bytes of one (plane, block of 16 levels): 64 rows x 16 pieces

// Packed 12-bit pairs -> one byte per index, in the order the score kernel wants.
//   pairs : per (sequence, KV head) L records of PB = ceil(12 R / 8) bytes; pair r of a token is bits
//           12 r .. 12 r + 11 of its record (little endian), a_r = low 6 bits, b_r = high 6 bits
//   bytes : [token-unit][blk][t][16]: level 16 blk + col of type t (0 = a, 1 = b); 0 for levels >= R
// One workgroup = 256 consecutive tokens of one (sequence, KV head); their records are contiguous and
// are staged through LDS with aligned dword loads.
__global__ __launch_bounds__(256) void k_unpack_pairs(const uint8_t *__restrict__ pairs, uint8_t *__restrict__ bytes,
                                                      const int32_t *__restrict__ cu, int Hkv, int R, int PB, int NB)
{
    __shared__ unsigned stage[256 * 32 / 4 + 12];  // a few dwords of slack: threads read 9 whole dwords each
    const int b = blockIdx.y / Hkv, g = blockIdx.y % Hkv;
    const int cu0 = cu[b], L = cu[b + 1] - cu0;
    const int i0 = blockIdx.x * 256;
    if (i0 >= L) return;
    const int cnt = min(256, L - i0);
    const size_t first = ((size_t)cu0 * Hkv + (size_t)g * L + i0) * PB;  // byte offset of the first record
    const size_t lo = first & ~(size_t)3, hi = first + (size_t)cnt * PB;  // hi never passes the end of the (b, g) stream
    const unsigned skew = (unsigned)(first - lo);
    const unsigned ndw = (unsigned)((hi - lo + 3) / 4);
    for (unsigned x = threadIdx.x; x < ndw; x += 256) {
        // the last dword may reach past the stream: read it byte by byte
        const size_t at = lo + (size_t)x * 4;
        unsigned v = 0;
        if (at + 4 <= hi) v = *reinterpret_cast<const unsigned *>(pairs + at);
        else for (unsigned k = 0; at + k < hi; ++k) v |= (unsigned)pairs[at + k] << (8 * k);
        stage[x] = v;
    }
    __syncthreads();
    if ((int)threadIdx.x >= cnt) return;
    // the thread's record as aligned dwords: whole dwords out of LDS, then one byte-granular funnel shift each
    const unsigned at = skew + threadIdx.x * PB;
    const unsigned sh = at & 3u;
    unsigned raw[9], rec[8];
#pragma unroll
    for (int k = 0; k < 9; ++k) raw[k] = 4 * k < PB + 3 ? stage[(at >> 2) + k] : 0u;  // PB <= 32: 9 dwords cover any skew
#pragma unroll
    for (int k = 0; k < 8; ++k) rec[k] = __builtin_amdgcn_alignbyte(raw[k + 1], raw[k], sh);
    uint4 *dst = reinterpret_cast<uint4 *>(bytes + ((size_t)cu0 * Hkv + (size_t)g * L + i0 + threadIdx.x) * (32 * NB));
#pragma unroll
    for (int blk = 0; blk < 2; ++blk) {
        if (blk >= NB) break;
        unsigned wa[4] = {0, 0, 0, 0}, wb[4] = {0, 0, 0, 0};
#pragma unroll
        for (int col = 0; col < 16; ++col) {
            const int r = 16 * blk + col;
            if (r < R && r < 21) {
                const int bit = 12 * r;  // a pair never needs more than two dwords
                const unsigned lo = rec[bit >> 5], hi = (bit >> 5) + 1 < 8 ? rec[(bit >> 5) + 1] : 0u;
                const unsigned pr = __builtin_amdgcn_alignbit(hi, lo, (unsigned)(bit & 31)) & 0xfffu;
                wa[col >> 2] |= (pr & 63u) << (8 * (col & 3));
                wb[col >> 2] |= (pr >> 6) << (8 * (col & 3));
            }
        }
        dst[2 * blk] = make_uint4(wa[0], wa[1], wa[2], wa[3]);
        dst[2 * blk + 1] = make_uint4(wb[0], wb[1], wb[2], wb[3]);
    }
}

// Tied table [Hkv][R][64][d] bf16 -> LDS images for k_score_pair:
//   packed[g][slice][plane][blk][c][col] 16-byte pieces = elements 8 (4 slice + plane) .. +7 of centre c of
//   level 16 blk + col (zeros for levels >= R).  One thread per piece of the output.
__global__ __launch_bounds__(256) void k_prep_pairs(const uint4 *__restrict__ table, uint4 *__restrict__ packed, int Hkv,
                                                    int R, int NB)
{
    const size_t n = (size_t)Hkv * 16 * NB * kPairK * 16;
    const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= n) return;
    const int col = (int)(t & 15);
    const int c = (int)((t >> 4) % kPairK);
    size_t rest = (t >> 4) / kPairK;
    const int blk = (int)(rest % NB);
    rest /= NB;
    const int plane16 = (int)(rest % 16);  // 4 slice + plane
    const int g = (int)(rest / 16);
    const int r = 16 * blk + col;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (r < R) v = table[(((size_t)g * R + r) * kPairK + c) * 16 + plane16];
    packed[t] = v;
}

// Score kernel for paired-code keys: same scheme as k_score_mfma (codebook streamed through LDS in
// slices, gather-sum and query product on the matrix cores), with
//   * a slice = 4 planes of 8 elements of every centre of every level (NB blocks of 16 levels, one
//     bank column per level, 64 rows = centre index): 64 KiB (R <= 16) or 128 KiB (R <= 32);
//   * k-groups = (a | b) x (levels 8h .. 8h + 7): lane (n, g) gathers the centres that the a (g < 2) or
//     b (g >= 2) indices of token n select in levels 8 (g & 1) + (n + step) mod 8 of every block;
//   * a selection matrix that routes the a-sum and the b-sum of sub-space g of the plane to rows
//     4g .. 4g + 3, so that lane (n, g) receives (SA_x, SA_y, SB_x, SB_y) and forms the decoded block
//     (SA_x - SB_y, SA_y + SB_x) of Eq. def_center locally;
//   * one cross-lane head total per slice: the 4x4x1 query MFMAs of the slice's 4 planes chain into
//     one accumulator before the row / half swaps.
template <int NB, int G, int TPT>
__global__ __launch_bounds__(kSliceThreads) void k_score_pair(
    const void *__restrict__ q, const uint8_t *__restrict__ codes_all, const uint4 *__restrict__ packed,
    const int32_t *__restrict__ cu, const int32_t *__restrict__ q_pos, const float2 *__restrict__ tbl_hi,
    const float2 *__restrict__ tbl_lo, float *__restrict__ scores, float2 *__restrict__ sstat, const SliceDims a)
{
    constexpr int PL = kPairPlanes;
    constexpr int S = 16 / PL;
    constexpr int CB = 32 * NB;                      // code bytes per token
    constexpr int SLICE = PL * NB * kPairBlock;      // LDS bytes of one slice
    constexpr int TILE = TPT * kSliceThreads;
    constexpr int NW = kSliceThreads / 64;
    constexpr int NPASS = TILE / (16 * NW);
    constexpr int NHR = TILE / kLo + 1;
    constexpr int NGRP = (G + 3) / 4;
    constexpr int PARTS = 8;                          // (sub-space of a plane) x (planes 0,1 | 2,3)
    constexpr int HROW = 12;                          // 16-byte entries per coarse phase row (8 used: conflict-free reads)
    static_assert(NPASS % 2 == 0, "code double-buffer parity assumes an even number of passes");
    extern __shared__ __attribute__((aligned(16))) uint4 tab[];  // [PL][NB][64][16] pieces, then the phase factors
    float4 *elo = reinterpret_cast<float4 *>(reinterpret_cast<char *>(tab) + SLICE);  // [PARTS][64]
    float4 *ehi = elo + PARTS * kLo;                                                   // [NHR][HROW]
    float2(*wstat)[G] = reinterpret_cast<float2(*)[G]>(ehi + HROW * NHR);             // [NW][G]
    static_assert(4 * ((TILE / kLo) * 68 + 16) * 4 <= SLICE + (PARTS * kLo + HROW * NHR) * 16, "the write-out stages its logits below the statistics");

    int id = blockIdx.x;
    const int g = id % a.Hkv;
    id /= a.Hkv;
    const int tile = id % a.nsplit;
    const int b = id / a.nsplit;
    const int cu0 = cu[b];
    const int L = cu[b + 1] - cu0;
    const int t0 = tile * TILE;
    if (t0 >= L) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, gk = lane >> 4;
    const int type = gk >> 1;                         // 0: the a indices, 1: the b indices
    const int half = gk & 1;                          // levels 8 half .. 8 half + 7 of every block
    const int qpos = q_pos[b];
    const uint8_t *codes = codes_all + ((size_t)cu0 * a.Hkv + (size_t)g * L) * CB;
    const uint4 *src = packed + (size_t)g * S * (SLICE / 16);
    const __amdgpu_buffer_rsrc_t cd_rs = make_rsrc(codes, (unsigned)L * CB);
    const unsigned qesz = a.q_bf16 ? 2u : 4u;
    const __amdgpu_buffer_rsrc_t q_rs =
        make_rsrc(static_cast<const char *>(q) + ((size_t)b * a.Hq + (size_t)g * G) * kD * qesz, (unsigned)G * kD * qesz);
    constexpr int PPT = SLICE / 16 / kSliceThreads;

    // Selection operand of the structured-sparse v_smfmac_f32_16x16x64_bf16 (layout: see k_score_mfma).  Second
    // operand: two pieces per lane, both from levels of the lane's own type.  Row i = n adds element
    // e = 2 (i >> 2) + (i & 1) of both pieces of the two lanes of its type (i >> 1) & 1: first-operand lane (i, q)
    // covers the pieces of second-operand lanes 2 (q & 1), 2 (q & 1) + 1, i.e. of type q & 1 (its first piece for
    // q < 2, its second for q >= 2), and keeps 1.0 at position e % 4 of groups e / 4 and 2 + e / 4.
    uint4_t sel = {0u, 0u, 0u, 0u};
    unsigned sidx = 0x44444444u;  // default positions (0, 1) of every stored pair
    if ((gk & 1) == ((n >> 1) & 1)) {
        const int e = 2 * (n >> 2) + (n & 1);
        const int t = e >> 2, pos = e & 3, other = pos == 0 ? 1 : 0;
        sel[t] = 0x00003f80u;
        sel[2 + t] = 0x00003f80u;
        const unsigned pair = (unsigned)pos | (unsigned)other << 2;
        sidx = (sidx & ~(0xfu << (4 * t)) & ~(0xfu << (4 * (2 + t)))) | pair << (4 * t) | pair << (4 * (2 + t));
        sidx = (sidx & 0xffffu) | sidx << 16;
    }
    const bf16x8_t selv = __builtin_bit_cast(bf16x8_t, sel);

    float sc[NPASS][NGRP][1];
#pragma unroll
    for (int p = 0; p < NPASS; ++p)
#pragma unroll
        for (int x = 0; x < NGRP; ++x) sc[p][x][0] = 0.f;

    // xreg[st]: byte 0 = 16 * bank column (= level within the block) read at step st, byte 2 = 0, byte 3 = 1;
    // a byte permute splices the centre index in as byte 1: address = 256 c + 16 col (+ 65536 via byte 3)
    unsigned xreg[8];
#pragma unroll
    for (int st = 0; st < 8; ++st) xreg[st] = (unsigned)(8 * half + ((n + st) & 7)) * 16u | 1u << 24;
    unsigned rsel_lo = 0u, rsel_hi = 0u;
#pragma unroll
    for (int x = 0; x < 4; ++x) {
        rsel_lo |= (unsigned)((x + n) & 7) << (8 * x);
        rsel_hi |= (unsigned)((x + 4 + n) & 7) << (8 * x);
    }

    // Token mapping as in k_score_mfma (M = 16): lane n of a wavefront's 16 token lanes takes fine position
    // 4 wave + n / 4 and coarse row n % 4 of the pass's block of four rows, so the lanes of a 4-lane block and all
    // passes of a lane are whole coarse rows apart and share the fine phase factor, which is folded into the query.
    int tb = t0 + 4 * wave + (n >> 2) + kLo * (n & 3);
    constexpr int PSTRIDE = 4 * kLo;
    unsigned cw[2][2 * NB];
    auto fetch_codes = [&](int p, unsigned(&dst)[2 * NB]) {
        const int tok = min(tb + p * PSTRIDE, L - 1);
#pragma unroll
        for (int v = 0; v < NB; ++v) {  // bytes 32 v + 16 type + 8 half .. + 7 of the token's indices
            const uint2_t c2 = __builtin_amdgcn_raw_buffer_load_b64(cd_rs, (unsigned)tok * CB + 32u * v + 16u * type + 8u * half, 0, 0);
            dst[2 * v + 0] = c2[0]; dst[2 * v + 1] = c2[1];
        }
    };
    // rotated index bytes of a pass: what its gather addresses are made from
    auto make_cc = [&](const unsigned(&c)[2 * NB], unsigned(&cc)[2 * NB]) {
#pragma unroll
        for (int v = 0; v < NB; ++v) {
            cc[2 * v + 0] = __builtin_amdgcn_perm(c[2 * v + 1], c[2 * v], rsel_lo);
            cc[2 * v + 1] = __builtin_amdgcn_perm(c[2 * v + 1], c[2 * v], rsel_hi);
        }
    };
    fetch_codes(0, cw[0]);
    const int hmin = (qpos - (t0 + TILE - 1)) >> kLoBits;
    const unsigned elo_base = (unsigned)SLICE + (unsigned)(2 * gk) * (kLo * 16u);
    const unsigned ehi_base = (unsigned)SLICE + (unsigned)(PARTS * kLo) * 16u + (unsigned)gk * 16u;

    for (int sl = 0; sl < S; ++sl) {
        // queries of this slice (head 4 grp + n % 4, sub-space gk of each of the 4 planes): requested ahead of the
        // slice itself, so that they have arrived when the first pass needs them
        uint2_t qraw[NGRP][PL];
#pragma unroll
        for (int x = 0; x < NGRP; ++x)
#pragma unroll
            for (int pl = 0; pl < PL; ++pl) {
                const unsigned off = (unsigned)(4 * x + (n & 3)) * kD + 2u * (unsigned)(16 * sl + 4 * pl + gk);  // elements
                if (a.q_bf16) {
                    qraw[x][pl][0] = __builtin_amdgcn_raw_buffer_load_b32(q_rs, off * 2u, 0, 0);
                    qraw[x][pl][1] = 0u;
                } else {
                    qraw[x][pl] = __builtin_amdgcn_raw_buffer_load_b64(q_rs, off * 4u, 0, 0);
                }
            }
        __syncthreads();  // everyone is done reading the previous slice
        {
            uint4 stage[PPT];
#pragma unroll
            for (int x = 0; x < PPT; ++x) stage[x] = src[(size_t)sl * (SLICE / 16) + x * kSliceThreads + tid];
#pragma unroll
            for (int x = 0; x < PPT; ++x) tab[x * kSliceThreads + tid] = stage[x];
        }
        // phase factors of this slice's 16 sub-spaces: an entry (s, h) holds sub-space s of planes 2h and 2h + 1;
        // fine table [2 s + h][64 positions], coarse table [row][4 h + s] (rows padded to 12 entries, so that the four
        // rows x four sub-spaces that the lanes of a read touch are 16 different 16-byte bank groups)
        if (tid < PARTS * kLo) {
            const int part = tid / kLo, lo = tid % kLo;
            const int j0 = 16 * sl + 8 * (part & 1) + (part >> 1);
            const float2 e0 = tbl_lo[(size_t)lo * kJ + j0], e1 = tbl_lo[(size_t)lo * kJ + j0 + 4];
            elo[tid] = make_float4(e0.x, e0.y, e1.x, e1.y);
        }
        for (int x = tid; x < PARTS * NHR; x += kSliceThreads) {
            const int c = x % PARTS, H = hmin + x / PARTS;
            const int hi = min(H < 0 ? -H : H, a.n_hi - 1);
            const int j0 = 16 * sl + 8 * (c >> 2) + (c & 3);
            const float2 e0 = tbl_hi[(size_t)hi * kJ + j0], e1 = tbl_hi[(size_t)hi * kJ + j0 + 4];
            const float sg = H < 0 ? -1.f : 1.f;
            ehi[(x / PARTS) * HROW + c] = make_float4(e0.x, sg * e0.y, e1.x, sg * e1.y);
        }
        __syncthreads();
        asm volatile("" : "+v"(tb));
        const int dist16 = (qpos - tb) * 16;
        // scaled queries of this slice, times the conjugate of the fine phase factor (shared by the lane's tokens of all
        // passes and by the four lanes of its block): q' = q conj(E_lo), Re(conj(q) k E_hi E_lo) = Re(conj(q') k E_hi)
        float qrow[NGRP][PL][2];
        {
            uint4_t elr[2];
#pragma unroll
            for (int h = 0; h < 2; ++h) elr[h] = lds_read_b128(elo_base + (unsigned)(dist16 & ((kLo - 1) * 16)) + (unsigned)(h * (kLo * 16)));
#pragma unroll
            for (int x = 0; x < NGRP; ++x)
#pragma unroll
                for (int pl = 0; pl < PL; ++pl) {
                    const unsigned u0 = qraw[x][pl][0], u1 = qraw[x][pl][1];
                    float qx, qy;
                    if (a.q_bf16) {
                        qx = bf16_lo(u0) * a.scale; qy = bf16_hi(u0) * a.scale;
                    } else {
                        qx = __builtin_bit_cast(float, u0) * a.scale; qy = __builtin_bit_cast(float, u1) * a.scale;
                    }
                    const unsigned lxr = elr[pl / 2][2 * (pl & 1)], lyr = elr[pl / 2][2 * (pl & 1) + 1];
                    const float lx = __builtin_bit_cast(float, lxr), ly = __builtin_bit_cast(float, lyr);
                    qrow[x][pl][0] = qx * lx + qy * ly;
                    qrow[x][pl][1] = qy * lx - qx * ly;
                }
        }
        // coarse phase row of the lane's token of the LAST pass; a pass is a whole number of rows further on
        const unsigned ehi_last = ehi_base + (unsigned)(((dist16 >> (kLoBits + 4)) - hmin - (NPASS - 1) * (PSTRIDE / kLo)) * (16 * HROW));
        // Gather: 8 NB pieces per lane and plane, in groups of RG reads; the groups of all planes of a pass form one
        // sequence, and a group's reads are issued before the matrix instructions of the group before it -- across
        // planes and passes, so that the first reads of the next plane (pass) travel while this one is rotated and
        // contracted with the queries.
        constexpr int NS = 8 * NB, RG = (NB == 2 || G == 8) ? 2 : 4, NG = NS / RG, NFLAT = PL * NG;  // fewer reads in flight where registers are short
        static_assert(NFLAT % 2 == 0, "read buffers alternate across passes");
        uint4_t v[2][RG];
        auto issue = [&](int flat, const unsigned(&cc)[2 * NB], uint4_t(&dst)[RG]) {
            const int pl = flat / NG, grp = flat % NG;
#pragma unroll
            for (int r = 0; r < RG; ++r) {
                const int st = grp * RG + r;       // level 16 (st / 8) + 8 half + (n + st) mod 8
                const int idx = pl * NB + st / 8;  // (plane, block) image of 16 KiB
                const unsigned selb = 0x0c000000u | (unsigned)(2 + idx / 4) << 16 | (unsigned)(4 + st % 4) << 8;
                const unsigned addr = __builtin_amdgcn_perm(cc[st / 4], xreg[st % 8], selb);
                dst[r] = lds_read_b128((unsigned)((idx % 4) * kPairBlock) + addr);
            }
        };
        unsigned cc[2 * NB];
        make_cc(cw[0], cc);  // (the last pass of the previous slice requested the codes of pass 0 again)
        issue(0, cc, v[0]);
#pragma unroll
        for (int p = 0; p < NPASS; ++p) {
            __builtin_amdgcn_sched_barrier(0);  // one pass at a time: keeps register pressure flat
            fetch_codes((p + 1) % NPASS, cw[(p + 1) & 1]);
            uint4_t ehr[2];
#pragma unroll
            for (int h = 0; h < 2; ++h)
                ehr[h] = lds_read_b128(ehi_last + (unsigned)((NPASS - 1 - p) * (PSTRIDE / kLo) * (16 * HROW) + h * 64));
            __builtin_amdgcn_sched_barrier(0);
            unsigned ccn[2 * NB];
            floatx4_t t[NGRP];
#pragma unroll
            for (int x = 0; x < NGRP; ++x) t[x] = floatx4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int pl = 0; pl < PL; ++pl) {
                // 1. gather-sum of the plane
                floatx4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int grp = 0; grp < NG; ++grp) {
                    const int flat = pl * NG + grp;
                    if (flat + 1 < NFLAT) {
                        issue(flat + 1, cc, v[(flat + 1) & 1]);
                    } else if (p + 1 < NPASS) {
                        make_cc(cw[(p + 1) & 1], ccn);
                        issue(0, ccn, v[(flat + 1) & 1]);
                    }
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int r = 0; r < RG; r += 2) {
                        const uint4_t pa = v[flat & 1][r], pb = v[flat & 1][r + 1];
                        const uint8v_t both = {pa[0], pa[1], pa[2], pa[3], pb[0], pb[1], pb[2], pb[3]};
                        acc = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(selv, __builtin_bit_cast(bf16x16_t, both), acc, (int)sidx, 0, 0);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
                // 2. decoded block of sub-space gk (Eq. def_center), rotated by the coarse phase factor
                const unsigned hxr = ehr[pl / 2][2 * (pl & 1)], hyr = ehr[pl / 2][2 * (pl & 1) + 1];
                const float ex = __builtin_bit_cast(float, hxr), ey = __builtin_bit_cast(float, hyr);
                const float kx = acc[0] - acc[3], ky = acc[1] + acc[2];
                const float bx = kx * ex - ky * ey;
                const float by = kx * ey + ky * ex;
                // 3. partial logits of 4 heads at a time; chained over the planes of the slice
#pragma unroll
                for (int x = 0; x < NGRP; ++x) {
                    t[x] = __builtin_amdgcn_mfma_f32_4x4x1f32(qrow[x][pl][0], bx, t[x], 0, 0, 0);
                    t[x] = __builtin_amdgcn_mfma_f32_4x4x1f32(qrow[x][pl][1], by, t[x], 0, 0, 0);
                }
            }
            // totals over the 4 lanes of the token: lane (n, gk) keeps head 4 grp + gk
#pragma unroll
            for (int x = 0; x < NGRP; ++x) sc[p][x][0] += swap16_add(swap32_add(t[x][0], t[x][2]), swap32_add(t[x][1], t[x][3]));
            if (p + 1 < NPASS) {
#pragma unroll
                for (int i = 0; i < 2 * NB; ++i) cc[i] = ccn[i];
            }
        }
    }

    float *srow = scores + (size_t)cu0 * a.Hq + (size_t)g * G * L;
    float2 *stat_dst = sstat + ((size_t)b * a.Hq + (size_t)g * G) * a.nsplit + tile;
    write_tile_logits<16, G, TPT, NPASS, NGRP, 1>(sc, reinterpret_cast<float *>(tab), wstat, srow, stat_dst, a.nsplit, tb, t0, L);
}

// ------------------------------------------------------------------ k_bins
struct BinsArgs {
    const uint8_t *val_codes;
    const int32_t *cu;
    const float *scores;
    const float2 *sstat;
    unsigned *bins;
    float *vscale, *lsum;
    int Hq, Hkv, nsplit, split_len;  // score-stage split geometry (for the statistics)
    int nvsplit, vsplit_len;
    int Gtot;  // query heads per KV head; a workgroup handles G of them (all, unless their bins exceed the LDS)
};

// One thread per token: w = exp(logit - max) for the G heads of the group, then M_v * G
// integer atomic adds into LDS bins indexed by the token's value codes (index form of
// Softmax(A) S_V).  w is added as round(w * 2^S): the score stage already produced the
// exp-sum l of this split (relative to the sequence maximum), every bin is bounded by it, so
// S = 30 - floor(log2 l) keeps every bin below 2^31 while the rounding error of the whole
// split stays below (tokens in split) * 2^-31 of its weight (half a unit per token, a unit being at most 2^-30 of the exp-sum).  Integer adds commute, so the
// result does not depend on the order in which wavefronts arrive.
template <int M, int G>
__global__ __launch_bounds__(kBinsThreads) void k_bins(BinsArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned bins[];  // G * M * K; for G >= 2 used as 64-bit pairs
    __shared__ float eoff_s[G];
    int id = blockIdx.x;
    const int g = id % a.Hkv;
    id /= a.Hkv;
    const int ngrp = a.Gtot / G;
    const int h0 = g * a.Gtot + (id % ngrp) * G;  // first of the G query heads of this workgroup
    id /= ngrp;
    const int vs = id % a.nvsplit;
    const int b = id / a.nvsplit;
    const int cu0 = a.cu[b];
    const int L = a.cu[b + 1] - cu0;
    const int v0 = vs * a.vsplit_len;
    if (v0 >= L) return;
    const int v1 = min(v0 + a.vsplit_len, L);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    constexpr int NB = G * M * kK;

    // For G >= 2 the bins of heads 2p and 2p + 1 share one 64-bit word (low / high half): one 64-bit LDS
    // atomic then serves two heads.  Each half stays below 2^31 (see above), so no carry crosses.
    // LDS layout [K codewords][G/2 pairs][M codebooks]: a 64-bit LDS operation is served 16 lanes at a time, and
    // 16 lanes that update the same pair of 16 consecutive codebooks (cyclically) touch 16 consecutive 8-byte
    // words -- 16 different bank pairs whatever their codes, where a [codebook][codeword] layout lets random
    // codes collide.  The pair is an immediate offset, so an atomic costs no address arithmetic of its own.
    constexpr int NP = G >= 2 ? G / 2 : 1;
    // The token's codes and logits are fetched one iteration ahead (the first before the statistics below), so
    // that their latency runs under the previous token's atomics.
    const uint8_t *codes = a.val_codes + ((size_t)cu0 * a.Hkv + (size_t)g * L) * M;
    const float *srow = a.scores + (size_t)cu0 * a.Hq + (size_t)h0 * L;
    uint4 cnext[M / 16];
    float snext[G];
#define COMMVQ_BINS_FETCH(i_)                                                                            \
    do {                                                                                                 \
        const uint4 *cp_ = reinterpret_cast<const uint4 *>(codes + (size_t)(i_) * M);                    \
        _Pragma("unroll") for (int v = 0; v < M / 16; ++v) cnext[v] = cp_[v];                            \
        _Pragma("unroll") for (int hh = 0; hh < G; ++hh) snext[hh] = srow[(size_t)hh * L + (i_)];        \
    } while (0)
    if (v0 + tid < v1) COMMVQ_BINS_FETCH(v0 + tid);
    for (int x = tid; x < NB / 4; x += kBinsThreads) reinterpret_cast<uint4 *>(bins)[x] = make_uint4(0u, 0u, 0u, 0u);
    if (wave < G) {
        const int ns = min((L + a.split_len - 1) / a.split_len, a.nsplit);
        const float2 *st = a.sstat + ((size_t)b * a.Hq + h0 + wave) * a.nsplit;
        // the first 64 splits' statistics stay in registers: one round of loads serves both passes
        const float2 first = lane < ns ? st[lane] : make_float2(-INFINITY, 0.f);
        float mx = first.x;  // maximum logit of head h0 + wave over the whole sequence
        for (int s = lane + 64; s < ns; s += 64) mx = fmaxf(mx, st[s].x);
        mx = wave_max(mx);
        // Sum of exp(logit - mx) over the score tiles that this value split touches: it bounds every bin of the split
        // (it IS the split's own sum when the split is a whole number of tiles) and fixes the fixed-point unit.  What
        // the split reports towards the softmax denominator (lown) are the tiles that BEGIN inside it, so that a tile
        // shared by several value splits is counted once.
        const int sa = v0 / a.split_len, sb = min((v1 + a.split_len - 1) / a.split_len, ns);
        float l = 0.f, lown = 0.f;
        if (lane >= sa && lane < sb) {
            l = first.y * __builtin_amdgcn_exp2f((first.x - mx) * kLog2e);
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
        if (l >= 1e-30f) S = min(30 - ilogbf(l), 120);
        if (lane == 0) {
            eoff_s[wave] = (float)S - mx * kLog2e;
            a.vscale[((size_t)b * a.Hq + h0 + wave) * a.nvsplit + vs] = ldexpf(1.f, -S);
            a.lsum[((size_t)b * a.Hq + h0 + wave) * a.nvsplit + vs] = lown;
        }
    }
    __syncthreads();
    float eoff[G];
#pragma unroll
    for (int hh = 0; hh < G; ++hh) eoff[hh] = eoff_s[hh];

    constexpr int CW = M / 4;
    const unsigned rot = (unsigned)lane & (unsigned)(M - 1);
    typedef __attribute__((address_space(3))) unsigned long long *lds_u64_ptr;
    const unsigned bins_base = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned *)bins;
    for (int i = v0 + tid; i < v1; i += kBinsThreads) {
        unsigned cw[M / 4];
#pragma unroll
        for (int v = 0; v < M / 16; ++v) {
            const uint4 c4 = cnext[v];
            cw[4 * v + 0] = c4.x; cw[4 * v + 1] = c4.y; cw[4 * v + 2] = c4.z; cw[4 * v + 3] = c4.w;
        }
        unsigned p[G];
#pragma unroll
        for (int hh = 0; hh < G; ++hh)
            p[hh] = (unsigned)(__builtin_amdgcn_exp2f(snext[hh] * kLog2e + eoff[hh]) + 0.5f);
        if (i + kBinsThreads < v1) COMMVQ_BINS_FETCH(i + kBinsThreads);
        asm volatile("" ::: "memory");  // keeps the compiler from sinking the fetch below the atomics
        // Lane l walks the codebooks in the order (l + k) % M, so that at every step the 64 lanes spread over
        // all M codebooks (bank columns, see above; skewed code usage would otherwise also put a dozen lanes on
        // the same LDS address in one instruction).  The code vector is rotated by `rot` bytes once per token
        // (dword selects + alignbyte).
#pragma unroll
        for (int st = 1; st < CW; st <<= 1) {
            unsigned t[CW];
#pragma unroll
            for (int j = 0; j < CW; ++j) t[j] = ((rot >> 2) & st) ? cw[(j + st) % CW] : cw[j];
#pragma unroll
            for (int j = 0; j < CW; ++j) cw[j] = t[j];
        }
        unsigned rv[CW];
#pragma unroll
        for (int j = 0; j < CW; ++j) rv[j] = __builtin_amdgcn_alignbyte(cw[(j + 1) % CW], cw[j], rot & 3u);
        unsigned long long pp[NP];
        if (G >= 2) {
#pragma unroll
            for (int hp = 0; hp < NP; ++hp) pp[hp] = (unsigned long long)p[(2 * hp) % G] | (unsigned long long)p[(2 * hp + 1) % G] << 32;
        }
#pragma unroll
        for (int k = 0; k < M; ++k) {
            const unsigned c = (rv[k / 4] >> (8 * (k % 4))) & 0xffu;
            const unsigned m = ((unsigned)k + rot) & (unsigned)(M - 1);
            if (G == 1) {
                atomicAdd(&bins[c * M + m], p[0]);
            } else {
                const unsigned ad = bins_base + c * (unsigned)(NP * M * 8) + m * 8u;
#pragma unroll
                for (int hp = 0; hp < NP; ++hp)
                    __hip_atomic_fetch_add(reinterpret_cast<lds_u64_ptr>(ad + (unsigned)(hp * M * 8)), pp[hp], __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_WORKGROUP);
            }
        }
    }
#undef COMMVQ_BINS_FETCH
    __syncthreads();
    // memory layout [K][M][Gtot] 32-bit bins (heads innermost: a pair's two halves are heads 2p, 2p + 1)
    unsigned *dst = a.bins + ((size_t)(b * a.Hkv + g) * a.nvsplit + vs) * (size_t)(a.Gtot * M * kK) + (h0 - g * a.Gtot);
    if (G == 1) {
        if (a.Gtot == 1) {
            for (int x = tid; x < NB / 4; x += kBinsThreads)
                reinterpret_cast<uint4 *>(dst)[x] = reinterpret_cast<const uint4 *>(bins)[x];
        } else {
            for (int x = tid; x < NB; x += kBinsThreads) dst[(size_t)x * a.Gtot] = bins[x];
        }
    } else {
        const uint2 *src = reinterpret_cast<const uint2 *>(bins);  // [K][NP][M] pairs
        for (int x = tid; x < kK * M; x += kBinsThreads) {
            const int c = x / M, m = x % M;
            uint2 v[NP];
#pragma unroll
            for (int hp = 0; hp < NP; ++hp) v[hp] = src[(c * NP + hp) * M + m];
            unsigned *row = dst + (size_t)x * a.Gtot;  // 8-byte aligned for G = 2, 16-byte aligned for G >= 4
            if (NP == 1) {
                *reinterpret_cast<uint2 *>(row) = v[0];
            } else {
#pragma unroll
                for (int hp = 0; hp < NP; hp += 2)
                    *reinterpret_cast<uint4 *>(row + 2 * hp) = make_uint4(v[hp].x, v[hp].y, v[(hp + 1) % NP].x, v[(hp + 1) % NP].y);
            }
        }
    }
}

// ------------------------------------------------------------------ k_out
struct OutArgs {
    const void *val_cb;
    const int32_t *cu;
    const unsigned *bins;
    const float *vscale, *lsum;
    float *partial, *out;
    int Hq, Hkv, nvsplit, vsplit_len, nchunk, Mv;
    int batch;
    // Index form: bins row r of a KV head = codeword r / M_v of codebook r % M_v, whose value-codebook row (of d
    // elements) is g * M_v K + (r % M_v) * K + r / M_v.  Binary code (cb_linear): bins row r = code bit c =
    // vbits_code_bit(r), codebook [N_c][Hkv * d], row of d elements c * Hkv + g.
    int cb_linear;
};

// Workgroup = (sequence, KV head, chunk of codebook rows): sums the chunk's bins over the
// context splits (fixed point -> fp32 with each split's unit), then multiplies them with the
// chunk's value-codebook rows (Eq. optimized_v).
template <int G, bool BF16>
__global__ __launch_bounds__(kOutThreads) void k_out(OutArgs a)
{
    __shared__ float wsum[G][kOutRows];
    __shared__ float red[kOutThreads / 64][G][kD];
    __shared__ float scl[G][kMaxValueSplits];                       // value of one fixed-point unit, per head and split
    __shared__ float part[kOutThreads / kOutRows][kOutRows][G];     // sums over every fourth split
    int id = blockIdx.x;
    const int chunk = id % a.nchunk;
    id /= a.nchunk;
    const int g = id % a.Hkv;
    const int b = id / a.Hkv;
    const int L = a.cu[b + 1] - a.cu[b];
    const int nvs = min((L + a.vsplit_len - 1) / a.vsplit_len, a.nvsplit);
    const int MK = a.Mv * kK;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    // bins: [split][K][Mv][G]; the chunk's 64 rows are kOutRows / Mv consecutive codewords of every codebook, one
    // contiguous run of 64 * G bins per split; local row r = (codeword - first) * Mv + codebook.  A thread reads
    // the G bins of its row with one vector load and takes every fourth split.
    constexpr int NSG = kOutThreads / kOutRows;
    constexpr int NCR = kOutRows / (kOutThreads / 64);  // codebook rows per wavefront
    const int r1 = tid % kOutRows, sg = tid / kOutRows;
    const unsigned *src = a.bins + (size_t)(b * a.Hkv + g) * a.nvsplit * G * MK + (size_t)(chunk * kOutRows + r1) * G;
    auto load_bins = [&](int v, unsigned(&bv)[G]) {
        const unsigned *pv = src + (size_t)v * G * MK;
        if (G >= 4) {
#pragma unroll
            for (int q4 = 0; q4 < G / 4; ++q4) {
                const uint4 t4 = reinterpret_cast<const uint4 *>(pv)[q4];
                bv[4 * q4 + 0] = t4.x; bv[4 * q4 + 1 < G ? 4 * q4 + 1 : 0] = t4.y; bv[4 * q4 + 2 < G ? 4 * q4 + 2 : 0] = t4.z; bv[4 * q4 + 3 < G ? 4 * q4 + 3 : 0] = t4.w;
            }
        } else if (G == 2) {
            const uint2 t2 = *reinterpret_cast<const uint2 *>(pv);
            bv[0] = t2.x; bv[G - 1] = t2.y;
        } else {
            bv[0] = pv[0];
        }
    };
    // a wavefront takes a quarter of the codebooks and the chunk's codewords of each: runs of consecutive rows
    const int cpc = kOutRows / a.Mv, mpw = a.Mv / (kOutThreads / 64);  // codewords per chunk, codebooks per wavefront
    auto load_row = [&](int i) -> float2 {
        const int m = wave * mpw + i / cpc, cl = i % cpc;
        const size_t row = a.cb_linear ? (size_t)vbits_code_bit(chunk * kOutRows + cl * a.Mv + m) * a.Hkv + g
                                       : (size_t)g * MK + (size_t)m * kK + (size_t)chunk * cpc + cl;
        if (BF16) {
            const unsigned v = static_cast<const unsigned *>(a.val_cb)[row * kJ + lane];
            return make_float2(bf16_lo(v), bf16_hi(v));
        }
        return static_cast<const float2 *>(a.val_cb)[row * kJ + lane];
    };
    for (int x = tid; x < G * nvs; x += kOutThreads)
        scl[x / nvs][x % nvs] = a.vscale[((size_t)b * a.Hq + (size_t)g * G + x / nvs) * a.nvsplit + x % nvs];
    __syncthreads();
    {
        float s[G];
#pragma unroll
        for (int hh = 0; hh < G; ++hh) s[hh] = 0.f;
        // eight splits' bins in flight where a thread has that many and the registers allow, else four (same order of
        // additions either way)
        int v = sg;
        if (G <= 4 && nvs >= 8 * NSG) {
            for (; v + 7 * NSG < nvs; v += 8 * NSG) {
                unsigned bv[8][G];
#pragma unroll
                for (int k = 0; k < 8; ++k) load_bins(v + k * NSG, bv[k]);
#pragma unroll
                for (int k = 0; k < 8; ++k)
#pragma unroll
                    for (int hh = 0; hh < G; ++hh) s[hh] += (float)bv[k][hh] * scl[hh][v + k * NSG];
            }
        }
#pragma unroll 4
        for (; v < nvs; v += NSG) {
            unsigned bv[G];
            load_bins(v, bv);
#pragma unroll
            for (int hh = 0; hh < G; ++hh) s[hh] += (float)bv[hh] * scl[hh][v];
        }
#pragma unroll
        for (int hh = 0; hh < G; ++hh) part[sg][r1][hh] = s[hh];
    }
    __syncthreads();
    for (int x = tid; x < G * kOutRows; x += kOutThreads) {
        const int hh = x % G, r = x / G;
        float s = 0.f;
#pragma unroll
        for (int q = 0; q < NSG; ++q) s += part[q][r][hh];
        wsum[hh][r] = s;
    }
    __syncthreads();
    float2 acc[G];
#pragma unroll
    for (int hh = 0; hh < G; ++hh) acc[hh] = make_float2(0.f, 0.f);
    // (unrolled: the wavefront's 16 row loads are requested together)
#pragma unroll
    for (int i = 0; i < NCR; ++i) {
        const int m = wave * mpw + i / cpc, cl = i % cpc;
        const int r = cl * a.Mv + m;
        const float2 c = load_row(i);
#pragma unroll
        for (int hh = 0; hh < G; ++hh) {
            const float w = wsum[hh][r];
            acc[hh].x += w * c.x;
            acc[hh].y += w * c.y;
        }
    }
#pragma unroll
    for (int hh = 0; hh < G; ++hh) {
        red[wave][hh][2 * lane] = acc[hh].x;
        red[wave][hh][2 * lane + 1] = acc[hh].y;
    }
    __syncthreads();
    for (int x = tid; x < G * kD; x += kOutThreads) {
        const int hh = x / kD, e = x % kD;
        float s = 0.f;
        for (int w = 0; w < kOutThreads / 64; ++w) s += red[w][hh][e];
        a.partial[(((size_t)b * a.Hq + (size_t)g * G + hh) * a.nchunk + chunk) * kD + e] = s;
    }
}

// Value codebook re-laid for k_out_mfma: vp[g][kt][dim][32] bf16, where row 32 kt + j of head g is codeword
// (32 kt + j) / M_v of codebook (32 kt + j) % M_v (the row order of the bins) -- the 32 rows of a k-step of the matrix
// instruction contiguous per output dimension.  One thread per 16-byte piece of the output (static data, done once).
__global__ __launch_bounds__(256) void k_prep_values(const uint16_t *__restrict__ val_cb, uint4 *__restrict__ vp, int Hkv, int Mv,
                                                     int linear)
{
    const int MK = Mv * kK;
    const size_t n = (size_t)Hkv * (MK / 32) * kD * 4;
    const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= n) return;
    const int kg = (int)(t & 3), dim = (int)((t >> 2) % kD);
    const size_t rest = (t >> 2) / kD;
    const int kt = (int)(rest % (MK / 32)), g = (int)(rest / (MK / 32));
    unsigned w[4];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int r = 32 * kt + 8 * kg + e;
        const unsigned v = linear ? val_cb[((size_t)vbits_code_bit(r) * Hkv + g) * kD + dim]  // binary code: [N_c][Hkv * d]
                                  : val_cb[(((size_t)g * Mv + r % Mv) * kK + r / Mv) * kD + dim];
        if (e & 1) w[e / 2] |= v << 16; else w[e / 2] = v;
    }
    vp[t] = make_uint4(w[0], w[1], w[2], w[3]);
}

// The output stage for batches (Eq. optimized_v's bins x C_V as what it is for several sequences, a matrix product):
// per KV head, [sequences x query heads] x [M_v K rows] times [rows] x [d].  A workgroup takes 16 output rows
// (16 / G sequences), kOutMfmaRows codebook rows and all d columns: it sums the fixed-point bins of its rows over the
// value splits (fp32, each split's unit applied), splits every fp32 weight EXACTLY into three bf16 parts (24 mantissa
// bits = 8 + 8 + 8) and multiplies them with the bf16 codebook by v_mfma_f32_16x16x32_bf16, accumulating in fp32: the
// fp32 product up to summation order, at a tenth of the vector instructions.  Each wavefront takes 32 of the 128 columns;
// the codebook comes straight from memory in the k_prep_values order (16 bytes per lane = 8 consecutive rows of one
// column), read once per 16 output rows instead of once per sequence.
template <int G>
__global__ __launch_bounds__(kOutThreads) void k_out_mfma(OutArgs a, const uint4 *__restrict__ vp)
{
    constexpr int KC = kOutMfmaRows, SPT = 16 / G, WS = KC + 8;  // (row stride padded: the 16 rows fall on different banks)
    __shared__ __attribute__((aligned(16))) uint16_t Wl[3][16][WS];
    int id = blockIdx.x;
    const int chunk = id % a.nchunk;
    id /= a.nchunk;
    const int g = id % a.Hkv;
    const int b0 = (id / a.Hkv) * SPT;
    const int MK = a.Mv * kK;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int it = tid; it < SPT * KC; it += kOutThreads) {
        const int sq = it / KC, k = it % KC, b = b0 + sq;
        float w[G];
#pragma unroll
        for (int hh = 0; hh < G; ++hh) w[hh] = 0.f;
        if (b < a.batch) {
            const int L = a.cu[b + 1] - a.cu[b];
            const int nvs = min((L + a.vsplit_len - 1) / a.vsplit_len, a.nvsplit);
            const unsigned *src = a.bins + (size_t)(b * a.Hkv + g) * a.nvsplit * G * MK + (size_t)(chunk * KC + k) * G;
            const float *scl = a.vscale + ((size_t)b * a.Hq + (size_t)g * G) * a.nvsplit;
#pragma unroll 4
            for (int v = 0; v < nvs; ++v) {
                const unsigned *pv = src + (size_t)v * G * MK;
                unsigned bv[G];
                if (G >= 4) {
#pragma unroll
                    for (int q4 = 0; q4 < G / 4; ++q4) {
                        const uint4 t4 = reinterpret_cast<const uint4 *>(pv)[q4];
                        bv[4 * q4 + 0] = t4.x; bv[4 * q4 + 1 < G ? 4 * q4 + 1 : 0] = t4.y; bv[4 * q4 + 2 < G ? 4 * q4 + 2 : 0] = t4.z; bv[4 * q4 + 3 < G ? 4 * q4 + 3 : 0] = t4.w;
                    }
                } else if (G == 2) {
                    const uint2 t2 = *reinterpret_cast<const uint2 *>(pv);
                    bv[0] = t2.x; bv[G - 1] = t2.y;
                } else {
                    bv[0] = pv[0];
                }
#pragma unroll
                for (int hh = 0; hh < G; ++hh) w[hh] += (float)bv[hh] * scl[(size_t)hh * a.nvsplit + v];
            }
        }
#pragma unroll
        for (int hh = 0; hh < G; ++hh) {
            // hi = the top 16 bits, mid = the top 16 bits of what is left, lo = the rest (exact: 8 + 8 + 8 mantissa bits)
            const unsigned u0 = __builtin_bit_cast(unsigned, w[hh]) & 0xffff0000u;
            const float r1 = w[hh] - __builtin_bit_cast(float, u0);
            const unsigned u1 = __builtin_bit_cast(unsigned, r1) & 0xffff0000u;
            const float r2 = r1 - __builtin_bit_cast(float, u1);
            const unsigned u2 = __builtin_bit_cast(unsigned, r2) & 0xffff0000u;
            Wl[0][sq * G + hh][k] = (uint16_t)(u0 >> 16);
            Wl[1][sq * G + hh][k] = (uint16_t)(u1 >> 16);
            Wl[2][sq * G + hh][k] = (uint16_t)(u2 >> 16);
        }
    }
    __syncthreads();
    // first operand: lane (i = lane % 16, kg = lane / 16) supplies weights of output row i for rows 8 kg .. 8 kg + 7 of the
    // k-step; second: lane (n, kg) the same rows of column n; result: lane (n, rg) holds rows 4 rg .. 4 rg + 3 of column n
    const int n = lane & 15, kg = lane >> 4;
    floatx4_t acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
    const uint4 *bsrc = vp + (((size_t)g * (MK / 32) + (size_t)chunk * (KC / 32)) * kD + 32 * wave + n) * 4 + kg;
#pragma unroll
    for (int kt = 0; kt < KC / 32; ++kt) {
        const uint4 B0 = bsrc[(size_t)(kt * kD) * 4], B1 = bsrc[(size_t)(kt * kD + 16) * 4];
#pragma unroll
        for (int p = 0; p < 3; ++p) {
            const uint4 A = *reinterpret_cast<const uint4 *>(&Wl[p][n][32 * kt + 8 * kg]);
            acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, A), __builtin_bit_cast(bf16x8_t, B0), acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, A), __builtin_bit_cast(bf16x8_t, B1), acc[1], 0, 0, 0);
        }
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int i = 4 * kg + r, b = b0 + i / G, hh = i % G;
        if (b < a.batch) {
            float *dst = a.partial + (((size_t)b * a.Hq + (size_t)g * G + hh) * a.nchunk + chunk) * kD + 32 * wave + n;
            dst[0] = acc[0][r];
            dst[16] = acc[1][r];
        }
    }
}

// One workgroup per (sequence, head): sum of the chunk partials in a fixed order, division
// by the softmax denominator (sum of the value splits' exp-sums).  Four threads per output element take every
// fourth chunk each, so that a thread's loads are one round of independent requests; their four sums are then
// added in a fixed order.  Measured: finishing inside k_out by a last-arriving workgroup costs more than this
// launch, because the device-scope release/acquire it needs writes back and invalidates L2.
constexpr int kFinalParts = 4;
__global__ __launch_bounds__(kD * kFinalParts) void k_out_final(OutArgs a)
{
    __shared__ float l_s;
    __shared__ float part[kFinalParts][kD];
    const int bh = blockIdx.x;
    const int b = bh / a.Hq;
    const int e = threadIdx.x % kD, q = threadIdx.x / kD;
    const float *pp = a.partial + (size_t)bh * a.nchunk * kD + e;
    float s = 0.f;
#pragma unroll 16
    for (int c = q; c < a.nchunk; c += kFinalParts) s += pp[(size_t)c * kD];
    part[q][e] = s;
    if (threadIdx.x < 64) {
        const int L = a.cu[b + 1] - a.cu[b];
        const int nvs = min((L + a.vsplit_len - 1) / a.vsplit_len, a.nvsplit);
        float l = 0.f;
        for (int v = threadIdx.x; v < nvs; v += 64) l += a.lsum[(size_t)bh * a.nvsplit + v];
        l = wave_sum(l);
        if (threadIdx.x == 0) l_s = l;
    }
    __syncthreads();
    if (q == 0) {
        float t = part[0][e];
#pragma unroll
        for (int k = 1; k < kFinalParts; ++k) t += part[k][e];
        a.out[(size_t)bh * kD + e] = l_s > 0.f ? t / l_s : 0.f;  // a sequence without context tokens: zeros
    }
}

// ------------------------------------------------------------------ host side
// What can be checked of a batch shape from host values alone.
commvq_status check_shape(const commvq_handle *h, int32_t batch, int64_t total_tokens, int32_t max_seqlen, bool explicit_positions)
{
    if (batch < 1 || max_seqlen < 1) return COMMVQ_ERR_SHAPE;
    if (total_tokens < max_seqlen) return COMMVQ_ERR_SHAPE;
    if (total_tokens > (int64_t)batch * max_seqlen) return COMMVQ_ERR_SHAPE;
    if (total_tokens > (int64_t)1 << 30) return COMMVQ_ERR_SHAPE;
    // the kernels address one (sequence, KV head)'s codes, unpacked pair indices and logits with 32-bit byte offsets
    const commvq_config &c = h->cfg;
    int64_t rec = bin_values(c) ? c.value_bits / 8 : c.m_val;
    if (pair_keys(c)) rec = std::max<int64_t>(rec, 32 * pair_blocks(c));
    else rec = std::max<int64_t>(rec, c.m_key);
    rec = std::max<int64_t>(rec, 4 * h->G);
    if ((int64_t)max_seqlen * rec > (int64_t)0xffffffffll) return COMMVQ_ERR_SHAPE;
    // keys at positions 0 .. L - 1 and the query at or after the last of them: the farthest key is at least
    // max_seqlen - 1 away, which the phase tables must cover (Eq. rope_ri is exact only inside them)
    if (!explicit_positions && !c.position_free && (int64_t)max_seqlen - 1 > c.max_position) return COMMVQ_ERR_SHAPE;
    return COMMVQ_OK;
}

commvq_status check_positions(const commvq_handle *h, const commvq_positions *p)
{
    if (!p) return COMMVQ_ERR_NULL;
    if (!p->cu_seqlens || !p->q_pos) return COMMVQ_ERR_NULL;
    return check_shape(h, p->batch, p->total_tokens, p->max_seqlen, p->key_pos != nullptr);
}

commvq_status prep(const commvq_handle *h, const commvq_positions *pos, void *workspace, size_t workspace_bytes,
                   commvq_plan *plan, Workspace *w)
{
    if (!h) return COMMVQ_ERR_NULL;
    commvq_status st = check_positions(h, pos);
    if (st != COMMVQ_OK) return st;
    if (pair_keys(h->cfg) && pos->key_pos) return COMMVQ_ERR_CONFIG;  // paired-code keys: contiguous positions only
    make_plan(h, pos->batch, pos->max_seqlen, use_sliced(h, pos->key_pos != nullptr), plan);
    carve(h, pos->batch, pos->total_tokens, pos->max_seqlen, workspace, w);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) || workspace_bytes < w->bytes)
        return COMMVQ_ERR_WORKSPACE;
    if (h->device < 0) return COMMVQ_ERR_NO_DEVICE;  // planner handle: every argument was acceptable, nothing is launched
    return COMMVQ_OK;
}

struct ScoreArgs {
    const void *q;
    const uint8_t *key_codes;
    const void *key_cb;
    const int32_t *cu, *q_pos, *key_pos;
    const float2 *tbl_hi, *tbl_lo;
    float *scores;
    float2 *sstat;
    ScoreDims d;
};

template <int M, int G>
hipError_t launch_score_mg(const ScoreArgs &a, bool bf16, int grid, hipStream_t s)
{
    if (bf16)
        hipLaunchKernelGGL((k_score<M, G, true>), dim3(grid), dim3(kScoreThreads), 0, s, a.q, a.key_codes, a.key_cb, a.cu,
                           a.q_pos, a.key_pos, a.tbl_hi, a.tbl_lo, a.scores, a.sstat, a.d);
    else
        hipLaunchKernelGGL((k_score<M, G, false>), dim3(grid), dim3(kScoreThreads), 0, s, a.q, a.key_codes, a.key_cb, a.cu,
                           a.q_pos, a.key_pos, a.tbl_hi, a.tbl_lo, a.scores, a.sstat, a.d);
    return hipGetLastError();
}
template <int M>
hipError_t launch_score_m(const ScoreArgs &a, int G, bool bf16, int grid, hipStream_t s)
{
    switch (G) {
    case 1: return launch_score_mg<M, 1>(a, bf16, grid, s);
    case 2: return launch_score_mg<M, 2>(a, bf16, grid, s);
    case 4: return launch_score_mg<M, 4>(a, bf16, grid, s);
    default: return launch_score_mg<M, 8>(a, bf16, grid, s);
    }
}

template <int M, int G>
hipError_t launch_bins_mg(BinsArgs a, int Gtot, int grid, hipStream_t s)
{
    a.Gtot = Gtot;
    grid *= Gtot / G;
    const size_t lds = (size_t)G * M * kK * sizeof(unsigned);
    static std::atomic<uint64_t> lds_ok{0};  // per instantiation and device
    if (hipError_t e = allow_dynamic_lds(&k_bins<M, G>, (int)lds, lds_ok); e != hipSuccess) return e;
    hipLaunchKernelGGL((k_bins<M, G>), dim3(grid), dim3(kBinsThreads), lds, s, a);
    return hipGetLastError();
}
template <int M>
hipError_t launch_bins_m(const BinsArgs &a, int G, int grid, hipStream_t s)
{
    switch (G) {
    case 1: return launch_bins_mg<M, 1>(a, 1, grid, s);
    case 2: return launch_bins_mg<M, 2>(a, 2, grid, s);
    case 4: return launch_bins_mg<M, 4>(a, 4, grid, s);
    default:
        // 8 heads x 32 codebooks of bins are 256 KiB, more than a compute unit's LDS: two workgroups of 4 heads
        if (M == 32) return launch_bins_mg<M, 4>(a, 8, grid, s);
        return launch_bins_mg<M, 8>(a, 8, grid, s);
    }
}

template <int G>
hipError_t launch_out_g(const OutArgs &a, bool bf16, int grid, hipStream_t s)
{
    if (bf16) hipLaunchKernelGGL((k_out<G, true>), dim3(grid), dim3(kOutThreads), 0, s, a);
    else hipLaunchKernelGGL((k_out<G, false>), dim3(grid), dim3(kOutThreads), 0, s, a);
    return hipGetLastError();
}

struct SliceArgs {
    const void *q;
    const uint8_t *key_codes;
    const uint4 *packed;
    const int32_t *cu, *q_pos;
    const float2 *tbl_hi, *tbl_lo;
    float *scores;
    float2 *sstat;
    SliceDims d;
};

template <int M, int G, int TPT>
hipError_t launch_sliced_mgt(const SliceArgs &a, int grid, hipStream_t s)
{
    static std::atomic<uint64_t> lds_ok{0};  // per instantiation and device
    if (hipError_t e = allow_dynamic_lds(&k_score_mfma<M, G, TPT>, kScoreLds, lds_ok); e != hipSuccess) return e;
    hipLaunchKernelGGL((k_score_mfma<M, G, TPT>), dim3(grid), dim3(kSliceThreads), kScoreLds, s, a.q, a.key_codes,
                       a.packed, a.cu, a.q_pos, a.tbl_hi, a.tbl_lo, a.scores, a.sstat, a.d);
    return hipGetLastError();
}
template <int M, int G>
hipError_t launch_sliced_mg(const SliceArgs &a, int tpt, int grid, hipStream_t s)
{
    switch (tpt) {
    case 1: return launch_sliced_mgt<M, G, 1>(a, grid, s);
    case 2: return launch_sliced_mgt<M, G, 2>(a, grid, s);
    default: return launch_sliced_mgt<M, G, 4>(a, grid, s);
    }
}
template <int M>
hipError_t launch_sliced_m(const SliceArgs &a, int G, int tpt, int grid, hipStream_t s)
{
    switch (G) {
    case 1: return launch_sliced_mg<M, 1>(a, tpt, grid, s);
    case 2: return launch_sliced_mg<M, 2>(a, tpt, grid, s);
    case 4: return launch_sliced_mg<M, 4>(a, tpt, grid, s);
    default: return launch_sliced_mg<M, 8>(a, tpt, grid, s);
    }
}

template <int NB, int G, int TPT>
hipError_t launch_pair_bgt(const SliceArgs &a, int grid, hipStream_t s)
{
    constexpr int tile = TPT * kSliceThreads;
    // slice + fine phase factors + coarse rows (12 entries each) + per-wavefront statistics; the write-out stages four
    // heads of the tile's logits, [64 positions padded to 68] per coarse row, over the slice and the phase factors
    constexpr int work = kPairPlanes * NB * kPairBlock + 8 * kLo * 16 + 12 * (tile / kLo + 1) * 16;
    constexpr int stg = 4 * ((tile / kLo) * 68 + 16) * 4;
    constexpr int lds = (work > stg ? work : stg) + kStatBytes;
    static std::atomic<uint64_t> lds_ok{0};  // per instantiation and device
    if (hipError_t e = allow_dynamic_lds(&k_score_pair<NB, G, TPT>, lds, lds_ok); e != hipSuccess) return e;
    hipLaunchKernelGGL((k_score_pair<NB, G, TPT>), dim3(grid), dim3(kSliceThreads), lds, s, a.q, a.key_codes, a.packed,
                       a.cu, a.q_pos, a.tbl_hi, a.tbl_lo, a.scores, a.sstat, a.d);
    return hipGetLastError();
}
template <int NB, int G>
hipError_t launch_pair_bg(const SliceArgs &a, int tpt, int grid, hipStream_t s)
{
    switch (tpt) {
    case 1: return launch_pair_bgt<NB, G, 1>(a, grid, s);
    case 2: return launch_pair_bgt<NB, G, 2>(a, grid, s);
    default: return launch_pair_bgt<NB, G, 4>(a, grid, s);
    }
}
template <int NB>
hipError_t launch_pair_b(const SliceArgs &a, int G, int tpt, int grid, hipStream_t s)
{
    switch (G) {
    case 1: return launch_pair_bg<NB, 1>(a, tpt, grid, s);
    case 2: return launch_pair_bg<NB, 2>(a, tpt, grid, s);
    case 4: return launch_pair_bg<NB, 4>(a, tpt, grid, s);
    default: return launch_pair_bg<NB, 8>(a, tpt, grid, s);
    }
}

// Re-lays a key codebook (index form) or a tied pair table into the LDS-image order of its score kernel.
hipError_t launch_prep(const commvq_config &c, const void *key_cb, uint4 *packed, hipStream_t s)
{
    const size_t n_pieces = packed_key_bytes(c) / 16;
    if (pair_keys(c))
        hipLaunchKernelGGL(k_prep_pairs, dim3((unsigned)((n_pieces + 255) / 256)), dim3(256), 0, s,
                           static_cast<const uint4 *>(key_cb), packed, c.n_kv_heads, c.key_levels, pair_blocks(c));
    else
        hipLaunchKernelGGL(k_prep, dim3((unsigned)((n_pieces + 255) / 256)), dim3(256), 0, s,
                           static_cast<const uint4 *>(key_cb), packed, c.n_kv_heads, c.m_key);
    return hipGetLastError();
}

hipError_t launch_prep_values(const commvq_config &c, const void *val_cb, uint4 *vp, hipStream_t s)
{
    const size_t n = (size_t)c.n_kv_heads * val_books(c) * kK * kD * 2 / 16;
    hipLaunchKernelGGL(k_prep_values, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, static_cast<const uint16_t *>(val_cb), vp,
                       c.n_kv_heads, val_books(c), bin_values(c) ? 1 : 0);
    return hipGetLastError();
}

template <int M, int G, int TPT>
hipError_t launch_lut_mgt(const float *lut, const uint8_t *key_codes, const int32_t *cu, float *scores, float2 *sstat,
                          const SliceDims &d, int grid, hipStream_t s)
{
    constexpr int lds = M * kK * (G < 4 ? G : 4) * 4 + (kSliceThreads / 64) * (G < 4 ? G : 4) * 8;  // table + per-wavefront statistics
    static std::atomic<uint64_t> lds_ok{0};  // per instantiation and device
    if (hipError_t e = allow_dynamic_lds(&k_score_lut<M, G, TPT>, lds, lds_ok); e != hipSuccess) return e;
    grid *= G < 4 ? 1 : G / 4;  // one workgroup per group of four heads
    hipLaunchKernelGGL((k_score_lut<M, G, TPT>), dim3(grid), dim3(kSliceThreads), lds, s, lut, key_codes, cu, scores, sstat, d);
    return hipGetLastError();
}
template <int M, int G>
hipError_t launch_lut_mg(const void *q, const void *key_cb, bool bf16, float *lut, const uint8_t *key_codes, const int32_t *cu,
                         float *scores, float2 *sstat, const SliceDims &d, int B, int tpt, int grid, hipStream_t s)
{
    const int blocks = B * d.Hkv * (M * kK / 256);
    if (bf16 && G >= 4)  // the table as a matrix product (16 rows per wavefront, 64 per workgroup)
        hipLaunchKernelGGL((k_lut_build_mfma<G>), dim3(4 * blocks), dim3(256), 0, s, q, static_cast<const uint16_t *>(key_cb), lut, d.Hkv,
                           M, d.q_bf16, d.scale);
    else if (bf16) hipLaunchKernelGGL((k_lut_build<G, true>), dim3(blocks), dim3(256), 0, s, q, key_cb, lut, d.Hkv, M, d.q_bf16, d.scale);
    else hipLaunchKernelGGL((k_lut_build<G, false>), dim3(blocks), dim3(256), 0, s, q, key_cb, lut, d.Hkv, M, d.q_bf16, d.scale);
    if (hipGetLastError() != hipSuccess) return hipErrorLaunchFailure;
    switch (tpt) {
    case 1: return launch_lut_mgt<M, G, 1>(lut, key_codes, cu, scores, sstat, d, grid, s);
    case 2: return launch_lut_mgt<M, G, 2>(lut, key_codes, cu, scores, sstat, d, grid, s);
    default: return launch_lut_mgt<M, G, 4>(lut, key_codes, cu, scores, sstat, d, grid, s);
    }
}
template <int M>
hipError_t launch_lut_m(int G, const void *q, const void *key_cb, bool bf16, float *lut, const uint8_t *key_codes,
                        const int32_t *cu, float *scores, float2 *sstat, const SliceDims &d, int B, int tpt, int grid, hipStream_t s)
{
    switch (G) {
    case 1: return launch_lut_mg<M, 1>(q, key_cb, bf16, lut, key_codes, cu, scores, sstat, d, B, tpt, grid, s);
    case 2: return launch_lut_mg<M, 2>(q, key_cb, bf16, lut, key_codes, cu, scores, sstat, d, B, tpt, grid, s);
    case 4: return launch_lut_mg<M, 4>(q, key_cb, bf16, lut, key_codes, cu, scores, sstat, d, B, tpt, grid, s);
    default: return launch_lut_mg<M, 8>(q, key_cb, bf16, lut, key_codes, cu, scores, sstat, d, B, tpt, grid, s);
    }
}

commvq_status run_scores(commvq_handle *h, const void *q, const uint8_t *key_codes, const void *key_cb,
                         const commvq_positions *pos, const commvq_plan &plan, const Workspace &w, hipStream_t s)
{
    const commvq_config &c = h->cfg;
    if (c.position_free) {  // scalar look-up table: build T = scale q C^T, then M look-ups per token
        SliceDims d;
        d.Hq = c.n_q_heads; d.Hkv = c.n_kv_heads; d.nsplit = plan.score_splits; d.n_hi = h->n_hi;
        d.q_bf16 = c.q_dtype == COMMVQ_BF16; d.scale = h->scale; d.groups = 1; d.part_stride = 0;
        const int grid = pos->batch * c.n_kv_heads * plan.score_splits;
        const int tpt = plan.score_split_len / kSliceThreads;
        const bool bf16 = c.codebook_dtype == COMMVQ_BF16;
        hipError_t e = c.m_key == 16 ? launch_lut_m<16>(h->G, q, key_cb, bf16, w.lut, key_codes, pos->cu_seqlens, w.scores, w.sstat, d, pos->batch, tpt, grid, s)
                                     : launch_lut_m<32>(h->G, q, key_cb, bf16, w.lut, key_codes, pos->cu_seqlens, w.scores, w.sstat, d, pos->batch, tpt, grid, s);
        return e == hipSuccess ? COMMVQ_OK : COMMVQ_ERR_LAUNCH;
    }
    if (plan.score_kernel) {  // slice-streaming kernel: needs the codebook in LDS-image order
        const uint4 *packed = nullptr;
        for (const auto &e : h->packed_keys)
            if (e.first == key_cb) packed = e.second;
        if (!packed) {  // not packed ahead of time: re-lay it into the workspace on every call
            if (launch_prep(c, key_cb, w.packed, s) != hipSuccess) return COMMVQ_ERR_LAUNCH;
            packed = w.packed;
        }
        SliceArgs sa;
        sa.q = q; sa.key_codes = key_codes; sa.packed = packed; sa.cu = pos->cu_seqlens; sa.q_pos = pos->q_pos;
        sa.tbl_hi = h->tbl_hi; sa.tbl_lo = h->tbl_lo; sa.scores = w.scores; sa.sstat = w.sstat;
        sa.d.Hq = c.n_q_heads; sa.d.Hkv = c.n_kv_heads; sa.d.nsplit = plan.score_splits; sa.d.n_hi = h->n_hi;
        sa.d.q_bf16 = c.q_dtype == COMMVQ_BF16; sa.d.scale = h->scale;
        const int groups = pair_keys(c) ? 1 : plan.score_slice_groups;
        sa.d.groups = groups; sa.d.part_stride = (long long)pos->total_tokens * c.n_q_heads;
        if (groups > 1) sa.scores = w.scores_part;
        const int grid = pos->batch * c.n_kv_heads * plan.score_splits * groups;
        const int tpt = plan.score_split_len / kSliceThreads;
        hipError_t e;
        if (pair_keys(c)) {
            // 12-bit pairs -> one byte per index, then the paired-code score kernel
            hipLaunchKernelGGL(k_unpack_pairs, dim3((unsigned)((pos->max_seqlen + 255) / 256), (unsigned)(pos->batch * c.n_kv_heads)),
                               dim3(256), 0, s, key_codes, w.pair_bytes, pos->cu_seqlens, c.n_kv_heads, c.key_levels,
                               pair_record_bytes(c), pair_blocks(c));
            if (hipGetLastError() != hipSuccess) return COMMVQ_ERR_LAUNCH;
            sa.key_codes = w.pair_bytes;
            e = pair_blocks(c) == 1 ? launch_pair_b<1>(sa, h->G, tpt, grid, s) : launch_pair_b<2>(sa, h->G, tpt, grid, s);
        } else {
            e = c.m_key == 16 ? launch_sliced_m<16>(sa, h->G, tpt, grid, s) : launch_sliced_m<32>(sa, h->G, tpt, grid, s);
            if (e == hipSuccess && groups > 1) {
                const int ns = stat_splits(plan, pos->max_seqlen);
                hipLaunchKernelGGL(k_score_combine, dim3((unsigned)(pos->batch * c.n_q_heads * ns)), dim3(kCombineThreads), 0, s,
                                   w.scores_part, w.scores, w.sstat, pos->cu_seqlens, c.n_q_heads, ns, stat_len(plan), groups,
                                   sa.d.part_stride);
                e = hipGetLastError();
            }
        }
        return e == hipSuccess ? COMMVQ_OK : COMMVQ_ERR_LAUNCH;
    }
    ScoreArgs a;
    a.q = q; a.key_codes = key_codes; a.key_cb = key_cb;
    a.cu = pos->cu_seqlens; a.q_pos = pos->q_pos; a.key_pos = pos->key_pos;
    a.tbl_hi = h->tbl_hi; a.tbl_lo = h->tbl_lo;
    a.scores = w.scores; a.sstat = w.sstat;
    a.d.Hq = c.n_q_heads; a.d.Hkv = c.n_kv_heads; a.d.nsplit = plan.score_splits; a.d.split_len = plan.score_split_len;
    a.d.n_hi = h->n_hi; a.d.q_bf16 = c.q_dtype == COMMVQ_BF16; a.d.scale = h->scale;
    const int grid = pos->batch * c.n_kv_heads * plan.score_splits;
    const bool bf16 = c.codebook_dtype == COMMVQ_BF16;
    hipError_t e = c.m_key == 16 ? launch_score_m<16>(a, h->G, bf16, grid, s) : launch_score_m<32>(a, h->G, bf16, grid, s);
    return e == hipSuccess ? COMMVQ_OK : COMMVQ_ERR_LAUNCH;
}

commvq_status run_bins(commvq_handle *h, const uint8_t *val_codes, const commvq_positions *pos,
                       const commvq_plan &plan, const Workspace &w, hipStream_t s)
{
    const commvq_config &c = h->cfg;
    if (bin_values(c)) {  // free binary code: Softmax(A) S_V as an integer matrix product (commvq_vbits.hip)
        VbitsArgs v;
        v.val_bits = val_codes; v.cu = pos->cu_seqlens; v.scores = w.scores; v.sstat = w.sstat;
        v.bins = w.bins; v.vscale = w.vscale; v.lsum = w.lsum;
        v.Hq = c.n_q_heads; v.Hkv = c.n_kv_heads; v.G = h->G;
        v.nsplit = stat_splits(plan, pos->max_seqlen); v.split_len = stat_len(plan);
        v.nvsplit = plan.value_splits; v.vsplit_len = plan.value_split_len;
        v.Nc = c.value_bits; v.batch = pos->batch;
        return commvq_launch_vbits(v, s) == hipSuccess ? COMMVQ_OK : COMMVQ_ERR_LAUNCH;
    }
    BinsArgs a;
    a.val_codes = val_codes; a.cu = pos->cu_seqlens; a.scores = w.scores; a.sstat = w.sstat;
    a.bins = w.bins; a.vscale = w.vscale; a.lsum = w.lsum;
    a.Hq = c.n_q_heads; a.Hkv = c.n_kv_heads; a.nsplit = stat_splits(plan, pos->max_seqlen); a.split_len = stat_len(plan);
    a.nvsplit = plan.value_splits; a.vsplit_len = plan.value_split_len;
    const int grid = pos->batch * c.n_kv_heads * plan.value_splits;
    hipError_t e = c.m_val == 16 ? launch_bins_m<16>(a, h->G, grid, s) : launch_bins_m<32>(a, h->G, grid, s);
    return e == hipSuccess ? COMMVQ_OK : COMMVQ_ERR_LAUNCH;
}

commvq_status run_output(commvq_handle *h, const void *val_cb, const commvq_positions *pos, const commvq_plan &plan,
                         const Workspace &w, float *out, hipStream_t s)
{
    const commvq_config &c = h->cfg;
    OutArgs a;
    a.val_cb = val_cb; a.cu = pos->cu_seqlens; a.bins = w.bins; a.vscale = w.vscale; a.lsum = w.lsum;
    a.partial = w.partial; a.out = out;
    a.Hq = c.n_q_heads; a.Hkv = c.n_kv_heads;
    a.nvsplit = plan.value_splits; a.vsplit_len = plan.value_split_len;
    a.nchunk = plan.out_chunks; a.Mv = val_books(c); a.batch = pos->batch;
    a.cb_linear = bin_values(c) ? 1 : 0;
    const int grid = pos->batch * c.n_kv_heads * plan.out_chunks;
    const bool bf16 = c.codebook_dtype == COMMVQ_BF16;
    hipError_t e;
    if (use_out_mfma(h, pos->batch)) {  // several sequences: the product with the value codebook on the matrix cores
        const uint4 *vp = nullptr;
        for (const auto &pv : h->packed_vals)
            if (pv.first == val_cb) vp = pv.second;
        if (!vp) {  // not packed ahead of time: re-lay the value codebook into the workspace on every call
            if (launch_prep_values(c, val_cb, w.packed_val, s) != hipSuccess) return COMMVQ_ERR_LAUNCH;
            vp = w.packed_val;
        }
        a.nchunk = val_books(c) * kK / kOutMfmaRows;
        const int spt = 16 / h->G;
        const int mgrid = ((pos->batch + spt - 1) / spt) * c.n_kv_heads * a.nchunk;
        switch (h->G) {
        case 1: hipLaunchKernelGGL(k_out_mfma<1>, dim3(mgrid), dim3(kOutThreads), 0, s, a, vp); break;
        case 2: hipLaunchKernelGGL(k_out_mfma<2>, dim3(mgrid), dim3(kOutThreads), 0, s, a, vp); break;
        case 4: hipLaunchKernelGGL(k_out_mfma<4>, dim3(mgrid), dim3(kOutThreads), 0, s, a, vp); break;
        default: hipLaunchKernelGGL(k_out_mfma<8>, dim3(mgrid), dim3(kOutThreads), 0, s, a, vp); break;
        }
        if (hipGetLastError() != hipSuccess) return COMMVQ_ERR_LAUNCH;
        hipLaunchKernelGGL(k_out_final, dim3(pos->batch * c.n_q_heads), dim3(kD * kFinalParts), 0, s, a);
        return hipGetLastError() == hipSuccess ? COMMVQ_OK : COMMVQ_ERR_LAUNCH;
    }
    switch (h->G) {
    case 1: e = launch_out_g<1>(a, bf16, grid, s); break;
    case 2: e = launch_out_g<2>(a, bf16, grid, s); break;
    case 4: e = launch_out_g<4>(a, bf16, grid, s); break;
    default: e = launch_out_g<8>(a, bf16, grid, s); break;
    }
    if (e != hipSuccess) return COMMVQ_ERR_LAUNCH;
    hipLaunchKernelGGL(k_out_final, dim3(pos->batch * c.n_q_heads), dim3(kD * kFinalParts), 0, s, a);
    return hipGetLastError() == hipSuccess ? COMMVQ_OK : COMMVQ_ERR_LAUNCH;
}

}  // namespace

// ------------------------------------------------------------------ C ABI
extern "C" {

const char *commvq_status_string(commvq_status s)
{
    switch (s) {
    case COMMVQ_OK: return "ok";
    case COMMVQ_ERR_NULL: return "required pointer is NULL";
    case COMMVQ_ERR_CONFIG: return "unsupported configuration";
    case COMMVQ_ERR_SHAPE: return "inconsistent batch shape";
    case COMMVQ_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case COMMVQ_ERR_LAUNCH: return "HIP runtime error";
    case COMMVQ_ERR_NO_DEVICE: return "no usable gfx950 device";
    }
    return "unknown status";
}

commvq_status commvq_validate_config(const commvq_config *c)
{
    if (!c) return COMMVQ_ERR_NULL;
    if (c->head_dim != kD || c->k != kK) return COMMVQ_ERR_CONFIG;
    if (c->n_q_heads < 1 || c->n_kv_heads < 1 || c->n_q_heads % c->n_kv_heads) return COMMVQ_ERR_CONFIG;
    const int G = c->n_q_heads / c->n_kv_heads;
    if (G != 1 && G != 2 && G != 4 && G != 8) return COMMVQ_ERR_CONFIG;
    if (c->value_format == COMMVQ_VALUES_INDEXED) {
        if (c->m_val != 16 && c->m_val != 32) return COMMVQ_ERR_CONFIG;
    } else if (c->value_format == COMMVQ_VALUES_BINARY) {
        // towards the output kernels N_c / 256 stands in for the number of value codebooks: 4, 8 or 16
        if (c->value_bits != 1024 && c->value_bits != 2048 && c->value_bits != 4096) return COMMVQ_ERR_CONFIG;
    } else {
        return COMMVQ_ERR_CONFIG;
    }
    if (c->key_format == COMMVQ_KEYS_INDEXED) {
        if (c->m_key != 16 && c->m_key != 32) return COMMVQ_ERR_CONFIG;
    } else if (c->key_format == COMMVQ_KEYS_PAIRED) {
        // 12 R bits per record must fit the unpack kernel's staging (R <= 21: 32 bytes); one table for a and b, bf16 only
        if (c->key_levels < 1 || c->key_levels > 21 || c->codebook_dtype != COMMVQ_BF16) return COMMVQ_ERR_CONFIG;
    } else {
        return COMMVQ_ERR_CONFIG;
    }
    if (c->position_free != 0 && (c->position_free != 1 || c->key_format != COMMVQ_KEYS_INDEXED)) return COMMVQ_ERR_CONFIG;
    if (c->q_dtype != COMMVQ_F32 && c->q_dtype != COMMVQ_BF16) return COMMVQ_ERR_CONFIG;
    if (c->codebook_dtype != COMMVQ_F32 && c->codebook_dtype != COMMVQ_BF16) return COMMVQ_ERR_CONFIG;
    if (!(c->rope_base > 1.0) || !(c->softmax_scale >= 0.0)) return COMMVQ_ERR_CONFIG;
    if (c->max_position < 0 || c->max_position > (1 << 24)) return COMMVQ_ERR_CONFIG;
    return COMMVQ_OK;
}

static commvq_handle *new_handle(const commvq_config *config, int device)
{
    commvq_handle *h = new (std::nothrow) commvq_handle();
    if (!h) return nullptr;
    h->cfg = *config;
    h->G = config->n_q_heads / config->n_kv_heads;
    h->scale = (float)(config->softmax_scale > 0.0 ? config->softmax_scale : 1.0 / std::sqrt((double)kD));
    h->n_hi = (config->max_position >> kLoBits) + 1;
    h->device = device;
    h->tbl_hi = h->tbl_lo = nullptr;
    h->static_scratch = nullptr;
    h->prof_every = 0; h->prof_calls = 0; h->prof_head = h->prof_count = 0; h->prof_ev_made = false;
    return h;
}

commvq_status commvq_create_planner(const commvq_config *config, commvq_handle **out)
{
    if (!out) return COMMVQ_ERR_NULL;
    commvq_status st = commvq_validate_config(config);
    if (st != COMMVQ_OK) return st;
    commvq_handle *h = new_handle(config, -1);
    if (!h) return COMMVQ_ERR_LAUNCH;
    *out = h;
    return COMMVQ_OK;
}

commvq_status commvq_create(const commvq_config *config, commvq_handle **out)
{
    if (!out) return COMMVQ_ERR_NULL;
    commvq_status st = commvq_validate_config(config);
    if (st != COMMVQ_OK) return st;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return COMMVQ_ERR_NO_DEVICE; }
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, dev) != hipSuccess) { (void)hipGetLastError(); return COMMVQ_ERR_NO_DEVICE; }
    if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0) return COMMVQ_ERR_NO_DEVICE;  // the kernels are gfx950 code only
    commvq_handle *h = new_handle(config, dev);
    if (!h) return COMMVQ_ERR_LAUNCH;
    // exact phases in fp64, rounded once to fp32
    std::vector<float2> hi((size_t)h->n_hi * kJ), lo((size_t)kLo * kJ);
    for (int j = 0; j < kJ; ++j) {
        const double theta = std::pow(config->rope_base, -2.0 * j / kD);
        for (int a = 0; a < h->n_hi; ++a) {
            const double ang = theta * (double)((int64_t)a << kLoBits);
            hi[(size_t)a * kJ + j] = make_float2((float)std::cos(ang), (float)std::sin(ang));
        }
        for (int a = 0; a < kLo; ++a) {
            const double ang = theta * (double)a;
            lo[(size_t)a * kJ + j] = make_float2((float)std::cos(ang), (float)std::sin(ang));
        }
    }
    bool ok = hipMalloc(reinterpret_cast<void **>(&h->tbl_hi), hi.size() * sizeof(float2)) == hipSuccess &&
              hipMalloc(reinterpret_cast<void **>(&h->tbl_lo), lo.size() * sizeof(float2)) == hipSuccess &&
              hipMemcpy(h->tbl_hi, hi.data(), hi.size() * sizeof(float2), hipMemcpyHostToDevice) == hipSuccess &&
              hipMemcpy(h->tbl_lo, lo.data(), lo.size() * sizeof(float2), hipMemcpyHostToDevice) == hipSuccess;
    // this device's address of the static scratch array (every GPU holds its own copy at its own address)
    void *sp = nullptr;
    ok = ok && hipGetSymbolAddress(&sp, HIP_SYMBOL(scratch)) == hipSuccess && sp != nullptr;
    h->static_scratch = sp;
    if (!ok) {
        (void)hipGetLastError();
        if (h->tbl_hi) (void)hipFree(h->tbl_hi);
        if (h->tbl_lo) (void)hipFree(h->tbl_lo);
        delete h;
        return COMMVQ_ERR_LAUNCH;
    }
    *out = h;
    return COMMVQ_OK;
}

commvq_status commvq_destroy(commvq_handle *h)
{
    if (!h) return COMMVQ_ERR_NULL;
    if (h->prof_ev_made)
        for (int i = 0; i < kProfRing; ++i)
            for (int k = 0; k < 4; ++k) (void)hipEventDestroy(h->prof_ev[i][k]);
    if (h->tbl_hi) (void)hipFree(h->tbl_hi);
    if (h->tbl_lo) (void)hipFree(h->tbl_lo);
    delete h;
    return COMMVQ_OK;
}

commvq_status commvq_plan_query(const commvq_handle *h, int32_t batch, int64_t total_tokens, int32_t max_seqlen,
                                commvq_plan *plan)
{
    if (!h || !plan) return COMMVQ_ERR_NULL;
    // explicit key positions are not known here: the distance check belongs to the calls that see them
    const commvq_status st = check_shape(h, batch, total_tokens, max_seqlen, true);
    if (st != COMMVQ_OK) return st;
    make_plan(h, batch, max_seqlen, use_sliced(h, false), plan);
    return COMMVQ_OK;
}

commvq_status commvq_workspace_bytes(const commvq_handle *h, int32_t batch, int64_t total_tokens, int32_t max_seqlen,
                                     size_t *bytes)
{
    if (!bytes) return COMMVQ_ERR_NULL;
    commvq_plan plan;
    commvq_status st = commvq_plan_query(h, batch, total_tokens, max_seqlen, &plan);
    if (st != COMMVQ_OK) return st;
    Workspace w;
    carve(h, batch, total_tokens, max_seqlen, nullptr, &w);
    *bytes = w.bytes;
    return COMMVQ_OK;
}

commvq_status commvq_packed_key_codebook_bytes(const commvq_handle *h, size_t *bytes)
{
    if (!h || !bytes) return COMMVQ_ERR_NULL;
    if (h->cfg.codebook_dtype != COMMVQ_BF16) return COMMVQ_ERR_CONFIG;
    *bytes = packed_key_bytes(h->cfg);
    return COMMVQ_OK;
}

commvq_status commvq_pack_key_codebooks(commvq_handle *h, const void *key_cb, void *packed, void *stream)
{
    if (!h || !key_cb || !packed) return COMMVQ_ERR_NULL;
    if (h->cfg.codebook_dtype != COMMVQ_BF16) return COMMVQ_ERR_CONFIG;
    if ((reinterpret_cast<uintptr_t>(key_cb) | reinterpret_cast<uintptr_t>(packed)) & 15u) return COMMVQ_ERR_SHAPE;
    if (h->device < 0) return COMMVQ_ERR_NO_DEVICE;
    if (launch_prep(h->cfg, key_cb, static_cast<uint4 *>(packed), static_cast<hipStream_t>(stream)) != hipSuccess)
        return COMMVQ_ERR_LAUNCH;
    for (auto &e : h->packed_keys)
        if (e.first == key_cb) {
            e.second = static_cast<const uint4 *>(packed);
            return COMMVQ_OK;
        }
    try {
        h->packed_keys.emplace_back(key_cb, static_cast<const uint4 *>(packed));
    } catch (...) {
        return COMMVQ_ERR_LAUNCH;
    }
    return COMMVQ_OK;
}

commvq_status commvq_packed_value_codebook_bytes(const commvq_handle *h, size_t *bytes)
{
    if (!h || !bytes) return COMMVQ_ERR_NULL;
    if (h->cfg.codebook_dtype != COMMVQ_BF16) return COMMVQ_ERR_CONFIG;
    *bytes = (size_t)h->cfg.n_kv_heads * val_books(h->cfg) * kK * kD * 2;
    return COMMVQ_OK;
}

commvq_status commvq_pack_value_codebooks(commvq_handle *h, const void *val_cb, void *packed, void *stream)
{
    if (!h || !val_cb || !packed) return COMMVQ_ERR_NULL;
    if (h->cfg.codebook_dtype != COMMVQ_BF16) return COMMVQ_ERR_CONFIG;
    if ((reinterpret_cast<uintptr_t>(val_cb) | reinterpret_cast<uintptr_t>(packed)) & 15u) return COMMVQ_ERR_SHAPE;
    if (h->device < 0) return COMMVQ_ERR_NO_DEVICE;
    if (launch_prep_values(h->cfg, val_cb, static_cast<uint4 *>(packed), static_cast<hipStream_t>(stream)) != hipSuccess)
        return COMMVQ_ERR_LAUNCH;
    for (auto &e : h->packed_vals)
        if (e.first == val_cb) {
            e.second = static_cast<const uint4 *>(packed);
            return COMMVQ_OK;
        }
    try {
        h->packed_vals.emplace_back(val_cb, static_cast<const uint4 *>(packed));
    } catch (...) {
        return COMMVQ_ERR_LAUNCH;
    }
    return COMMVQ_OK;
}

commvq_status commvq_forget_packed_value_codebooks(commvq_handle *h, const void *val_cb)
{
    if (!h) return COMMVQ_ERR_NULL;
    for (size_t i = 0; i < h->packed_vals.size(); ++i)
        if (!val_cb || h->packed_vals[i].first == val_cb) {
            h->packed_vals.erase(h->packed_vals.begin() + (long)i);
            --i;
        }
    return COMMVQ_OK;
}

commvq_status commvq_forget_packed_key_codebooks(commvq_handle *h, const void *key_cb)
{
    if (!h) return COMMVQ_ERR_NULL;
    for (size_t i = 0; i < h->packed_keys.size(); ++i)
        if (!key_cb || h->packed_keys[i].first == key_cb) {
            h->packed_keys.erase(h->packed_keys.begin() + (long)i);
            --i;
        }
    return COMMVQ_OK;
}

commvq_status commvq_stage_scores(commvq_handle *h, const void *q, const uint8_t *key_codes, const void *key_cb,
                                  const commvq_positions *pos, void *workspace, size_t workspace_bytes,
                                  float *scores_out, void *stream)
{
    if (!h || !q || !key_codes || !key_cb) return COMMVQ_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(key_codes) & 15u) return COMMVQ_ERR_SHAPE;
    commvq_plan plan;
    Workspace w;
    commvq_status st = prep(h, pos, workspace, workspace_bytes, &plan, &w);
    if (st != COMMVQ_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    st = run_scores(h, q, key_codes, key_cb, pos, plan, w, s);
    if (st != COMMVQ_OK) return st;
    if (scores_out &&
        hipMemcpyAsync(scores_out, w.scores, (size_t)pos->total_tokens * h->cfg.n_q_heads * sizeof(float),
                       hipMemcpyDeviceToDevice, s) != hipSuccess)
        return COMMVQ_ERR_LAUNCH;
    return COMMVQ_OK;
}

commvq_status commvq_stage_bins(commvq_handle *h, const uint8_t *val_codes, const commvq_positions *pos,
                                void *workspace, size_t workspace_bytes, void *stream)
{
    if (!h || !val_codes) return COMMVQ_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(val_codes) & 15u) return COMMVQ_ERR_SHAPE;
    commvq_plan plan;
    Workspace w;
    commvq_status st = prep(h, pos, workspace, workspace_bytes, &plan, &w);
    if (st != COMMVQ_OK) return st;
    return run_bins(h, val_codes, pos, plan, w, static_cast<hipStream_t>(stream));
}

commvq_status commvq_stage_output(commvq_handle *h, const void *val_cb, const commvq_positions *pos, float *out,
                                  void *workspace, size_t workspace_bytes, void *stream)
{
    if (!h || !val_cb || !out) return COMMVQ_ERR_NULL;
    commvq_plan plan;
    Workspace w;
    commvq_status st = prep(h, pos, workspace, workspace_bytes, &plan, &w);
    if (st != COMMVQ_OK) return st;
    return run_output(h, val_cb, pos, plan, w, out, static_cast<hipStream_t>(stream));
}

commvq_status commvq_decode_attn(commvq_handle *h, const void *q, const uint8_t *key_codes, const uint8_t *val_codes,
                                 const void *key_cb, const void *val_cb, const commvq_positions *pos, float *out,
                                 void *workspace, size_t workspace_bytes, void *stream)
{
    if (!h || !q || !key_codes || !val_codes || !key_cb || !val_cb || !out) return COMMVQ_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(key_codes) | reinterpret_cast<uintptr_t>(val_codes)) & 15u) return COMMVQ_ERR_SHAPE;
    commvq_plan plan;
    Workspace w;
    commvq_status st = prep(h, pos, workspace, workspace_bytes, &plan, &w);
    if (st != COMMVQ_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipEvent_t *ev = nullptr;
    if (h->prof_every > 0 && h->prof_calls++ % h->prof_every == 0) {
        if (!h->prof_ev_made) {
            for (int i = 0; i < kProfRing; ++i)
                for (int k = 0; k < 4; ++k)
                    if (hipEventCreate(&h->prof_ev[i][k]) != hipSuccess) return COMMVQ_ERR_LAUNCH;
            h->prof_ev_made = true;
        }
        ev = h->prof_ev[h->prof_head];
        if (hipEventRecord(ev[0], s) != hipSuccess) return COMMVQ_ERR_LAUNCH;
    }
    st = run_scores(h, q, key_codes, key_cb, pos, plan, w, s);
    if (st != COMMVQ_OK) return st;
    if (ev && hipEventRecord(ev[1], s) != hipSuccess) return COMMVQ_ERR_LAUNCH;
    st = run_bins(h, val_codes, pos, plan, w, s);
    if (st != COMMVQ_OK) return st;
    if (ev && hipEventRecord(ev[2], s) != hipSuccess) return COMMVQ_ERR_LAUNCH;
    st = run_output(h, val_cb, pos, plan, w, out, s);
    if (st != COMMVQ_OK) return st;
    if (ev) {
        if (hipEventRecord(ev[3], s) != hipSuccess) return COMMVQ_ERR_LAUNCH;
        h->prof_head = (h->prof_head + 1) % kProfRing;
        if (h->prof_count < kProfRing) ++h->prof_count;
    }
    return COMMVQ_OK;
}

commvq_status commvq_decode_attn_static(commvq_handle *h, const void *q, const uint8_t *key_codes, const uint8_t *val_codes,
                                        const void *key_cb, const void *val_cb, const commvq_positions *pos, float *out,
                                        void *stream)
{
    if (!h || !q || !key_codes || !val_codes || !key_cb || !val_cb || !out) return COMMVQ_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(key_codes) | reinterpret_cast<uintptr_t>(val_codes)) & 15u) return COMMVQ_ERR_SHAPE;
    commvq_plan plan;
    Workspace w;
    // the handle's copy of the scratch array is the workspace; a batch shape that needs more than the array holds
    // comes back as COMMVQ_ERR_WORKSPACE from the same check that vets a caller's workspace
    commvq_status st = prep(h, pos, h->device < 0 ? reinterpret_cast<void *>(256) : h->static_scratch, kStaticScratchBytes, &plan, &w);
    if (st != COMMVQ_OK) return st;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev != h->device) return COMMVQ_ERR_NO_DEVICE;  // the array of another GPU
    hipStream_t s = static_cast<hipStream_t>(stream);
    st = run_scores(h, q, key_codes, key_cb, pos, plan, w, s);
    if (st != COMMVQ_OK) return st;
    st = run_bins(h, val_codes, pos, plan, w, s);
    if (st != COMMVQ_OK) return st;
    return run_output(h, val_cb, pos, plan, w, out, s);
}

commvq_status commvq_static_scratch_bytes(size_t *bytes)
{
    if (!bytes) return COMMVQ_ERR_NULL;
    *bytes = kStaticScratchBytes;
    return COMMVQ_OK;
}

commvq_status commvq_profile_enable(commvq_handle *h, int32_t every)
{
    if (!h) return COMMVQ_ERR_NULL;
    h->prof_every = every > 0 ? every : 0;
    h->prof_calls = 0;
    h->prof_head = h->prof_count = 0;
    return COMMVQ_OK;
}

commvq_status commvq_profile_read(commvq_handle *h, float *mean_ms, int32_t *n_calls)
{
    if (!h || !mean_ms || !n_calls) return COMMVQ_ERR_NULL;
    double acc[3] = {0, 0, 0};
    const int n = h->prof_count;
    for (int k = 0; k < n; ++k) {
        const int i = (h->prof_head - 1 - k + 2 * kProfRing) % kProfRing;
        if (hipEventSynchronize(h->prof_ev[i][3]) != hipSuccess) return COMMVQ_ERR_LAUNCH;
        for (int st = 0; st < 3; ++st) {
            float ms = 0.f;
            if (hipEventElapsedTime(&ms, h->prof_ev[i][st], h->prof_ev[i][st + 1]) != hipSuccess) return COMMVQ_ERR_LAUNCH;
            acc[st] += ms;
        }
    }
    for (int st = 0; st < 3; ++st) mean_ms[st] = n ? (float)(acc[st] / n) : 0.f;
    *n_calls = n;
    h->prof_head = h->prof_count = 0;
    return COMMVQ_OK;
}

}  // extern "C"
