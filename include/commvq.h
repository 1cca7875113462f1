/*
 * libcommvq -- single-token decode attention computed directly on a
 * CommVQ-compressed KV cache, for AMD MI355X (gfx950).
 *
 * Every cached key and value is stored as M uint8 code indices into learned
 * codebooks (additive quantization, paper Sec. 4.1, Eq. vanilla_decode), or in
 * the paper's own record formats (commvq_key_format, commvq_value_format).  The
 * library never decompresses the cache.  Scores follow the commutative
 * reformulation of Sec. 4.2 (Eq. new_attention): the selected key codewords are
 * gather-summed, rotated once by the RoPE matrix of the relative position and
 * contracted with the query.  Values follow the re-association of
 * Eq. optimized_v: softmax weights are accumulated into per-codeword bins
 * (Softmax(A) S_V) and the bins are multiplied by the value codebook once.
 * The result equals Eq. v1_formula (decode, RoPE, dense softmax attention) up
 * to fp32 rounding.  Results are bit-reproducible from call to call.
 *
 * Conventions
 *   - Pointers are DEVICE pointers unless a comment says "host".  The caller
 *     owns every buffer; the library only allocates its RoPE phase tables (in
 *     commvq_create) and frees them in commvq_destroy.
 *   - All work is enqueued on the caller's stream; nothing synchronises.
 *   - Functions return a commvq_status; nothing throws or aborts.  Arguments
 *     that can be checked from host values are checked before any launch.
 *   - RoPE is the paper's (Sec. 3.2, Eq. rope_ri): adjacent pairs (2j, 2j+1),
 *     row vector times [[cos, -sin], [sin, cos]], theta_j = rope_base^(-2j/d).
 *   - Query head h reads KV head h / (n_q_heads / n_kv_heads).
 */
#ifndef COMMVQ_H
#define COMMVQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    COMMVQ_OK = 0,
    COMMVQ_ERR_NULL = 1,      /* a required pointer is NULL */
    COMMVQ_ERR_CONFIG = 2,    /* unsupported head_dim / M / K / dtype / head counts */
    COMMVQ_ERR_SHAPE = 3,     /* batch, total_tokens or max_seqlen inconsistent, < 1, or beyond what the
                                 kernels' 32-bit offsets or the phase tables cover; misaligned buffers */
    COMMVQ_ERR_WORKSPACE = 4, /* workspace NULL, misaligned or too small */
    COMMVQ_ERR_LAUNCH = 5,    /* the HIP runtime reported an error (allocation, launch) */
    COMMVQ_ERR_NO_DEVICE = 6  /* the current device is not a gfx950, or the handle is a planner handle */
} commvq_status;

typedef enum { COMMVQ_F32 = 0, COMMVQ_BF16 = 1 } commvq_dtype;

/*
 * How the keys are stored.
 *   COMMVQ_KEYS_INDEXED  m_key independent codebooks of K = 256 codewords, one uint8 index per codebook.
 *   COMMVQ_KEYS_PAIRED   the paper's own key format (Sec. 4.2 with all 64 sub-spaces in one group, App. A.1):
 *                        key_levels = R residual levels; a token stores R pairs (a_r, b_r) of 6-bit indices into
 *                        ONE table of N_c' = 64 centres per level, and decodes to sum_r C[r][a_r] + i C[r][b_r],
 *                        i.e. per 2-D sub-space (x_a - y_b, y_a + x_b) (Eq. def_center).  12 R bits per token and
 *                        KV head: R = 11 is the paper's 1-bit setting, R = 21 its 2-bit setting.
 */
typedef enum { COMMVQ_KEYS_INDEXED = 0, COMMVQ_KEYS_PAIRED = 1 } commvq_key_format;

/*
 * How the values are stored.
 *   COMMVQ_VALUES_INDEXED  m_val independent codebooks of K = 256 codewords per KV head, one uint8 index per codebook
 *                          (Eq. vanilla_decode with exactly one 1 per codebook).
 *   COMMVQ_VALUES_BINARY   the paper's own value code (Sec. 4.1): the encoder maps a token's whole value vector -- the
 *                          n_kv_heads heads side by side, n_kv_heads * head_dim scalars -- to a binary sequence s of
 *                          value_bits = N_c bits with ANY number of ones, and the vector decodes to s C_V with ONE
 *                          codebook C_V [N_c][n_kv_heads * head_dim] (Eq. vanilla_decode); N_c = 1024 is the paper's
 *                          1-bit setting for an 8-KV-head model, 2048 its 2-bit setting (App., Table codebook_conf).
 *                          Softmax(A) S_V of Eq. optimized_v is then a dense product over the context and runs on the
 *                          matrix cores.
 */
typedef enum { COMMVQ_VALUES_INDEXED = 0, COMMVQ_VALUES_BINARY = 1 } commvq_value_format;

/* Host struct, copied by commvq_create. */
typedef struct {
    int32_t n_q_heads;       /* Hq */
    int32_t n_kv_heads;      /* Hkv; Hq / Hkv must be 1, 2, 4 or 8 */
    int32_t head_dim;        /* d; must be 128 */
    int32_t m_key;           /* M_k: key codebooks per KV head; 16 or 32 */
    int32_t m_val;           /* M_v: value codebooks per KV head; 16 or 32 */
    int32_t k;               /* K: codewords per codebook; must be 256 (one byte per code) */
    int32_t q_dtype;         /* commvq_dtype of q */
    int32_t codebook_dtype;  /* commvq_dtype of both codebooks */
    double rope_base;        /* > 1; 500000 for LLaMA-3.1 */
    double softmax_scale;    /* 0 selects 1/sqrt(head_dim) (Eq. v1_formula) */
    int32_t max_position;    /* largest |q_pos - key position| that will occur, <= 2^24; sizes the phase tables */
    int32_t key_format;      /* commvq_key_format; 0 (indexed) keeps every field above as described */
    int32_t key_levels;      /* R, 1..21; COMMVQ_KEYS_PAIRED only (m_key is then ignored; bf16 tables, implicit key positions) */
    int32_t position_free;   /* 1: no rotation at all -- the case Sec. 4.2 sets aside ("R_i independent of i", e.g. keys
                                quantized after RoPE): scores are (q . k_hat_i) * scale, computed with a scalar look-up
                                table T[m][c] = scale * q . C[m][c] and M_k look-ups per token; q_pos / key_pos are
                                ignored.  Indexed keys only.  0: RoPE as described above. */
    int32_t value_format;    /* commvq_value_format; 0 (indexed) keeps every field above as described */
    int32_t value_bits;      /* N_c: 1024, 2048 or 4096; COMMVQ_VALUES_BINARY only (m_val is then ignored) */
} commvq_config;

/* Host struct of device pointers: where the tokens sit (ragged batch). */
typedef struct {
    int32_t batch;             /* B >= 1 */
    const int32_t *cu_seqlens; /* device [B+1]: prefix sums of the context lengths L_b >= 0; a sequence with
                                  L_b = 0 (softmax over nothing) gets all-zero output rows */
    const int32_t *q_pos;      /* device [B]: position t of the query token (q <- q R_t) */
    const int32_t *key_pos;    /* device [T] or NULL; NULL means token i of a sequence sits at position i */
    int64_t total_tokens;      /* T = cu_seqlens[B] (host copy, sizes grids without a sync) */
    int32_t max_seqlen;        /* host copy of max_b L_b.  With key_pos == NULL the keys sit at 0 .. L_b - 1, and a
                                  query at or after the last of them is at least max_seqlen - 1 away from the first:
                                  max_seqlen - 1 > max_position is refused (COMMVQ_ERR_SHAPE) */
} commvq_positions;

/* How one call is cut into workgroups (host struct, filled by commvq_plan_query). */
typedef struct {
    int32_t score_split_len;  /* context tokens per score workgroup */
    int32_t score_splits;     /* score workgroups per (sequence, KV head) for max_seqlen */
    int32_t value_split_len;  /* context tokens per value workgroup */
    int32_t value_splits;     /* value workgroups per (sequence, KV head) for max_seqlen */
    int32_t out_chunks;       /* codebook-row chunks per (sequence, KV head) in the bins x codebook product */
    int32_t score_kernel;     /* 0: rows gathered through L1 (fp32 codebooks or explicit key positions);
                                 1: codebook slices streamed through LDS (or the look-up table of position_free) */
    int32_t score_slice_groups; /* score workgroups per tile: contexts too short to fill the chip are also cut along the
                                 codebook slices, and the groups' partial logits are added by a small kernel; 1 otherwise */
} commvq_plan;

typedef struct commvq_handle commvq_handle;

/* Validates the config and builds the RoPE phase tables on the current device.
 * *out is set only on COMMVQ_OK. */
commvq_status commvq_create(const commvq_config *config, commvq_handle **out);
commvq_status commvq_destroy(commvq_handle *handle);

/* Host-only check of a config (what commvq_create checks before touching the device). */
commvq_status commvq_validate_config(const commvq_config *config);

/*
 * A handle without device resources, for hosts that size buffers or vet arguments where no GPU is present
 * (schedulers, admission checks, CPU-only tests).  commvq_plan_query, commvq_workspace_bytes,
 * commvq_packed_key_codebook_bytes and commvq_encoder_table_bytes answer as for a full handle; every call that
 * would launch kernels runs all of its argument checks (pointers are only compared with NULL and tested for
 * alignment, never dereferenced), and returns COMMVQ_ERR_NO_DEVICE where a full handle would go on to launch.
 * Freed with commvq_destroy.
 */
commvq_status commvq_create_planner(const commvq_config *config, commvq_handle **out);

/* Host-only: work decomposition and workspace size for a batch shape.  COMMVQ_ERR_SHAPE if batch < 1,
 * max_seqlen < 1, total_tokens outside [max_seqlen, batch * max_seqlen] or above 2^30, or if one (sequence,
 * KV head) stream (max_seqlen * bytes per token of codes, unpacked pair indices or logits) passes 2^32 - 1 bytes. */
commvq_status commvq_plan_query(const commvq_handle *handle, int32_t batch, int64_t total_tokens,
                                int32_t max_seqlen, commvq_plan *plan);
commvq_status commvq_workspace_bytes(const commvq_handle *handle, int32_t batch, int64_t total_tokens,
                                     int32_t max_seqlen, size_t *bytes);

/*
 * Decode attention over the compressed cache (Eq. new_attention + Eq. optimized_v;
 * equals Eq. v1_formula).  For every sequence b and query head h:
 *     out[b][h] = Softmax_i( (q[b][h] R_t) . (k_hat_i R_{p_i}) * scale ) . v_hat_i
 * with k_hat_i / v_hat_i the sums of the M_k / M_v codeword rows that the codes of
 * token i select in the codebooks of KV head h / G.
 *
 *   q              [B][Hq][d], q_dtype
 *   key_codes      uint8; sequence b holds [Hkv][L_b][M_k], sequences concatenated
 *                  (byte offset of sequence b = cu_seqlens[b] * Hkv * M_k); 16-byte aligned.
 *                  COMMVQ_KEYS_PAIRED: [Hkv][L_b][PB] with PB = ceil(12 R / 8) bytes per record; pair r of a
 *                  token is bits 12 r .. 12 r + 11 of its record (little endian), a_r the low 6 bits, b_r the
 *                  high 6 bits; sequence offset cu_seqlens[b] * Hkv * PB
 *   val_codes      uint8; same with M_v.
 *                  COMMVQ_VALUES_BINARY: sequence b holds [L_b][N_c / 8], ONE record per token for all KV heads (byte
 *                  offset of sequence b = cu_seqlens[b] * N_c / 8); bit c of a record is bit c % 8 of its byte c / 8
 *   key_codebooks  [Hkv][M_k][K][d], codebook_dtype, row-major; a key codeword row is the
 *                  sequence of (x, y) first rows of its RoPE-commuting 2x2 blocks (Eq. C_struct).
 *                  COMMVQ_KEYS_PAIRED: the tied table [Hkv][R][64][d] bf16, same row convention
 *   val_codebooks  [Hkv][M_v][K][d].  COMMVQ_VALUES_BINARY: [N_c][Hkv * d]; query head h attends over columns
 *                  (h / G) d .. (h / G) d + d - 1 of the decoded vectors
 *   positions      host struct, see above; |q_pos - key position| must not exceed max_position.  What the host
 *                  can see of that is checked (see max_seqlen); q_pos and key_pos live on the device, and a
 *                  distance beyond the tables there is clamped to their last row: no fault, wrong rotation
 *   out            [B][Hq][d] fp32, fully overwritten
 *   workspace      >= commvq_workspace_bytes(...) bytes, 256-byte aligned, contents undefined after
 *   stream         a hipStream_t (NULL = the default stream)
 * Inputs are never written.  Concurrent calls need distinct workspaces.
 */
commvq_status commvq_decode_attn(commvq_handle *handle, const void *q, const uint8_t *key_codes,
                                 const uint8_t *val_codes, const void *key_codebooks, const void *val_codebooks,
                                 const commvq_positions *positions, float *out, void *workspace,
                                 size_t workspace_bytes, void *stream);

/*
 * commvq_decode_attn for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and bit-identical
 * results, but the workspace is a static device array inside the library (48 MiB on every GPU the library is
 * loaded on, held until the process ends; commvq_static_scratch_bytes reports the size).  The call allocates
 * nothing, creates no events (commvq_profile_enable is ignored here) and clears nothing with memset.
 *   COMMVQ_ERR_WORKSPACE  the batch shape needs more than the array holds (commvq_workspace_bytes tells how much a
 *                         shape needs; key codebooks packed ahead of time do not need their share of it, but the
 *                         size check still counts it)
 *   COMMVQ_ERR_NO_DEVICE  the current device is not the one the handle was created on
 * Every call on a GPU uses that GPU's one array, and the array keeps the previous call's contents: calls that
 * overlap in time on one GPU (two streams, two handles, two threads) race.  Run them one after the other, or use
 * commvq_decode_attn with separate workspaces.
 */
commvq_status commvq_decode_attn_static(commvq_handle *handle, const void *q, const uint8_t *key_codes,
                                        const uint8_t *val_codes, const void *key_codebooks, const void *val_codebooks,
                                        const commvq_positions *positions, float *out, void *stream);
commvq_status commvq_static_scratch_bytes(size_t *bytes /* host */);

/*
 * Optional one-time preparation of static key codebooks (they are per-layer constants, Sec. 4.1).
 * The score kernel for bf16 codebooks streams the key codebook through LDS in slices of
 * 256 / M_k elements (Eq. new_attention is evaluated slice by slice) and wants it in that order.
 * Without preparation every commvq_decode_attn call re-lays the codebook into its workspace
 * first (one extra read + write of the codebook).  commvq_pack_key_codebooks does it once:
 *   key_codebooks  [Hkv][M_k][K][d] bf16, as for commvq_decode_attn
 *   packed         device buffer of commvq_packed_key_codebook_bytes() bytes, 16-byte aligned,
 *                  owned by the caller; must stay alive and unchanged while registered
 * and remembers the pair in the handle: later calls that pass the same key_codebooks pointer
 * use `packed` instead of re-laying (the caller vouches that the contents did not change).
 * Results are bit-identical either way.  commvq_forget_packed_key_codebooks drops one pair
 * (or all, with NULL).  COMMVQ_ERR_CONFIG for fp32 codebooks (they take another kernel).
 * COMMVQ_KEYS_PAIRED: key_codebooks is the tied table; `packed` then holds it padded to blocks of
 * 16 levels, in LDS-image order.
 */
commvq_status commvq_packed_key_codebook_bytes(const commvq_handle *handle, size_t *bytes);
commvq_status commvq_pack_key_codebooks(commvq_handle *handle, const void *key_codebooks, void *packed, void *stream);
commvq_status commvq_forget_packed_key_codebooks(commvq_handle *handle, const void *key_codebooks);

/*
 * The same for the value codebooks (Eq. optimized_v: bins x C_V).  For batches of several sequences (16 or more
 * output rows = sequences x query heads per KV head, bf16 codebooks) the product with the value codebook runs on the
 * matrix cores and reads the codebook in k-step order ([KV head][32 rows][dimension][32] with rows ordered
 * codeword * M_v + codebook).  Without preparation every such call re-lays the value codebook into its workspace first;
 * commvq_pack_value_codebooks does it once and remembers (val_codebooks -> packed) in the handle, exactly as above:
 *   val_codebooks  [Hkv][M_v][K][d] bf16, as for commvq_decode_attn
 *   packed         device buffer of commvq_packed_value_codebook_bytes() bytes, 16-byte aligned, caller-owned
 * Results are bit-identical either way; smaller batches do not use it.  COMMVQ_ERR_CONFIG for fp32 codebooks.
 * COMMVQ_VALUES_BINARY: val_codebooks is [N_c][Hkv * d]; row r of head g is then the code bit that the value stage
 * keeps in row r of its bins (the six low bits of r permuted), restricted to the head's columns.
 */
commvq_status commvq_packed_value_codebook_bytes(const commvq_handle *handle, size_t *bytes);
commvq_status commvq_pack_value_codebooks(commvq_handle *handle, const void *val_codebooks, void *packed, void *stream);
commvq_status commvq_forget_packed_value_codebooks(commvq_handle *handle, const void *val_codebooks);

/*
 * Key encoding for cache append: the step before the attention call in every decode iteration.
 * Each new (pre-RoPE) key vector is assigned to its nearest clustering centre (the E step of Sec. 4.2),
 * level by level on the error left by the previous levels (residual refinement, Sec. 4.2); a centre of
 * the paired format is C[r][a] + i C[r][b] (Eq. def_center, App. A.1), searched over all 64 x 64 pairs.
 * Distances are compared in fp32 as ||c||^2 - 2 res.c; ties go to the lowest index (a * 64 + b).
 *   commvq_encoder_table_bytes / commvq_encoder_prepare
 *       one-time tables for a set of key codebooks (squared norms of all rows; paired: plus the
 *       cross terms 2 C[a].(i C[b])): `tables` is a device buffer of that many bytes, 16-byte aligned
 *   commvq_encode_keys
 *       keys        [n_tokens][Hkv][d], q_dtype, 16-byte aligned (as are key_codebooks and tables)
 *       codes_out   the record of token t, KV head g is written at codes_out + t * token_stride +
 *                   g * head_stride (bytes): M_k index bytes, or the ceil(12 R / 8)-byte packed
 *                   pair record, so that the caller can point straight into its cache layout
 *       COMMVQ_ERR_SHAPE if strides are smaller than a record, COMMVQ_ERR_CONFIG for fp32 paired tables
 */
commvq_status commvq_encoder_table_bytes(const commvq_handle *handle, size_t *bytes);
commvq_status commvq_encoder_prepare(commvq_handle *handle, const void *key_codebooks, void *tables, void *stream);
commvq_status commvq_encode_keys(commvq_handle *handle, const void *keys, int32_t n_tokens, const void *key_codebooks,
                                 const void *tables, uint8_t *codes_out, int64_t token_stride, int64_t head_stride,
                                 void *stream);

/*
 * Value encoding for cache append -- a stand-in for the paper's value encoder.  Sec. 4.1 encodes a value vector with a
 * small trained network E (x -> binary code s) whose weights come out of the training of Sec. 4.1 and are not part
 * of this library; what IS fixed by the cache format is the decoder (Eq. vanilla_decode in index form: the sum of the
 * m_val selected rows).  These calls produce codes for that decoder by the same greedy residual assignment as the
 * key encoder -- level m takes the row of value codebook m nearest to what the earlier levels left -- so that a
 * cache can be appended to end to end without the trained network.  Arguments, layouts, tie rule and status codes as
 * commvq_encoder_table_bytes / commvq_encoder_prepare / commvq_encode_keys in index form, with val_codebooks
 * [Hkv][m_val][K][d] and m_val index bytes per record.  COMMVQ_ERR_CONFIG for COMMVQ_VALUES_BINARY (no greedy
 * stand-in exists for a free binary code; the trained encoder is the only producer of such records).
 */
commvq_status commvq_value_encoder_table_bytes(const commvq_handle *handle, size_t *bytes);
commvq_status commvq_value_encoder_prepare(commvq_handle *handle, const void *val_codebooks, void *tables, void *stream);
commvq_status commvq_encode_values(commvq_handle *handle, const void *values, int32_t n_tokens, const void *val_codebooks,
                                   const void *tables, uint8_t *codes_out, int64_t token_stride, int64_t head_stride,
                                   void *stream);

/*
 * Offline: one iteration of the EM-like learner of the RoPE-commutative key codebook (Sec. 4.2,
 * Algorithm 1; App. A.2), for n_subspaces independent 2-D sub-spaces at once.  Needs no handle.
 *   data         device [n_subspaces][n_points][2] fp32: the calibration points of every sub-space
 *   phi          device [n_subspaces][n_centres][2] fp32, in/out: (x_l, y_l) of the blocks [[x, y], [-y, x]];
 *                the n_centres^2 clustering centres are (x_a - y_b, y_a + x_b) (Eq. def_center)
 *   temperature  T > 0 of the soft assignment W = softmax(-D / T), D = Euclidean distance (Eq. W); the caller
 *                anneals it over the iterations
 *   n_centres    1..64
 * E step and M step as in App. A.2; the M step solves the 2 n_centres x 2 n_centres normal equations of
 * the closed form phi* = (T^T S T)^-1 T^T S m by Cholesky factorisation.  COMMVQ_ERR_SHAPE for sizes out
 * of range, COMMVQ_ERR_CONFIG for T <= 0, COMMVQ_ERR_WORKSPACE as for commvq_decode_attn.
 */
commvq_status commvq_em_workspace_bytes(int32_t n_subspaces, int32_t n_points, int32_t n_centres, size_t *bytes);
commvq_status commvq_em_step(const float *data, int32_t n_subspaces, int32_t n_points, int32_t n_centres,
                             float temperature, float *phi, void *workspace, size_t workspace_bytes, void *stream);

/*
 * The same iteration when a group of sub-spaces shares its quantized value (Sec. 4.2: s^0 = ... = s^{g-1};
 * g = 64, the whole head, in the paper's configurations), i.e. the learner of the tied table that the paired
 * key format stores.  A clustering centre is the pair (a, b) applied in all `group` sub-spaces at once: the E step
 * weighs whole vectors, W_i,ab = softmax_ab(-D_i,ab / T) with D_i,ab = sqrt(sum_j ||k_i^j - c_ab^j||^2), and the
 * M step is App. A.2's closed form in every sub-space with that common W (one matrix T^T S T, `group`
 * right-hand sides).  Residual levels are learned one after the other by the caller, on the residuals.
 *   data         device [n_points][group][2] fp32: the calibration vectors (d = 2 * group values each)
 *   phi          device [group][n_centres][2] fp32, in/out
 *   group        1..64;  n_centres 1..64;  n_points 1..2^24
 * Results do not depend on the launch shape (all sums run in a fixed order).  A first or second index whose
 * total weight underflows to zero makes the system singular (as in the paper's closed form): keep T large
 * enough for every index to keep weight.  Status codes as commvq_em_step.
 */
commvq_status commvq_em_shared_workspace_bytes(int32_t group, int32_t n_points, int32_t n_centres, size_t *bytes);
commvq_status commvq_em_step_shared(const float *data, int32_t group, int32_t n_points, int32_t n_centres,
                                    float temperature, float *phi, void *workspace, size_t workspace_bytes, void *stream);

/*
 * The three stages of commvq_decode_attn, callable on their own (tests and profiling).
 * They read/write the same workspace; run them in this order on one stream.
 *   commvq_stage_scores  Eq. new_attention: scaled logits for every (b, h, token) and the
 *                        per-split maxima.  If scores_out is not NULL it receives a copy of the
 *                        logits, fp32 [T*Hq], (b, h, i) at cu_seqlens[b]*Hq + h*L_b + i.
 *   commvq_stage_bins    Softmax(A) S_V of Eq. optimized_v, unnormalised: exp(score - max)
 *                        accumulated per (head, value codebook, codeword) in 32-bit fixed point
 *                        (unit chosen per context split from its exp-sum; error below
 *                        tokens-per-split * 2^-31 of the split's weight), plus the exp sums.
 *                        COMMVQ_VALUES_BINARY: per (head, code bit), as an 8-bit integer matrix product over
 *                        four signed digits of the same fixed-point weights (error below tokens * 2^-30).
 *   commvq_stage_output  (bins C_V) / sum of Eq. optimized_v -> out.
 */
commvq_status commvq_stage_scores(commvq_handle *handle, const void *q, const uint8_t *key_codes,
                                  const void *key_codebooks, const commvq_positions *positions,
                                  void *workspace, size_t workspace_bytes, float *scores_out, void *stream);
commvq_status commvq_stage_bins(commvq_handle *handle, const uint8_t *val_codes,
                                const commvq_positions *positions, void *workspace, size_t workspace_bytes,
                                void *stream);
commvq_status commvq_stage_output(commvq_handle *handle, const void *val_codebooks,
                                  const commvq_positions *positions, float *out, void *workspace,
                                  size_t workspace_bytes, void *stream);

/*
 * Per-stage timing.  commvq_profile_enable(handle, every): every > 0 makes every `every`-th commvq_decode_attn
 * (the first, the every + 1-th, ...) bracket each of its stages with HIP events on the caller's stream (a ring of
 * 64 recorded calls); 0 switches it off.  An event between two kernels costs a few microseconds of GPU time
 * (the next kernel's dispatch no longer overlaps the previous one's end), which is why a caller that times whole
 * calls as well samples with every > 1.  commvq_profile_read synchronises on the recorded events and returns the
 * mean duration in milliseconds of [scores, bins, output] over the calls recorded since the last read (host
 * array of 3 floats) and their count.
 */
commvq_status commvq_profile_enable(commvq_handle *handle, int32_t every);
commvq_status commvq_profile_read(commvq_handle *handle, float *mean_ms /* host [3] */, int32_t *n_calls /* host */);

const char *commvq_status_string(commvq_status status);

#ifdef __cplusplus
}
#endif
#endif /* COMMVQ_H */
