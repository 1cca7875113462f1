/*
 * CommVQ decode attention -- CPU ORACLE (test infrastructure, not product code).
 *
 * This file is the slow, plain, fp64 definition that the HIP library is checked
 * against.  Only tests, the smoke check and the benchmark's cpu_baseline leg may
 * call it; the product path never does.  It shares no code with the HIP path.
 *
 * What it computes is the *naive* decode-then-attend form of the paper
 * (Sec. 3.1 "Computation Complexity", the four-line summary ending in
 * Eq. v1_formula):
 *
 *     q  <- q R_t
 *     K  <- rows  s_i C_K R_i            (decode every key, then RoPE it)
 *     V  <- S_V C_V                      (Eq. decode_v)
 *     out = Softmax(q K^T / sqrt(d)) V   (Eq. v1_formula)
 *
 * The commutative reformulation (Eq. new_attention) and the value
 * re-association (Eq. optimized_v) are exact re-bracketings of this, so the
 * definition above is the reference for them.
 *
 * Readings (paper silent or config-bound):
 *   - codes are in index form: token i of KV head g stores M indices, one per
 *     codebook; s_i C is the sum of the M selected codeword rows
 *     (Eq. vanilla_decode with exactly one 1 per codebook);
 *   - RoPE follows Sec. 3.2 literally: adjacent pairs (2j, 2j+1), row vector
 *     times R_m^j = [[cos, -sin],[sin, cos]] (Eq. rope_ri), theta_j =
 *     base^(-2j/d) with j counted from 0;
 *   - query head h reads KV head h / (Hq/Hkv);
 *   - token i of a sequence sits at position i unless key_pos is given.
 *
 * Everything is double precision; callers widen bf16/fp32 inputs exactly.
 */
#include <math.h>
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* u <- u R_pos : Sec. 3.2, Eq. rope_ri applied to every adjacent pair. */
void commvq_oracle_rope(double *u, int d, double pos, double rope_base)
{
    for (int j = 0; j < d / 2; ++j) {
        double theta = pow(rope_base, -2.0 * (double)j / (double)d);
        double c = cos(pos * theta), s = sin(pos * theta);
        double x = u[2 * j], y = u[2 * j + 1];
        /* (x, y) [[c, -s], [s, c]] = (x c + y s, -x s + y c) */
        u[2 * j] = x * c + y * s;
        u[2 * j + 1] = -x * s + y * c;
    }
}

/* t_hat = s C : sum of the M selected codeword rows (Eq. vanilla_decode). */
void commvq_oracle_decode(const uint8_t *codes, const double *codebooks, /* [M][K][d] */
                          int M, int K, int d, double *t_hat)
{
    for (int e = 0; e < d; ++e) t_hat[e] = 0.0;
    for (int m = 0; m < M; ++m) {
        const double *row = codebooks + ((size_t)m * K + codes[m]) * d;
        for (int e = 0; e < d; ++e) t_hat[e] += row[e];
    }
}

/*
 * The paper's own value code (Sec. 4.1): the encoder turns the whole value vector of a token -- all KV heads
 * side by side, `width` = Hkv * d scalars -- into a binary sequence s of length Nc with any number of ones, and the
 * decoder is the matrix product s C with C [Nc][width] (Eq. vanilla_decode): the sum of the rows whose bit is set.
 * Bit c of a record is bit c % 8 of its byte c / 8.  Writes columns first .. first + n - 1 of s C to t_hat.
 */
void commvq_oracle_decode_bits(const uint8_t *bits, const double *codebook, /* [Nc][width] */
                               int Nc, int width, int first, int n, double *t_hat)
{
    for (int e = 0; e < n; ++e) t_hat[e] = 0.0;
    for (int c = 0; c < Nc; ++c)
        if ((bits[c / 8] >> (c % 8)) & 1) {
            const double *row = codebook + (size_t)c * width + first;
            for (int e = 0; e < n; ++e) t_hat[e] += row[e];
        }
}

typedef struct {
    int B, Hq, Hkv, d, Mk, Mv, K;
    const double *q;
    const uint8_t *key_codes, *val_codes;
    const double *key_cb, *val_cb;
    const int32_t *cu_seqlens, *q_pos, *key_pos;
    double rope_base, scale;
    double *out, *scores_out, *weights_out;
    const uint8_t *unit_mask; /* [B*Hkv] or NULL: which (b, g) units to compute */
    int Nc;                   /* > 0: values in the binary form of Sec. 4.1 (see commvq_oracle_decode_attn_bits) */
} job_t;

/* One (sequence b, KV head g) unit: all query heads of the group. */
static int run_unit(const job_t *J, int b, int g)
{
    const int d = J->d, G = J->Hq / J->Hkv;
    const int64_t off = J->cu_seqlens[b];
    const int64_t L = J->cu_seqlens[b + 1] - off;
    const uint8_t *kc = J->key_codes + ((size_t)off * J->Hkv + (size_t)g * L) * J->Mk;
    const uint8_t *vc = J->Nc > 0 ? J->val_codes + (size_t)off * (size_t)(J->Nc / 8)
                                  : J->val_codes + ((size_t)off * J->Hkv + (size_t)g * L) * J->Mv;
    const double *kcb = J->key_cb + (size_t)g * J->Mk * J->K * d;
    const double *vcb = J->Nc > 0 ? J->val_cb : J->val_cb + (size_t)g * J->Mv * J->K * d;

    double *qr = (double *)malloc(sizeof(double) * (size_t)G * d);
    double *s = (double *)malloc(sizeof(double) * (size_t)G * L);
    double *kv = (double *)malloc(sizeof(double) * d);
    if (!qr || !s || !kv) { free(qr); free(s); free(kv); return 1; }

    /* q <- q R_t */
    for (int hh = 0; hh < G; ++hh) {
        int h = g * G + hh;
        memcpy(qr + (size_t)hh * d, J->q + ((size_t)b * J->Hq + h) * d, sizeof(double) * d);
        commvq_oracle_rope(qr + (size_t)hh * d, d, (double)J->q_pos[b], J->rope_base);
    }
    /* K row i = s_i C_K R_i ; score = q K^T * scale */
    for (int64_t i = 0; i < L; ++i) {
        double pos = J->key_pos ? (double)J->key_pos[off + i] : (double)i;
        commvq_oracle_decode(kc + (size_t)i * J->Mk, kcb, J->Mk, J->K, d, kv);
        commvq_oracle_rope(kv, d, pos, J->rope_base);
        for (int hh = 0; hh < G; ++hh) {
            double acc = 0.0;
            for (int e = 0; e < d; ++e) acc += qr[(size_t)hh * d + e] * kv[e];
            s[(size_t)hh * L + i] = acc * J->scale;
        }
    }
    /* softmax over the context, then weights times decoded values */
    for (int hh = 0; hh < G; ++hh) {
        int h = g * G + hh;
        double *sh = s + (size_t)hh * L;
        int64_t so = off * J->Hq + (int64_t)h * L; /* [b][h][i] inside the ragged batch */
        if (J->scores_out) memcpy(J->scores_out + so, sh, sizeof(double) * (size_t)L);
        double mx = sh[0];
        for (int64_t i = 1; i < L; ++i) if (sh[i] > mx) mx = sh[i];
        double Z = 0.0;
        for (int64_t i = 0; i < L; ++i) { sh[i] = exp(sh[i] - mx); Z += sh[i]; }
        for (int64_t i = 0; i < L; ++i) sh[i] /= Z;
        if (J->weights_out) memcpy(J->weights_out + so, sh, sizeof(double) * (size_t)L);
    }
    for (int hh = 0; hh < G; ++hh) {
        double *o = J->out + ((size_t)b * J->Hq + (size_t)g * G + hh) * d;
        for (int e = 0; e < d; ++e) o[e] = 0.0;
    }
    for (int64_t i = 0; i < L; ++i) {
        if (J->Nc > 0) commvq_oracle_decode_bits(vc + (size_t)i * (size_t)(J->Nc / 8), vcb, J->Nc, J->Hkv * d, g * d, d, kv);
        else commvq_oracle_decode(vc + (size_t)i * J->Mv, vcb, J->Mv, J->K, d, kv);
        for (int hh = 0; hh < G; ++hh) {
            double w = s[(size_t)hh * L + i];
            double *o = J->out + ((size_t)b * J->Hq + (size_t)g * G + hh) * d;
            for (int e = 0; e < d; ++e) o[e] += w * kv[e];
        }
    }
    free(qr); free(s); free(kv);
    return 0;
}

typedef struct { const job_t *J; int tid, nthreads, rc; } worker_t;

static void *worker(void *arg)
{
    worker_t *w = (worker_t *)arg;
    const job_t *J = w->J;
    int n_units = J->B * J->Hkv;
    for (int u = w->tid; u < n_units; u += w->nthreads) {
        if (J->unit_mask && !J->unit_mask[u]) continue;
        if (run_unit(J, u / J->Hkv, u % J->Hkv)) w->rc = 1;
    }
    return NULL;
}

static int run_job(const job_t *J, int n_threads);

/*
 * Layouts (all host memory):
 *   q            [B][Hq][d]
 *   key_codes    per sequence b: [Hkv][L_b][Mk] bytes, sequences concatenated
 *   val_codes    per sequence b: [Hkv][L_b][Mv]
 *   key_cb       [Hkv][Mk][K][d],  val_cb [Hkv][Mv][K][d]
 *   cu_seqlens   [B+1] prefix sums of L_b;  q_pos [B];  key_pos [T] or NULL
 *   out          [B][Hq][d]
 *   scores_out / weights_out: NULL or [T*Hq], sequence b head h token i at
 *                cu_seqlens[b]*Hq + h*L_b + i  (scaled logits / softmax weights)
 *   unit_mask    NULL or [B*Hkv] bytes; units with 0 are skipped (their out rows
 *                are left untouched)
 * Returns 0 on success, 1 on bad arguments, 2 on allocation failure.
 */
int commvq_oracle_decode_attn(int B, int Hq, int Hkv, int d, int Mk, int Mv, int K,
                              const double *q, const uint8_t *key_codes, const uint8_t *val_codes,
                              const double *key_cb, const double *val_cb,
                              const int32_t *cu_seqlens, const int32_t *q_pos, const int32_t *key_pos,
                              double rope_base, double scale, double *out, double *scores_out,
                              double *weights_out, const uint8_t *unit_mask, int n_threads)
{
    if (B < 1 || Hq < 1 || Hkv < 1 || Hq % Hkv || d < 2 || d % 2 || Mk < 1 || Mv < 1 || K < 1 || K > 256)
        return 1;
    if (!q || !key_codes || !val_codes || !key_cb || !val_cb || !cu_seqlens || !q_pos || !out) return 1;
    for (int b = 0; b < B; ++b) if (cu_seqlens[b + 1] - cu_seqlens[b] < 1) return 1;
    job_t J = { B, Hq, Hkv, d, Mk, Mv, K, q, key_codes, val_codes, key_cb, val_cb, cu_seqlens,
                q_pos, key_pos, rope_base, scale, out, scores_out, weights_out, unit_mask, 0 };
    return run_job(&J, n_threads);
}

static int run_job(const job_t *Jp, int n_threads)
{
    job_t J = *Jp;
    const int B = J.B, Hkv = J.Hkv;
    if (n_threads < 1) n_threads = 1;
    if (n_threads > B * Hkv) n_threads = B * Hkv;
    pthread_t *th = (pthread_t *)malloc(sizeof(pthread_t) * (size_t)n_threads);
    worker_t *ws = (worker_t *)malloc(sizeof(worker_t) * (size_t)n_threads);
    if (!th || !ws) { free(th); free(ws); return 2; }
    int rc = 0;
    for (int t = 0; t < n_threads; ++t) {
        ws[t].J = &J; ws[t].tid = t; ws[t].nthreads = n_threads; ws[t].rc = 0;
        if (t > 0) pthread_create(&th[t], NULL, worker, &ws[t]);
    }
    worker(&ws[0]);
    for (int t = 1; t < n_threads; ++t) pthread_join(th[t], NULL);
    for (int t = 0; t < n_threads; ++t) if (ws[t].rc) rc = 2;
    free(th); free(ws);
    return rc;
}

/*
 * The same attention with the values in the paper's binary form (Sec. 4.1, Eq. vanilla_decode; Eq. decode_v):
 *   val_bits  per sequence b: [L_b][Nc / 8] bytes, one record per token for ALL KV heads together, sequences
 *             concatenated (offset cu_seqlens[b] * Nc / 8)
 *   val_cb    [Nc][Hkv * d]: row c is added to the token's whole value vector when bit c of its record is set;
 *             the value of KV head g is columns g d .. g d + d - 1 of that vector (the heads' values side by side)
 * Keys, positions, outputs and return codes as commvq_oracle_decode_attn.  Nc must be a multiple of 8.
 */
int commvq_oracle_decode_attn_bits(int B, int Hq, int Hkv, int d, int Mk, int Nc, int K,
                                   const double *q, const uint8_t *key_codes, const uint8_t *val_bits,
                                   const double *key_cb, const double *val_cb,
                                   const int32_t *cu_seqlens, const int32_t *q_pos, const int32_t *key_pos,
                                   double rope_base, double scale, double *out, double *scores_out,
                                   double *weights_out, const uint8_t *unit_mask, int n_threads)
{
    if (B < 1 || Hq < 1 || Hkv < 1 || Hq % Hkv || d < 2 || d % 2 || Mk < 1 || Nc < 8 || Nc % 8 || K < 1 || K > 256)
        return 1;
    if (!q || !key_codes || !val_bits || !key_cb || !val_cb || !cu_seqlens || !q_pos || !out) return 1;
    for (int b = 0; b < B; ++b) if (cu_seqlens[b + 1] - cu_seqlens[b] < 1) return 1;
    job_t J = { B, Hq, Hkv, d, Mk, 0, K, q, key_codes, val_bits, key_cb, val_cb, cu_seqlens,
                q_pos, key_pos, rope_base, scale, out, scores_out, weights_out, unit_mask, Nc };
    return run_job(&J, n_threads);
}

/*
 * Key encoding for cache append (Sec. 4.2: the E step of the clustering -- every vector goes to its
 * nearest clustering centre -- applied level by level to the quantization error of the previous
 * level, "conceptually similar to residual vector quantization"; App. A.1 for what a centre is).
 *
 *   paired == 0  index form: level m has the K centres C[m][c]; the token stores c_m.
 *   paired != 0  paper's format: level r has the K*K centres C[r][a] + (second rows of the blocks of
 *                C[r][b]), i.e. per sub-space (x_a - y_b, y_a + x_b) (Eq. def_center); the token stores
 *                (a_r, b_r).
 *
 *   keys   [n][d]            vectors of ONE KV head (pre-RoPE)
 *   cb     [levels][K][d]    that head's codebooks / tied table
 *   given  [n][levels*(paired?2:1)] or NULL.  If not NULL, level l takes the given codes instead of its
 *          own nearest centre when updating the residual (the search result is still reported), so a
 *          caller can ask "how good was somebody else's choice at each level, given their earlier ones".
 *   codes  [n][levels*(paired?2:1)]  nearest centre at each level (a, b interleaved when paired)
 *   best   [n][levels]       squared distance of that nearest centre to the residual it was searched for
 *   taken  [n][levels] or NULL  squared distance of the centre actually used (== best when given is NULL)
 * Every candidate's distance is computed from scratch as sum_e (res_e - centre_e)^2; ties go to the
 * lowest candidate index (a * K + b when paired).
 */
int commvq_oracle_encode_keys(int n, int d, int levels, int K, int paired, const double *keys, const double *cb,
                              const uint8_t *given, uint8_t *codes, double *best, double *taken)
{
    if (n < 0 || d < 2 || (d & 1) || levels < 1 || K < 1 || K > 256) return 1;
    const int per = paired ? 2 : 1;
    double *res = (double *)malloc(sizeof(double) * (size_t)d);
    double *cen = (double *)malloc(sizeof(double) * (size_t)d);
    if (!res || !cen) { free(res); free(cen); return 2; }
    for (int t = 0; t < n; ++t) {
        memcpy(res, keys + (size_t)t * d, sizeof(double) * (size_t)d);
        for (int l = 0; l < levels; ++l) {
            const double *C = cb + (size_t)l * K * d;
            double bd = INFINITY;
            int ba = 0, bb = 0;
            const int nb = paired ? K : 1;
            for (int a = 0; a < K; ++a)
                for (int b = 0; b < nb; ++b) {
                    double dist = 0.0;
                    for (int j = 0; j < d / 2; ++j) {
                        double cx = C[(size_t)a * d + 2 * j], cy = C[(size_t)a * d + 2 * j + 1];
                        if (paired) {  /* + second row (-y, x) of block j of centre b */
                            cx += -C[(size_t)b * d + 2 * j + 1];
                            cy += C[(size_t)b * d + 2 * j];
                        }
                        const double ex = res[2 * j] - cx, ey = res[2 * j + 1] - cy;
                        dist += ex * ex + ey * ey;
                    }
                    if (dist < bd) { bd = dist; ba = a; bb = b; }
                }
            codes[((size_t)t * levels + l) * per] = (uint8_t)ba;
            if (paired) codes[((size_t)t * levels + l) * per + 1] = (uint8_t)bb;
            best[(size_t)t * levels + l] = bd;
            int ua = ba, ub = bb;
            if (given) {
                ua = given[((size_t)t * levels + l) * per];
                ub = paired ? given[((size_t)t * levels + l) * per + 1] : 0;
                if (ua >= K || ub >= K) { free(res); free(cen); return 3; }
            }
            for (int j = 0; j < d / 2; ++j) {
                double cx = C[(size_t)ua * d + 2 * j], cy = C[(size_t)ua * d + 2 * j + 1];
                if (paired) {
                    cx += -C[(size_t)ub * d + 2 * j + 1];
                    cy += C[(size_t)ub * d + 2 * j];
                }
                cen[2 * j] = cx;
                cen[2 * j + 1] = cy;
            }
            double td = 0.0;
            for (int e = 0; e < d; ++e) {
                res[e] -= cen[e];
                td += res[e] * res[e];
            }
            if (taken) taken[(size_t)t * levels + l] = td;
        }
    }
    free(res);
    free(cen);
    return 0;
}
