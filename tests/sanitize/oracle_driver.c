/*
 * Runs every entry point of the CPU oracle on small, exactly sized heap buffers so that an
 * AddressSanitizer / UndefinedBehaviorSanitizer build (tests/test_sanitize_cpu.py compiles this file together
 * with oracle/commvq_oracle.c) reports any read or write outside them: ragged batch, several KV heads,
 * explicit and implicit key positions, a unit mask, threads, both encoder formats and the "given" replay.
 * Test infrastructure only.  Exit status 0 = every call returned what it should.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

void commvq_oracle_rope(double *u, int d, double pos, double rope_base);
void commvq_oracle_decode(const uint8_t *codes, const double *codebooks, int M, int K, int d, double *t_hat);
int commvq_oracle_decode_attn(int B, int Hq, int Hkv, int d, int Mk, int Mv, int K, const double *q,
                              const uint8_t *key_codes, const uint8_t *val_codes, const double *key_cb,
                              const double *val_cb, const int32_t *cu_seqlens, const int32_t *q_pos,
                              const int32_t *key_pos, double rope_base, double scale, double *out,
                              double *scores_out, double *weights_out, const uint8_t *unit_mask, int n_threads);
void commvq_oracle_decode_bits(const uint8_t *bits, const double *codebook, int Nc, int width, int first, int n, double *t_hat);
int commvq_oracle_decode_attn_bits(int B, int Hq, int Hkv, int d, int Mk, int Nc, int K, const double *q,
                                   const uint8_t *key_codes, const uint8_t *val_bits, const double *key_cb, const double *val_cb,
                                   const int32_t *cu_seqlens, const int32_t *q_pos, const int32_t *key_pos, double rope_base,
                                   double scale, double *out, double *scores_out, double *weights_out, const uint8_t *unit_mask,
                                   int n_threads);
int commvq_oracle_encode_keys(int n, int d, int levels, int K, int paired, const double *keys, const double *cb,
                              const uint8_t *given, uint8_t *codes, double *best, double *taken);

static uint64_t state = 88172645463325252ull;
static uint32_t next_u32(void) { state ^= state << 13; state ^= state >> 7; state ^= state << 17; return (uint32_t)(state >> 16); }
static double next_unit(void) { return (double)(next_u32() % 20001u) / 10000.0 - 1.0; }
static double *rand_doubles(size_t n) { double *p = malloc(n * sizeof *p); for (size_t i = 0; i < n; ++i) p[i] = next_unit(); return p; }
static uint8_t *rand_bytes(size_t n, unsigned below) { uint8_t *p = malloc(n ? n : 1); for (size_t i = 0; i < n; ++i) p[i] = (uint8_t)(next_u32() % below); return p; }

#define CHECK(cond) do { if (!(cond)) { fprintf(stderr, "oracle_driver: check failed at line %d: %s\n", __LINE__, #cond); return 1; } } while (0)

int main(void)
{
    enum { B = 3, Hq = 4, Hkv = 2, d = 6, Mk = 3, Mv = 2, K = 5 };
    const int32_t cu[B + 1] = { 0, 4, 5, 12 };
    const int T = 12;
    int32_t q_pos[B] = { 3, 0, 40 };
    int32_t *key_pos = malloc(T * sizeof *key_pos);
    for (int i = 0; i < T; ++i) key_pos[i] = (int32_t)(next_u32() % 50u);
    double *q = rand_doubles((size_t)B * Hq * d);
    double *kcb = rand_doubles((size_t)Hkv * Mk * K * d), *vcb = rand_doubles((size_t)Hkv * Mv * K * d);
    uint8_t *kc = rand_bytes((size_t)T * Hkv * Mk, K), *vc = rand_bytes((size_t)T * Hkv * Mv, K);
    double *out = malloc(sizeof(double) * B * Hq * d);
    double *scores = malloc(sizeof(double) * T * Hq), *weights = malloc(sizeof(double) * T * Hq);

    /* single pieces */
    double *u = rand_doubles(d), *dec = malloc(sizeof(double) * d);
    commvq_oracle_rope(u, d, 17.0, 500000.0);
    commvq_oracle_decode(kc, kcb, Mk, K, d, dec);

    /* whole attention: implicit positions, one thread, with intermediates */
    CHECK(commvq_oracle_decode_attn(B, Hq, Hkv, d, Mk, Mv, K, q, kc, vc, kcb, vcb, cu, q_pos, NULL, 500000.0,
                                    1.0 / sqrt((double)d), out, scores, weights, NULL, 1) == 0);
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < Hq; ++h) {
            double sum = 0.0;
            const int L = cu[b + 1] - cu[b];
            for (int i = 0; i < L; ++i) sum += weights[(size_t)cu[b] * Hq + (size_t)h * L + i];
            CHECK(fabs(sum - 1.0) < 1e-12);
        }
    /* explicit positions, more threads than units, a unit mask */
    uint8_t mask[B * Hkv] = { 1, 0, 1, 1, 0, 1 };
    CHECK(commvq_oracle_decode_attn(B, Hq, Hkv, d, Mk, Mv, K, q, kc, vc, kcb, vcb, cu, q_pos, key_pos, 10000.0,
                                    0.5, out, NULL, NULL, mask, 16) == 0);
    /* rejected arguments never touch the buffers */
    const int32_t cu_empty[B + 1] = { 0, 4, 4, 12 };
    CHECK(commvq_oracle_decode_attn(B, Hq, Hkv, d, Mk, Mv, K, q, kc, vc, kcb, vcb, cu_empty, q_pos, NULL, 500000.0,
                                    1.0, out, NULL, NULL, NULL, 2) == 1);
    CHECK(commvq_oracle_decode_attn(B, Hq, 3, d, Mk, Mv, K, q, kc, vc, kcb, vcb, cu, q_pos, NULL, 500000.0, 1.0, out,
                                    NULL, NULL, NULL, 2) == 1);

    /* binary value code: exactly-sized record and codebook buffers (Nc / 8 bytes per token, Nc rows of Hkv * d) */
    enum { NC = 24 };
    uint8_t *vb = rand_bytes((size_t)T * (NC / 8), 256);
    double *vfull = rand_doubles((size_t)NC * Hkv * d);
    commvq_oracle_decode_bits(vb + (size_t)(T - 1) * (NC / 8), vfull, NC, Hkv * d, (Hkv - 1) * d, d, dec);
    CHECK(commvq_oracle_decode_attn_bits(B, Hq, Hkv, d, Mk, NC, K, q, kc, vb, kcb, vfull, cu, q_pos, NULL, 500000.0,
                                         1.0 / sqrt((double)d), out, scores, weights, NULL, 1) == 0);
    CHECK(commvq_oracle_decode_attn_bits(B, Hq, Hkv, d, Mk, NC, K, q, kc, vb, kcb, vfull, cu, q_pos, key_pos, 10000.0,
                                         0.5, out, NULL, NULL, mask, 16) == 0);
    CHECK(commvq_oracle_decode_attn_bits(B, Hq, Hkv, d, Mk, 20, K, q, kc, vb, kcb, vfull, cu, q_pos, NULL, 500000.0,
                                         1.0, out, NULL, NULL, NULL, 2) == 1);
    CHECK(commvq_oracle_decode_attn_bits(B, Hq, Hkv, d, Mk, NC, K, q, kc, NULL, kcb, vfull, cu, q_pos, NULL, 500000.0,
                                         1.0, out, NULL, NULL, NULL, 2) == 1);
    free(vb); free(vfull);

    /* encoder: index form, paired form, replay of given codes, a bad given code */
    enum { N = 7, LEV = 3 };
    double *keys = rand_doubles((size_t)N * d), *cb = rand_doubles((size_t)LEV * K * d);
    uint8_t *codes = malloc(N * LEV * 2), *codes2 = malloc(N * LEV * 2);
    double *best = malloc(sizeof(double) * N * LEV), *taken = malloc(sizeof(double) * N * LEV);
    CHECK(commvq_oracle_encode_keys(N, d, LEV, K, 0, keys, cb, NULL, codes, best, taken) == 0);
    for (int i = 0; i < N * LEV; ++i) CHECK(codes[i] < K && fabs(best[i] - taken[i]) <= 1e-12 * (1.0 + best[i]));
    CHECK(commvq_oracle_encode_keys(N, d, LEV, K, 1, keys, cb, NULL, codes, best, NULL) == 0);
    CHECK(commvq_oracle_encode_keys(N, d, LEV, K, 1, keys, cb, codes, codes2, best, taken) == 0);
    for (int i = 0; i < N * LEV * 2; ++i) CHECK(codes[i] == codes2[i]);
    codes[5] = K;
    CHECK(commvq_oracle_encode_keys(N, d, LEV, K, 1, keys, cb, codes, codes2, best, taken) == 3);
    CHECK(commvq_oracle_encode_keys(0, d, LEV, K, 0, keys, cb, NULL, codes, best, taken) == 0);

    free(key_pos); free(q); free(kcb); free(vcb); free(kc); free(vc); free(out); free(scores); free(weights);
    free(u); free(dec); free(keys); free(cb); free(codes); free(codes2); free(best); free(taken);
    puts("oracle_driver: ok");
    return 0;
}
