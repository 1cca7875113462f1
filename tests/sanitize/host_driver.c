/*
 * Drives the host side of libcommvq (configuration checks, planning, workspace carving, argument validation of
 * every entry point) through planner handles, so that a build of the library whose HOST code is instrumented with
 * AddressSanitizer / UndefinedBehaviorSanitizer (tests/test_sanitize_cpu.py) reports overflows, bad shifts and
 * out-of-bounds accesses in that logic.  No GPU is touched: a planner handle launches nothing, and the pointers
 * passed below are never dereferenced by the library.  Exit status 0 = every call returned the documented status.
 */
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "commvq.h"

#define EXPECT(call, want) do { int got_ = (int)(call); if (got_ != (int)(want)) { \
    fprintf(stderr, "host_driver: line %d: %s returned %d, expected %d\n", __LINE__, #call, got_, (int)(want)); return 1; } } while (0)

static void *fake(uintptr_t a) { return (void *)a; }

static int drive(commvq_config c, int32_t B, int64_t T, int32_t L)
{
    commvq_handle *h = NULL;
    EXPECT(commvq_create_planner(&c, &h), COMMVQ_OK);
    commvq_plan plan;
    size_t ws = 0, nb = 0;
    EXPECT(commvq_plan_query(h, B, T, L, &plan), COMMVQ_OK);
    EXPECT(commvq_workspace_bytes(h, B, T, L, &ws), COMMVQ_OK);
    if (plan.score_splits < 1 || plan.value_splits < 1 || plan.out_chunks < 1 || ws == 0 || (ws & 255)) {
        fprintf(stderr, "host_driver: implausible plan\n");
        return 1;
    }
    commvq_positions pos = { B, (const int32_t *)fake(4096), (const int32_t *)fake(8192), NULL, T, L };
    EXPECT(commvq_decode_attn(h, fake(1 << 16), (const uint8_t *)fake(1 << 20), (const uint8_t *)fake(1 << 21), fake(1 << 22),
                              fake(1 << 23), &pos, (float *)fake(1 << 24), fake(1 << 25), ws, NULL), COMMVQ_ERR_NO_DEVICE);
    EXPECT(commvq_decode_attn(h, fake(1 << 16), (const uint8_t *)fake(1 << 20), (const uint8_t *)fake(1 << 21), fake(1 << 22),
                              fake(1 << 23), &pos, (float *)fake(1 << 24), fake(1 << 25), ws - 1, NULL), COMMVQ_ERR_WORKSPACE);
    EXPECT(commvq_stage_scores(h, fake(1 << 16), (const uint8_t *)fake(1 << 20), fake(1 << 22), &pos, fake(1 << 25), ws, NULL, NULL),
           COMMVQ_ERR_NO_DEVICE);
    EXPECT(commvq_stage_bins(h, (const uint8_t *)fake(1 << 21), &pos, fake(1 << 25), ws, NULL), COMMVQ_ERR_NO_DEVICE);
    EXPECT(commvq_stage_output(h, fake(1 << 23), &pos, (float *)fake(1 << 24), fake(1 << 25), ws, NULL), COMMVQ_ERR_NO_DEVICE);
    EXPECT(commvq_stage_output(h, NULL, &pos, (float *)fake(1 << 24), fake(1 << 25), ws, NULL), COMMVQ_ERR_NULL);
    if (c.codebook_dtype == COMMVQ_BF16) {
        EXPECT(commvq_packed_key_codebook_bytes(h, &nb), COMMVQ_OK);
        EXPECT(commvq_pack_key_codebooks(h, fake(1 << 22), fake(1 << 26), NULL), COMMVQ_ERR_NO_DEVICE);
        EXPECT(commvq_pack_key_codebooks(h, fake((1 << 22) + 4), fake(1 << 26), NULL), COMMVQ_ERR_SHAPE);
        EXPECT(commvq_packed_value_codebook_bytes(h, &nb), COMMVQ_OK);
        EXPECT(commvq_pack_value_codebooks(h, fake(1 << 22), fake(1 << 26), NULL), COMMVQ_ERR_NO_DEVICE);
        EXPECT(commvq_pack_value_codebooks(h, fake(1 << 22), fake((1 << 26) + 8), NULL), COMMVQ_ERR_SHAPE);
        EXPECT(commvq_pack_value_codebooks(h, NULL, fake(1 << 26), NULL), COMMVQ_ERR_NULL);
    } else {
        EXPECT(commvq_packed_key_codebook_bytes(h, &nb), COMMVQ_ERR_CONFIG);
        EXPECT(commvq_packed_value_codebook_bytes(h, &nb), COMMVQ_ERR_CONFIG);
    }
    EXPECT(commvq_forget_packed_key_codebooks(h, NULL), COMMVQ_OK);
    EXPECT(commvq_forget_packed_value_codebooks(h, NULL), COMMVQ_OK);
    EXPECT(commvq_encoder_table_bytes(h, &nb), COMMVQ_OK);
    EXPECT(commvq_encoder_prepare(h, fake(1 << 22), fake(1 << 27), NULL), COMMVQ_ERR_NO_DEVICE);
    EXPECT(commvq_encode_keys(h, fake(1 << 16), 3, fake(1 << 22), fake(1 << 27), (uint8_t *)fake(1 << 28), 1024, 64, NULL),
           COMMVQ_ERR_NO_DEVICE);
    EXPECT(commvq_encode_keys(h, fake(1 << 16), 3, fake(1 << 22), fake(1 << 27), (uint8_t *)fake(1 << 28), 1, 1, NULL), COMMVQ_ERR_SHAPE);
    EXPECT(commvq_decode_attn_static(h, fake(1 << 16), (const uint8_t *)fake(1 << 20), (const uint8_t *)fake(1 << 21), fake(1 << 22),
                                     fake(1 << 23), &pos, (float *)fake(1 << 24), NULL),
           ws <= ((size_t)48 << 20) ? COMMVQ_ERR_NO_DEVICE : COMMVQ_ERR_WORKSPACE);
    if (c.value_format == COMMVQ_VALUES_BINARY) {  /* no greedy stand-in for a free binary code */
        EXPECT(commvq_value_encoder_table_bytes(h, &nb), COMMVQ_ERR_CONFIG);
        EXPECT(commvq_value_encoder_prepare(h, fake(1 << 23), fake(1 << 27), NULL), COMMVQ_ERR_CONFIG);
        EXPECT(commvq_encode_values(h, fake(1 << 16), 3, fake(1 << 23), fake(1 << 27), (uint8_t *)fake(1 << 28), 1024, 64, NULL),
               COMMVQ_ERR_CONFIG);
    } else {
        EXPECT(commvq_value_encoder_table_bytes(h, &nb), COMMVQ_OK);
        EXPECT(commvq_value_encoder_prepare(h, fake(1 << 23), fake(1 << 27), NULL), COMMVQ_ERR_NO_DEVICE);
        EXPECT(commvq_encode_values(h, fake(1 << 16), 3, fake(1 << 23), fake(1 << 27), (uint8_t *)fake(1 << 28), 1024, 64, NULL),
               COMMVQ_ERR_NO_DEVICE);
        EXPECT(commvq_encode_values(h, fake(1 << 16), 3, fake(1 << 23), fake(1 << 27), (uint8_t *)fake(1 << 28), 1024, 8, NULL),
               COMMVQ_ERR_SHAPE);
    }
    EXPECT(commvq_profile_enable(h, 4), COMMVQ_OK);
    float ms[3];
    int32_t n = -1;
    EXPECT(commvq_profile_read(h, ms, &n), COMMVQ_OK);
    /* shapes at and beyond the limits */
    EXPECT(commvq_plan_query(h, 0, T, L, &plan), COMMVQ_ERR_SHAPE);
    EXPECT(commvq_plan_query(h, B, (int64_t)B * L + 1, L, &plan), COMMVQ_ERR_SHAPE);
    EXPECT(commvq_plan_query(h, 1, ((int64_t)1 << 30) + 1, INT32_MAX, &plan), COMMVQ_ERR_SHAPE);
    EXPECT(commvq_plan_query(h, 4, (int64_t)1 << 30, 1 << 28, &plan), COMMVQ_ERR_SHAPE);
    EXPECT(commvq_plan_query(h, 65536, 65536, 1, &plan), COMMVQ_OK);
    EXPECT(commvq_workspace_bytes(h, 65536, 65536, 1, &ws), COMMVQ_OK);
    EXPECT(commvq_destroy(h), COMMVQ_OK);
    return 0;
}

int main(void)
{
    commvq_config base = { 32, 8, 128, 16, 16, 256, COMMVQ_BF16, COMMVQ_BF16, 500000.0, 0.0, 1 << 24, COMMVQ_KEYS_INDEXED, 0, 0 };
    commvq_config c;
    EXPECT(commvq_validate_config(NULL), COMMVQ_ERR_NULL);
    EXPECT(commvq_create_planner(&base, NULL), COMMVQ_ERR_NULL);
    for (int i = 0; i < 8; ++i)
        if (!commvq_status_string((commvq_status)i)) return 1;

    if (drive(base, 1, 131072, 131072)) return 1;                       /* the benchmark layer at 128K */
    if (drive(base, 1, 8192, 8192)) return 1;                           /* short context: tiles cut along the slices */
    if (drive(base, 3, 20000, 9000)) return 1;
    c = base; c.m_key = 32; c.m_val = 32;
    if (drive(c, 8, 300001, 65536)) return 1;                           /* ragged batch */
    c = base; c.n_q_heads = 64; c.m_key = 32;
    if (drive(c, 4, 4 * 131072, 131072)) return 1;                      /* eight heads per group */
    c = base; c.n_q_heads = 1; c.n_kv_heads = 1; c.m_key = 32; c.m_val = 32; c.q_dtype = COMMVQ_F32; c.codebook_dtype = COMMVQ_F32;
    if (drive(c, 1, 4096, 4096)) return 1;                              /* fp32, one head */
    c = base; c.key_format = COMMVQ_KEYS_PAIRED; c.key_levels = 11; c.m_key = 0;
    if (drive(c, 2, 3000, 2000)) return 1;                              /* paired keys, 1-bit setting */
    c.key_levels = 21;
    if (drive(c, 1, 131072, 131072)) return 1;                          /* 2-bit setting */
    c = base; c.position_free = 1; c.max_position = 0;
    if (drive(c, 3, 7000, 3000)) return 1;                              /* scalar look-up table variant */
    c = base; c.n_q_heads = 8;
    if (drive(c, 1, 1, 1)) return 1;                                    /* one token */
    c = base; c.value_format = COMMVQ_VALUES_BINARY; c.value_bits = 1024; c.m_val = 0;
    if (drive(c, 1, 131072, 131072)) return 1;                          /* binary values, the paper's 1-bit width */
    if (drive(c, 300, 300 * 70000, 70000)) return 1;                    /* one token range per sequence, capped in length */
    c.value_bits = 4096; c.n_q_heads = 64; c.m_key = 32;
    if (drive(c, 4, 4 * 131072, 131072)) return 1;
    c = base; c.key_format = COMMVQ_KEYS_PAIRED; c.key_levels = 11; c.value_format = COMMVQ_VALUES_BINARY; c.value_bits = 1024;
    if (drive(c, 2, 3000, 2000)) return 1;                              /* the paper's formats on both sides */
    c = base; c.value_format = COMMVQ_VALUES_BINARY; c.value_bits = 1000;
    EXPECT(commvq_validate_config(&c), COMMVQ_ERR_CONFIG);
    c.value_format = 2; c.value_bits = 1024;
    EXPECT(commvq_validate_config(&c), COMMVQ_ERR_CONFIG);

    size_t nb = 0;
    EXPECT(commvq_static_scratch_bytes(&nb), COMMVQ_OK);
    EXPECT(commvq_em_workspace_bytes(65535, 1 << 24, 64, &nb), COMMVQ_OK);
    EXPECT(commvq_em_workspace_bytes(65536, 16, 4, &nb), COMMVQ_ERR_SHAPE);
    EXPECT(commvq_em_shared_workspace_bytes(64, 1 << 24, 64, &nb), COMMVQ_OK);
    EXPECT(commvq_em_step(NULL, 1, 1, 1, 1.0f, NULL, NULL, 0, NULL), COMMVQ_ERR_NULL);
    EXPECT(commvq_em_step((const float *)fake(4096), 4, 100, 8, 0.0f, (float *)fake(8192), fake(1 << 20), 1 << 20, NULL), COMMVQ_ERR_CONFIG);
    EXPECT(commvq_em_step_shared((const float *)fake(4096), 4, 100, 8, 1.0f, (float *)fake(8192), fake(1 << 20), 16, NULL), COMMVQ_ERR_WORKSPACE);
    puts("host_driver: ok");
    return 0;
}
