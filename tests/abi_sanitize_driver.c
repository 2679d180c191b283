/*
 * Driver for the sanitizer run of the library's host code (tests/test_sanitizers.py): it is linked against a
 * build of libsmtm.so whose host side carries AddressSanitizer and UndefinedBehaviorSanitizer and walks the
 * paths that run before any GPU work: configuration checks, NULL handles for every entry point, and the
 * clean-up of a context whose creation fails half-way (no GPU is needed: without one, a valid configuration
 * fails in the first HIP call and must release what it had).  Exit status 0 when every call answered as declared.
 */
#include <stdio.h>
#include <string.h>

#include "../include/smtm.h"

static int failures = 0;
#define CHECK(cond) do { if (!(cond)) { fprintf(stderr, "check failed, line %d: %s\n", __LINE__, #cond); ++failures; } } while (0)

static smtm_config good(void)
{
    smtm_config c;
    memset(&c, 0, sizeof c);
    c.n_classes = 10; c.n_exits = 2; c.dims[0] = 8; c.dims[1] = 16; c.max_batch = 4;
    c.hot_init = 2; c.hot_min = 2; c.hot_max = 4; c.tiers = 2; c.tau = 1.0f; c.window = 8;
    c.cl_num = 19; c.cl_den = 20; c.init_count = 1;
    return c;
}

int main(void)
{
    smtm_ctx* ctx = (smtm_ctx*)0x1;
    smtm_config c = good();
    CHECK(smtm_create(NULL, &c) == SMTM_ERR_INVALID_ARG);
    CHECK(smtm_create(&ctx, NULL) == SMTM_ERR_INVALID_ARG && ctx == NULL);
    CHECK(strstr(smtm_last_error(NULL), "NULL") != NULL);

    /* one field wrong at a time */
    struct { int field; int value; int want; } bad[] = {
        {0, 1, SMTM_ERR_INVALID_ARG}, {0, SMTM_MAX_CLASSES + 1, SMTM_ERR_INVALID_ARG},
        {1, 0, SMTM_ERR_INVALID_ARG}, {1, SMTM_MAX_EXITS + 1, SMTM_ERR_INVALID_ARG},
        {2, 0, SMTM_ERR_SHAPE}, {2, 65537, SMTM_ERR_SHAPE},
        {3, 0, SMTM_ERR_INVALID_ARG}, {3, SMTM_MAX_BATCH + 1, SMTM_ERR_INVALID_ARG},
        {4, 1, SMTM_ERR_INVALID_ARG}, {5, 11, SMTM_ERR_INVALID_ARG}, {6, 3, SMTM_ERR_INVALID_ARG},
        {7, 0, SMTM_ERR_INVALID_ARG}, {8, 0, SMTM_ERR_INVALID_ARG}, {9, 21, SMTM_ERR_INVALID_ARG},
        {10, -1, SMTM_ERR_INVALID_ARG}, {11, 9, SMTM_ERR_INVALID_ARG}, {12, 2, SMTM_ERR_INVALID_ARG},
    };
    for (unsigned i = 0; i < sizeof bad / sizeof bad[0]; ++i) {
        c = good();
        switch (bad[i].field) {
            case 0: c.n_classes = bad[i].value; break;
            case 1: c.n_exits = bad[i].value; break;
            case 2: c.dims[1] = bad[i].value; break;
            case 3: c.max_batch = bad[i].value; break;
            case 4: c.hot_min = bad[i].value; break;
            case 5: c.hot_max = bad[i].value; break;
            case 6: c.tiers = bad[i].value; break;
            case 7: c.window = bad[i].value; break;
            case 8: c.cl_num = bad[i].value; break;
            case 9: c.cl_num = bad[i].value; break;
            case 10: c.init_count = bad[i].value; break;
            case 11: c.score_path = bad[i].value; break;
            default: c.forgetting = bad[i].value; break;
        }
        ctx = (smtm_ctx*)0x1;
        const int rc = smtm_create(&ctx, &c);
        if (rc != bad[i].want || ctx != NULL) {
            fprintf(stderr, "bad config %u: rc %d, wanted %d (%s)\n", i, rc, bad[i].want, smtm_last_error(NULL));
            ++failures;
        }
    }
    c = good(); c.tau = -1.0f;
    CHECK(smtm_create(&ctx, &c) == SMTM_ERR_INVALID_ARG);
    c = good(); c.tau = 0.0f / 0.0f;
    CHECK(smtm_create(&ctx, &c) == SMTM_ERR_INVALID_ARG);

    /* a valid configuration: with a GPU this is a context, without one the first HIP call fails and whatever
     * had been allocated is released again */
    c = good();
    ctx = (smtm_ctx*)0x1;
    const int rc = smtm_create(&ctx, &c);
    if (rc == SMTM_OK) {
        CHECK(ctx != NULL);
        CHECK(smtm_begin_batch(ctx, 5, NULL) == SMTM_ERR_SHAPE);
        CHECK(smtm_lookup(ctx, 1, NULL, NULL, NULL, NULL) == SMTM_ERR_STATE);
        CHECK(smtm_encode(ctx, 3, NULL, SMTM_F16, 1, 1, NULL, NULL, NULL) == SMTM_ERR_INVALID_ARG);
        CHECK(smtm_destroy(ctx) == SMTM_OK);
    } else {
        CHECK((rc == SMTM_ERR_HIP || rc == SMTM_ERR_NOMEM) && ctx == NULL);
        CHECK(smtm_last_error(NULL)[0] != 0);
    }

    /* NULL handle: every entry point answers with an error code (or NULL / ""), none dereferences it */
    CHECK(smtm_destroy(NULL) == SMTM_OK);
    CHECK(smtm_memory_load(NULL, 1, NULL, NULL) != SMTM_OK);
    CHECK(smtm_memory_import(NULL, 1, NULL, NULL, NULL) != SMTM_OK);
    CHECK(smtm_memory_export(NULL, 1, NULL, NULL, NULL) != SMTM_OK);
    CHECK(smtm_warmup_begin(NULL, NULL) != SMTM_OK && smtm_warmup_batch(NULL, NULL, 1, NULL) != SMTM_OK);
    CHECK(smtm_hot_set(NULL, NULL, 2, NULL) != SMTM_OK);
    CHECK(smtm_tables_export(NULL, NULL, NULL, NULL, NULL, NULL) != SMTM_OK);
    CHECK(smtm_tables_import(NULL, NULL, NULL, NULL) != SMTM_OK);
    CHECK(smtm_set_tau(NULL, 1.0f) != SMTM_OK);
    CHECK(smtm_begin_batch(NULL, 1, NULL) != SMTM_OK);
    CHECK(smtm_encode(NULL, 1, NULL, SMTM_F16, 1, 1, NULL, NULL, NULL) != SMTM_OK);
    CHECK(smtm_encode_nhwc(NULL, 1, NULL, SMTM_F16, 1, 1, NULL, NULL, NULL) != SMTM_OK);
    CHECK(smtm_lookup(NULL, 1, NULL, NULL, NULL, NULL) != SMTM_OK);
    CHECK(smtm_separability(NULL, 1, NULL, NULL, NULL) != SMTM_OK);
    CHECK(smtm_exit_compact(NULL, 1, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, 0, NULL) != SMTM_OK);
    CHECK(smtm_lookup_exit(NULL, 1, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, 0, NULL) != SMTM_OK);
    CHECK(smtm_stage(NULL, 1, NULL, SMTM_F16, 1, 1, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL) != SMTM_OK);
    CHECK(smtm_stage_nhwc(NULL, 1, NULL, SMTM_F16, 1, 1, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL) != SMTM_OK);
    CHECK(smtm_live_ids(NULL) == NULL && smtm_encode_kernel(NULL, 1)[0] == 0);
    CHECK(smtm_batch_results(NULL, NULL, NULL, NULL, NULL) != SMTM_OK);
    CHECK(smtm_read_counts(NULL, NULL, NULL, NULL) != SMTM_OK && smtm_read_stats(NULL, NULL, NULL) != SMTM_OK);
    CHECK(smtm_cache_update(NULL, NULL, NULL, 1, NULL) != SMTM_OK);
    CHECK(smtm_cache_update_static(NULL, NULL, NULL, 1, NULL) != SMTM_OK);
    CHECK(smtm_version() >= 200 && strlen(smtm_build_id()) == 16);

    if (failures) { fprintf(stderr, "%d checks failed\n", failures); return 1; }
    puts("library host-side sanitizer driver: all checks hold");
    return 0;
}
