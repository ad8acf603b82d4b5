/* A plain C99 translation unit that includes include/lychee.h and calls through it: the host-only
 * entry points and the error paths that need no GPU.  Built and run by tests/test_c_header.py.
 * Prints one line per check; exit status 0 = all passed. */
#include "lychee.h"

#include <stdio.h>
#include <string.h>

static int failures = 0;
#define CHECK(cond)                                                      \
    do {                                                                 \
        if (!(cond)) {                                                   \
            printf("FAILED line %d: %s\n", __LINE__, #cond);             \
            ++failures;                                                  \
        }                                                                \
    } while (0)

int main(void)
{
    lychee_shape s;
    uint8_t mask[32];
    int64_t a = 0, b = 0;
    float ms[LYCHEE_N_KERNEL_CLASSES];
    int32_t n[LYCHEE_N_KERNEL_CLASSES];
    size_t one, two;

    memset(&s, 0, sizeof s);
    s.batch = 1;
    s.n_q_heads = 32;
    s.n_kv_heads = 8;
    s.head_dim = LYCHEE_HEAD_DIM;
    s.max_len = 131072;
    s.k = 4096;
    s.kv_stride_batch = (int64_t)8 * 131072 * 128;
    s.kv_stride_head = (int64_t)131072 * 128;
    s.kv_stride_tok = 128;
    printf("sizeof(lychee_shape) = %u\n", (unsigned)sizeof s);
    CHECK(sizeof s == 64);

    /* shapes */
    CHECK(lychee_check_shape(&s, NULL, 0) == LYCHEE_OK);
    CHECK(lychee_check_shape(NULL, NULL, 0) == LYCHEE_EINVAL);
    memset(mask, 0, sizeof mask);
    mask[3] = 1;
    CHECK(lychee_check_shape(&s, mask, 1) == LYCHEE_OK);
    CHECK(lychee_check_shape(&s, mask, 0) == LYCHEE_EINVAL);   /* sparse heads without an inherited set */
    memset(mask, 1, sizeof mask);
    CHECK(lychee_check_shape(&s, mask, 0) == LYCHEE_OK);       /* the first layer: every head retrieves */
    s.head_dim = 64;
    CHECK(lychee_check_shape(&s, NULL, 0) == LYCHEE_EUNSUPPORTED);
    CHECK(lychee_workspace_bytes(&s) == 0);
    s.head_dim = LYCHEE_HEAD_DIM;
    s.k = 0;
    CHECK(lychee_check_shape(&s, NULL, 0) == LYCHEE_EINVAL);
    s.k = 4096;
    s.prob_rule = LYCHEE_RULE_TOP_P;
    s.prob_param = 1.5f;
    CHECK(lychee_check_shape(&s, NULL, 0) == LYCHEE_EINVAL);
    s.prob_param = 0.9f;
    CHECK(lychee_check_shape(&s, NULL, 0) == LYCHEE_OK);
    s.block_size = 64;
    CHECK(lychee_check_shape(&s, NULL, 0) == LYCHEE_EUNSUPPORTED);  /* probability rules rank positions */
    s.block_size = 0;
    s.prob_rule = 0;
    s.prob_param = 0.0f;

    /* workspace sizes */
    one = lychee_workspace_bytes(&s);
    two = lychee_step_workspace_bytes(&s, 2);
    printf("workspace: %lu bytes per layer\n", (unsigned long)one);
    CHECK(one > 0 && one % 256 == 0);
    CHECK(two == 2 * one);
    CHECK(lychee_step_workspace_bytes(&s, 0) == 0);
    CHECK(one <= LYCHEE_STATIC_SCRATCH_BYTES);   /* the 128K layer at batch 1 fits the static scratch */
    s.batch = 8;
    CHECK(lychee_workspace_bytes(&s) > LYCHEE_STATIC_SCRATCH_BYTES);
    s.batch = 1;

    /* calls without a context return EINVAL before they touch anything */
    CHECK(lychee_destroy(NULL) == LYCHEE_EINVAL);
    CHECK(lychee_create(NULL, 0) == LYCHEE_EINVAL);
    CHECK(lychee_set_option(NULL, LYCHEE_OPT_STEP_MODE, LYCHEE_STEP_LAYERWISE) == LYCHEE_EINVAL);
    CHECK(lychee_select_flush(NULL, NULL) == LYCHEE_EINVAL);
    CHECK(lychee_decode_attn(NULL, &s, &s, &s, &s, mask, NULL, &s, (int32_t *)&s, (const int32_t *)&s, &s, one, NULL) == LYCHEE_EINVAL);
    CHECK(lychee_decode_attn_static(NULL, &s, &s, &s, &s, mask, NULL, &s, (int32_t *)&s, (const int32_t *)&s, NULL) == LYCHEE_EINVAL);
    CHECK(lychee_decode_attn_deferred(NULL, &s, &s, &s, &s, mask, NULL, &s, (int32_t *)&s, (const int32_t *)&s, &s, two, NULL) == LYCHEE_EINVAL);
    CHECK(lychee_dense_decode_attn(NULL, &s, &s, &s, &s, &s, (const int32_t *)&s, &s, one, NULL) == LYCHEE_EINVAL);
    CHECK(lychee_decode_step(NULL, &s, 2, NULL, NULL, NULL, mask, NULL, NULL, NULL, NULL, NULL, 0, NULL) == LYCHEE_EINVAL);
    CHECK(lychee_append_kv(NULL, &s, &s, &s, &s, &s, (const int32_t *)&s, NULL) == LYCHEE_EINVAL);
    CHECK(lychee_select_stats(NULL, &a, &b, NULL) == LYCHEE_EINVAL);
    CHECK(lychee_timing_enable(NULL, 1) == LYCHEE_EINVAL);
    CHECK(lychee_timing_read(NULL, ms, n) == LYCHEE_EINVAL);

    /* messages */
    CHECK(strcmp(lychee_strerror(LYCHEE_OK), "ok") == 0);
    CHECK(strlen(lychee_strerror(LYCHEE_EWORKSPACE)) > 0);
    CHECK(strlen(lychee_strerror(-99)) > 0);

    printf(failures ? "%d checks failed\n" : "all checks passed%.0d\n", failures);
    return failures != 0;
}
