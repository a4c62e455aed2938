/*
 * Calls the host-side paths of libhot that need no GPU (argument validation of every entry point, the
 * host-only queries) against a build of the library whose HOST code is compiled with
 * -fsanitize=address,undefined, so that a wild read in a validation path or an overflow in the host
 * arithmetic aborts the program.  Every call here must return before anything is launched.
 * Test infrastructure; built and run by tests/test_sanitizers_cpu.py.  Prints "abi driver ok".
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "hot.h"

static int failures = 0;
#define CHECK(cond) do { if (!(cond)) { fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #cond); ++failures; } } while (0)

int main(void)
{
    CHECK(hot_version() == HOT_VERSION);
    CHECK(strcmp(hot_strerror(HOT_OK), "success") == 0);
    CHECK(strstr(hot_strerror(HOT_EINVAL), "invalid") != NULL && strstr(hot_strerror(HOT_ERANGE), "capacity") != NULL);
    CHECK(strcmp(hot_strerror(-99), "unknown error code") == 0);
    CHECK(hot_recommended_ld(1) == 64 && hot_recommended_ld(32024) == 32064 && hot_recommended_ld(0) == HOT_EINVAL);
    CHECK(hot_recommended_ld(INT64_MAX - 100) < 0 || hot_recommended_ld(INT64_MAX - 100) >= INT64_MAX - 100);

    /* a heap block of exactly 16 floats stands for every array: no valid call may read past it on the host */
    float *buf = malloc(16 * sizeof(float));
    double *dbl = malloc(2 * sizeof(double));
    if (!buf || !dbl) abort();
    memset(buf, 0, 16 * sizeof(float));
    float *odd = (float *)((char *)buf + 2);       /* not 4-byte aligned */

    hot_plan *plan = (hot_plan *)0;
    CHECK(hot_create(NULL, NULL) == HOT_EINVAL);
    const hot_desc bad[] = {
        {0, 0, 1, 1, 1.0, 0, 0}, {8, 7, 1, 1, 1.0, 0, 0}, {8, 8, 0, 1, 1.0, 0, 0}, {8, 8, 3, 2, 1.0, 0, 0},
        {8, 8, 1, 1, 0.0, 0, 0}, {8, 8, 1, 1, -1.0, 0, 0}, {8, 8, 1, 1, 1.0, 0, 3},
        {INT64_MAX / 2, INT64_MAX / 2, 7, 7, 1.0, 0, 0}};
    for (size_t i = 0; i < sizeof bad / sizeof bad[0]; ++i) {
        CHECK(hot_create(&plan, &bad[i]) == HOT_EINVAL && plan == NULL);
        CHECK(hot_forward_static(&bad[i], buf, buf, buf, buf, NULL, NULL) == HOT_EINVAL);
    }
    const hot_desc too_big = {HOT_STATIC_MAX_WEIGHTS + 1LL, HOT_STATIC_MAX_WEIGHTS + 1LL, 1, 1, 1.0, 0, 0};
    CHECK(hot_forward_static(&too_big, buf, buf, buf, buf, NULL, NULL) == HOT_ERANGE);
    const hot_desc far_device = {16, 16, 1, 1, 1.0, 4096, 0}, neg_device = {16, 16, 1, 1, 1.0, -1, 0};
    CHECK(hot_forward_static(&far_device, buf, buf, buf, buf, NULL, NULL) == HOT_EINVAL);
    CHECK(hot_forward_static(&neg_device, buf, buf, buf, buf, NULL, NULL) == HOT_EINVAL);
    const hot_desc ok16 = {16, 16, 1, 1, 1.0, 0, 0};
    CHECK(hot_forward_static(&ok16, NULL, buf, buf, buf, NULL, NULL) == HOT_EINVAL);
    CHECK(hot_forward_static(&ok16, buf, odd, buf, buf, NULL, NULL) == HOT_EINVAL);
    CHECK(hot_forward_static(&ok16, buf, buf, buf, buf, (double *)((char *)dbl + 4), NULL) == HOT_EINVAL);
    CHECK(hot_forward_static(NULL, buf, buf, buf, buf, NULL, NULL) == HOT_EINVAL);

    CHECK(hot_destroy(NULL) == HOT_OK);
    CHECK(hot_forward(NULL, buf, buf, buf, buf, NULL, NULL) == HOT_EINVAL);
    CHECK(hot_kl(NULL, buf, buf, dbl, NULL) == HOT_EINVAL);
    CHECK(hot_backward(NULL, buf, buf, buf, buf, buf, buf, NULL) == HOT_EINVAL);
    const hot_rng rng = {1, 0, 0};
    CHECK(hot_forward_rng(NULL, &rng, buf, buf, buf, NULL, NULL) == HOT_EINVAL);
    CHECK(hot_backward_rng(NULL, &rng, buf, buf, buf, buf, buf, NULL) == HOT_EINVAL);
    CHECK(hot_backward_rows(NULL, &rng, buf, buf, NULL, buf, 0, 1, 0, 1, buf, buf, NULL) == HOT_EINVAL);
    CHECK(hot_sample_eps(NULL, &rng, buf, NULL) == HOT_EINVAL && hot_sample_bits(NULL, &rng, (uint32_t *)buf, NULL) == HOT_EINVAL);
    hot_launch cfg = {0, 0, 0, 0};
    CHECK(hot_set_launch(NULL, 0, &cfg) == HOT_EINVAL && hot_get_launch(NULL, 0, &cfg) == HOT_EINVAL);
    CHECK(hot_last_hip_error(NULL) == 0);
    const hot_adam adam = {1e-3, 0.9, 0.999, 1e-8, 1.0, 0.0, 1}, adam_bad = {1e-3, 0.9, 0.999, 1e-8, 1.0, 0.0, 0};
    CHECK(hot_adam_step(NULL, 16, buf, buf, buf, buf, buf, buf, buf, buf, NULL) == HOT_EINVAL);
    CHECK(hot_adam_step(&adam_bad, 16, buf, buf, buf, buf, buf, buf, buf, buf, NULL) == HOT_EINVAL);
    CHECK(hot_adam_step(&adam, 0, buf, buf, buf, buf, buf, buf, buf, buf, NULL) == HOT_EINVAL);
    CHECK(hot_adam_step(&adam, 16, buf, buf, buf, NULL, buf, buf, buf, buf, NULL) == HOT_EINVAL);
    CHECK(hot_backward_adam(NULL, &rng, &adam, buf, buf, NULL, buf, buf, buf, buf, buf, NULL) == HOT_EINVAL);
    CHECK(hot_backward_adam_forward(NULL, &rng, &rng, &adam, buf, buf, buf, buf, buf, buf, buf, buf, NULL, NULL) == HOT_EINVAL);
    CHECK(hot_adam_forward(NULL, &rng, &adam, buf, buf, buf, buf, buf, buf, buf, buf, NULL, buf, NULL, NULL) == HOT_EINVAL);

    CHECK(hot_forward_dropout_rng(NULL, &rng, 0.5, buf, buf, NULL) == HOT_EINVAL);
    CHECK(hot_forward_dropout_rng(&ok16, &rng, 0.0, buf, buf, NULL) == HOT_EINVAL);
    CHECK(hot_forward_dropout_rng(&ok16, &rng, 1.5, buf, buf, NULL) == HOT_EINVAL);
    CHECK(hot_forward_dropout_rng(&ok16, NULL, 0.5, buf, buf, NULL) == HOT_EINVAL);
    CHECK(hot_backward_dropout_rng(&ok16, &rng, 0.5, NULL, buf, NULL) == HOT_EINVAL);
    CHECK(hot_forward_dropout_units_rng(&ok16, &rng, 0.5, 2, 0, buf, buf, NULL) == HOT_EINVAL);
    CHECK(hot_backward_dropout_units_rng(&ok16, &rng, 0.5, 4, 3, buf, buf, NULL) == HOT_EINVAL);

    CHECK(hot_stats_local(NULL, 1, 1, 1, dbl, dbl, NULL) == HOT_EINVAL);
    CHECK(hot_stats_local(buf, 4, 2, 1, dbl, dbl, NULL) == HOT_EINVAL);
    CHECK(hot_stats_whole(buf, 4, 4, 1, 1, buf, buf, NULL) == HOT_EINVAL || hot_stats_whole(buf, 4, 4, 1, 1, buf, buf, NULL) == HOT_EHIP);
    const int32_t counts[2] = {1, 0};
    CHECK(hot_stats_merge(dbl, dbl, NULL, 1, 1, 1, 0, buf, buf, NULL) == HOT_EINVAL);
    CHECK(hot_stats_merge(dbl, dbl, counts, 2, 1, 1, 0, buf, buf, NULL) == HOT_EINVAL);
    CHECK(hot_stats_merge(dbl, dbl, counts, 65, 1, 1, 0, buf, buf, NULL) == HOT_EINVAL);

    hot_linear_desc lin = {4, 8, 2, 8, 0, 0, 1, 0, 0};
    CHECK(hot_linear_forward_rng(NULL, &rng, buf, buf, buf, NULL, NULL, buf, NULL) == HOT_EINVAL);
    lin.in_features = 6;       /* not a multiple of 4 */
    CHECK(hot_linear_forward_rng(&lin, &rng, buf, buf, buf, NULL, NULL, buf, NULL) == HOT_EINVAL);
    CHECK(hot_linear_backward_workspace_bytes(&lin) == HOT_EINVAL);
    lin.in_features = 8;
    lin.reserved = 1;
    CHECK(hot_linear_forward_rng(&lin, &rng, buf, buf, buf, NULL, NULL, buf, NULL) == HOT_EINVAL);
    lin.reserved = 0;
    CHECK(hot_linear_forward_rng(&lin, &rng, buf, buf, buf, buf, NULL, buf, NULL) == HOT_EINVAL);     /* one bias array only */
    CHECK(hot_linear_backward_rng(&lin, 0, 1.0, 0, &rng, buf, buf, buf, buf, NULL, NULL, buf, buf, NULL, NULL, NULL, NULL) == HOT_EINVAL);
    CHECK(hot_linear_backward_rng(&lin, 1, 1.0, 7, &rng, buf, buf, buf, buf, NULL, NULL, buf, buf, NULL, NULL, NULL, NULL) == HOT_EINVAL);
    CHECK(hot_linear_backward_rng_ws(&lin, 1, 1.0, 0, &rng, buf, buf, buf, buf, NULL, NULL, buf, buf, NULL, NULL, NULL, odd, 64, NULL) == HOT_EINVAL);
    CHECK(hot_linear_backward_workspace_bytes(NULL) == HOT_EINVAL);
    /* the workspace query is host arithmetic over the whole range of sizes: no overflow may occur in it */
    int64_t most = 0;
    const int64_t rows[] = {1, 255, 256, 7260, 16640, 1 << 20, INT64_MAX / 4096};
    const int64_t ks[] = {4, 64, 192, 540, 4096, 1 << 20};
    const int64_t os[] = {1, 15, 768, 2160, 1 << 20, INT64_MAX / (1 << 22)};
    for (size_t a = 0; a < sizeof rows / sizeof rows[0]; ++a)
        for (size_t b = 0; b < sizeof ks / sizeof ks[0]; ++b)
            for (size_t c = 0; c < sizeof os / sizeof os[0]; ++c)
                for (int32_t s = 1; s <= 16; s *= 4) {
                    const hot_linear_desc d = {rows[a], ks[b], os[c], ks[b], 0, 0, s, 0, 0};
                    const int64_t bytes = hot_linear_backward_workspace_bytes(&d);
                    CHECK(bytes >= 0 || bytes == HOT_EINVAL);
                    if (bytes > most) most = bytes;
                }
    CHECK(most > 0);

    CHECK(hot_probe_copy(NULL, NULL, 16, 0, NULL) == HOT_EINVAL && hot_probe_copy(buf, buf, 24, 0, NULL) == HOT_EINVAL);
    CHECK(hot_probe_streams(NULL, 16, 1, 1, NULL) == HOT_EINVAL);

    free(buf);
    free(dbl);
    if (failures) {
        fprintf(stderr, "abi driver: %d check(s) failed\n", failures);
        return 1;
    }
    puts("abi driver ok");
    return 0;
}
