/*
 * Runs every function of the CPU oracle on exactly sized heap buffers (pitched rows, ragged sizes, column
 * windows, optional pointers NULL) and checks closed-form values of each, so that a build with
 * -fsanitize=address,undefined sees every access the oracle makes: an index past an array, a misaligned or
 * overflowing operation aborts the program.  Test infrastructure; built and run by tests/test_sanitizers_cpu.py.
 * Prints "oracle driver ok" and returns 0 when every check holds.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    double lr, beta1, beta2, eps, grad_scale, sigma_min;
    int64_t step;
} update_oracle_adam_params;

void bbb_oracle_reparam(int64_t, int64_t, int32_t, const float *, const float *, const float *, double *, int64_t, int);
double bbb_oracle_kl(int64_t, const float *, const float *);
void bbb_oracle_grad(int64_t, int64_t, int32_t, int32_t, double, int, const float *, const float *, const float *,
                     const float *, double *, double *, int);
void eps_oracle_philox4x32(const uint32_t ctr[4], const uint32_t key[2], int rounds, uint32_t out[4]);
void eps_oracle_bits(int64_t, int64_t, int64_t, int32_t, uint64_t, uint32_t, uint32_t, uint32_t *);
void eps_oracle_normal(int64_t, int64_t, int64_t, int32_t, uint64_t, uint32_t, uint32_t, double *, double *);
void linear_oracle_forward(int32_t, int64_t, int64_t, int64_t, int64_t, int64_t, const float *, const float *, const float *,
                           const double *, const float *, const float *, const double *, double *);
void linear_oracle_backward(int32_t, int64_t, int64_t, int64_t, int64_t, int64_t, double, double, const float *,
                            const float *, const float *, const float *, const double *, const float *, const float *,
                            const double *, double *, double *, double *, double *, double *);
void stats_oracle_whole(int64_t, int64_t, int32_t, const float *, int32_t, double *, double *);
void stats_oracle_partial(int64_t, int64_t, int32_t, const float *, double *, double *);
void stats_oracle_merge(int32_t, int64_t, int64_t, const int32_t *, const double *, const double *, int32_t, double *, double *);
void update_oracle_adam(int64_t, const update_oracle_adam_params *, double *, double *, const double *, const double *,
                        double *, double *, double *, double *);
uint64_t update_oracle_dropout_threshold(double);
void update_oracle_dropout_forward(int64_t, int64_t, int32_t, double, const float *, const uint32_t *, double *);
void update_oracle_dropout_backward(int64_t, int64_t, int64_t, int32_t, int32_t, int, double, const float *,
                                    const uint32_t *, double *);

static int failures = 0;
#define CHECK(cond) do { if (!(cond)) { fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #cond); ++failures; } } while (0)

static int close_to(double a, double b, double rel) { return fabs(a - b) <= rel * (fabs(a) + fabs(b)) + 1e-300; }

static float *floats(size_t n) { float *p = malloc(n * sizeof(float)); if (!p) abort(); return p; }
static double *doubles(size_t n) { double *p = malloc(n * sizeof(double)); if (!p) abort(); return p; }

/* a small deterministic value in (-1, 1), different for every (tag, i) */
static float val(unsigned tag, size_t i)
{
    uint32_t h = (uint32_t)(i * 2654435761u) ^ (tag * 0x9E3779B9u);
    h ^= h >> 15; h *= 0x2C1B3C6Du; h ^= h >> 12;
    return (float)((double)(h & 0xFFFFFF) / 8388608.0 - 1.0);
}

static void sample_layer(int64_t n, int64_t ld, int32_t s_loc, int32_t s_total)
{
    /* eps and G end exactly at the last element read: (s_loc - 1) * ld + n floats */
    const size_t mat = (size_t)(s_loc - 1) * (size_t)ld + (size_t)n;
    float *mu = floats((size_t)n), *sg = floats((size_t)n), *eps = floats(mat), *G = floats(mat);
    for (int64_t i = 0; i < n; ++i) { mu[i] = val(1, (size_t)i); sg[i] = 0.5f + 0.4f * val(2, (size_t)i); }
    for (size_t i = 0; i < mat; ++i) { eps[i] = 3.0f * val(3, i); G[i] = val(4, i); }
    const int64_t ld_out = n + 3;
    double *w = doubles((size_t)(s_loc - 1) * (size_t)ld_out + (size_t)n);
    bbb_oracle_reparam(n, ld, s_loc, mu, sg, eps, w, ld_out, 3);
    for (int32_t s = 0; s < s_loc; ++s)
        for (int64_t i = 0; i < n; i += (n > 7 ? n / 7 : 1))
            CHECK(w[(size_t)s * (size_t)ld_out + (size_t)i] == (double)mu[i] + (double)sg[i] * (double)eps[(size_t)s * (size_t)ld + (size_t)i]);
    const double kl = bbb_oracle_kl(n, mu, sg);
    CHECK(kl > 0.0);
    double *gm = doubles((size_t)n), *gs = doubles((size_t)n);
    for (int mean = 0; mean < 2; ++mean) {
        bbb_oracle_grad(n, ld, s_loc, s_total, 45000.0, mean, mu, sg, eps, G, gm, gs, 2);
        const double g = mean ? 1.0 / s_loc : 1.0 / s_total, k = mean ? 1.0 / 45000.0 : (double)s_loc / (s_total * 45000.0);
        const int64_t i = n - 1;
        double a = 0.0, b = 0.0;
        for (int32_t s = 0; s < s_loc; ++s) {
            a += (double)G[(size_t)s * (size_t)ld + (size_t)i];
            b += (double)G[(size_t)s * (size_t)ld + (size_t)i] * (double)eps[(size_t)s * (size_t)ld + (size_t)i];
        }
        CHECK(close_to(gm[i], g * a + k * (double)mu[i], 1e-14));
        CHECK(close_to(gs[i], g * b + k * ((double)sg[i] - 1.0 / (double)sg[i]), 1e-14));
    }
    free(mu); free(sg); free(eps); free(G); free(w); free(gm); free(gs);
}

static void kl_closed_forms(void)
{
    /* per-weight values of the prior-matching line: (0,1) -> 0, (1,1) -> 1/2, (0,2) -> (3 - ln 4)/2, (0,1/2) -> (ln 4 - 3/4)/2 */
    float *mu = floats(4), *sg = floats(4);
    mu[0] = 0.0f; sg[0] = 1.0f; mu[1] = 1.0f; sg[1] = 1.0f; mu[2] = 0.0f; sg[2] = 2.0f; mu[3] = 0.0f; sg[3] = 0.5f;
    CHECK(bbb_oracle_kl(1, mu, sg) == 0.0);
    CHECK(bbb_oracle_kl(1, mu + 1, sg + 1) == 0.5);
    CHECK(close_to(bbb_oracle_kl(1, mu + 2, sg + 2), 0.5 * (3.0 - log(4.0)), 1e-15));
    CHECK(close_to(bbb_oracle_kl(1, mu + 3, sg + 3), 0.5 * (log(4.0) - 0.75), 1e-15));
    CHECK(close_to(bbb_oracle_kl(4, mu, sg), 0.5 + 0.5 * (3.0 - log(4.0)) + 0.5 * (log(4.0) - 0.75), 1e-15));
    free(mu); free(sg);
}

static void generator(void)
{
    /* the published known-answer vector of Philox-4x32-10 for an all-ones counter and key */
    const uint32_t ctr[4] = {0xffffffffu, 0xffffffffu, 0xffffffffu, 0xffffffffu}, key[2] = {0xffffffffu, 0xffffffffu};
    uint32_t out[4];
    eps_oracle_philox4x32(ctr, key, 10, out);
    CHECK(out[0] == 0x408f276du && out[1] == 0x41c83b0eu && out[2] == 0xa20bc7c6u && out[3] == 0x6d5451fdu);
    /* a window that starts inside a quad and ends inside another, pitched output, exactly sized */
    const int64_t col0 = 4294967296LL * 4 - 3, n = 11, ld = 13;
    const int32_t s_loc = 3;
    const size_t count = (size_t)(s_loc - 1) * (size_t)ld + (size_t)n;
    uint32_t *bits = malloc(count * sizeof(uint32_t));
    double *eps = doubles(count), *rad = doubles(count);
    if (!bits) abort();
    eps_oracle_bits(col0, n, ld, s_loc, 0x123456789abcdef0ULL, 7, 0xfffffffdu, bits);
    eps_oracle_normal(col0, n, ld, s_loc, 0x123456789abcdef0ULL, 7, 0xfffffffdu, eps, rad);
    eps_oracle_normal(col0, n, ld, s_loc, 0x123456789abcdef0ULL, 7, 0xfffffffdu, eps, NULL);
    for (int32_t s = 0; s < s_loc; ++s)
        for (int64_t c = 0; c + 1 < n; ++c) {
            const int64_t i = col0 + c;
            if (i % 2 == 0) {      /* a Box-Muller pair: cos and sin of one angle times one radius */
                const size_t at = (size_t)s * (size_t)ld + (size_t)c;
                CHECK(close_to(eps[at] * eps[at] + eps[at + 1] * eps[at + 1], rad[at] * rad[at], 1e-12));
                const double u = ((double)(bits[at] >> 8) + 1.0) / 16777216.0;
                CHECK(close_to(rad[at] * rad[at], -2.0 * log(u), 1e-12));
            }
        }
    free(bits); free(eps); free(rad);
}

static void linear_layer(int with_bias, int own_x, int with_dx)
{
    const int32_t s_loc = 2;
    const int64_t R = 5, K = 8, O = 3, ldx = 12;
    const int64_t xs = own_x ? R * ldx + 4 : 0;
    const size_t x_count = (size_t)(own_x ? (s_loc - 1) * xs : 0) + (size_t)(R - 1) * (size_t)ldx + (size_t)K;
    float *x = floats(x_count), *mu = floats((size_t)(O * K)), *sg = floats((size_t)(O * K));
    float *mb = floats((size_t)O), *sb = floats((size_t)O), *dy = floats((size_t)(s_loc * R * O));
    double *ew = doubles((size_t)(s_loc * O * K)), *eb = doubles((size_t)(s_loc * O));
    for (size_t i = 0; i < x_count; ++i) x[i] = val(5, i);
    for (size_t i = 0; i < (size_t)(O * K); ++i) { mu[i] = val(6, i); sg[i] = 0.3f + 0.2f * val(7, i); }
    for (size_t i = 0; i < (size_t)O; ++i) { mb[i] = val(8, i); sb[i] = 0.2f; }
    for (size_t i = 0; i < (size_t)(s_loc * R * O); ++i) dy[i] = val(9, i);
    for (size_t i = 0; i < (size_t)(s_loc * O * K); ++i) ew[i] = 2.0 * val(10, i);
    for (size_t i = 0; i < (size_t)(s_loc * O); ++i) eb[i] = val(11, i);
    double *y = doubles((size_t)(s_loc * R * O));
    linear_oracle_forward(s_loc, R, K, O, ldx, xs, x, mu, sg, ew, with_bias ? mb : NULL, with_bias ? sb : NULL,
                          with_bias ? eb : NULL, y);
    /* one output by hand */
    {
        const int32_t s = 1; const int64_t r = 4, o = 2;
        double acc = 0.0;
        for (int64_t k = 0; k < K; ++k)
            acc += (double)x[(size_t)s * (size_t)xs + (size_t)(r * ldx + k)] * ((double)mu[o * K + k] + (double)sg[o * K + k] * ew[(s * O + o) * K + k]);
        if (with_bias) acc += (double)mb[o] + (double)sb[o] * eb[s * O + o];
        CHECK(close_to(y[(s * R + r) * O + o], acc, 1e-14));
    }
    double *gmw = doubles((size_t)(O * K)), *gsw = doubles((size_t)(O * K)), *gmb = doubles((size_t)O), *gsb = doubles((size_t)O);
    double *dx = doubles((size_t)(s_loc * R * K));
    linear_oracle_backward(s_loc, R, K, O, ldx, xs, 0.25, 1e-3, x, dy, mu, sg, ew, with_bias ? mb : NULL,
                           with_bias ? sb : NULL, with_bias ? eb : NULL, gmw, gsw, with_bias ? gmb : NULL,
                           with_bias ? gsb : NULL, with_dx ? dx : NULL);
    {
        const int64_t o = 1, k = 7;
        double a = 0.0, b = 0.0;
        for (int32_t s = 0; s < s_loc; ++s) {
            double G = 0.0;
            for (int64_t r = 0; r < R; ++r) G += (double)dy[(s * R + r) * O + o] * (double)x[(size_t)s * (size_t)xs + (size_t)(r * ldx + k)];
            a += G;
            b += G * ew[(s * O + o) * K + k];
        }
        CHECK(close_to(gmw[o * K + k], 0.25 * a + 1e-3 * (double)mu[o * K + k], 1e-13));
        CHECK(close_to(gsw[o * K + k], 0.25 * b + 1e-3 * ((double)sg[o * K + k] - 1.0 / (double)sg[o * K + k]), 1e-13));
    }
    free(x); free(mu); free(sg); free(mb); free(sb); free(dy); free(ew); free(eb); free(y);
    free(gmw); free(gsw); free(gmb); free(gsb); free(dx);
}

static void statistics(void)
{
    const int64_t m = 7, ld = 9;
    const int32_t s = 6;
    const size_t count = (size_t)(s - 1) * (size_t)ld + (size_t)m;
    float *y = floats(count);
    for (size_t i = 0; i < count; ++i) y[i] = 10.0f * val(12, i);
    for (int32_t r = 0; r < s; ++r) y[(size_t)r * (size_t)ld] = (float)(r + 1);       /* column 0: 1..6 */
    double *mean = doubles((size_t)m), *sd = doubles((size_t)m);
    stats_oracle_whole(m, ld, s, y, 0, mean, sd);
    CHECK(mean[0] == 3.5 && close_to(sd[0], sqrt(35.0 / 12.0), 1e-15));
    stats_oracle_whole(m, ld, s, y, 1, mean, sd);
    CHECK(close_to(sd[0], sqrt(3.5), 1e-15));
    /* partials of 2 + 4 rows, merged, equal the whole */
    const int64_t ldp = m + 1;
    double *means = doubles((size_t)ldp + (size_t)m), *m2s = doubles((size_t)ldp + (size_t)m);
    stats_oracle_partial(m, ld, 2, y, means, m2s);
    stats_oracle_partial(m, ld, 4, y + 2 * ld, means + ldp, m2s + ldp);
    const int32_t counts[2] = {2, 4};
    double *mean2 = doubles((size_t)m), *sd2 = doubles((size_t)m);
    stats_oracle_merge(2, m, ldp, counts, means, m2s, 1, mean2, sd2);
    for (int64_t j = 0; j < m; ++j) CHECK(close_to(mean2[j], mean[j], 1e-13) && close_to(sd2[j], sd[j], 1e-13));
    free(y); free(mean); free(sd); free(means); free(m2s); free(mean2); free(sd2);
}

static void update_and_dropout(void)
{
    const int64_t n = 5;
    double *a[8];
    for (int i = 0; i < 8; ++i) a[i] = doubles((size_t)n);
    for (int64_t i = 0; i < n; ++i) {
        a[0][i] = val(13, (size_t)i); a[1][i] = 0.5; a[2][i] = 1.0 + val(14, (size_t)i); a[3][i] = -2.0;
        a[4][i] = a[5][i] = a[6][i] = a[7][i] = 0.0;
    }
    const double mu0 = a[0][2], g0 = a[2][2];
    const update_oracle_adam_params p = {1e-2, 0.9, 0.999, 1e-8, 1.0, 0.0, 1};
    update_oracle_adam(n, &p, a[0], a[1], a[2], a[3], a[4], a[5], a[6], a[7]);
    /* first step from zero moments: theta moves by lr * g / (|g| + eps) */
    CHECK(close_to(a[0][2], mu0 - 1e-2 * g0 / (fabs(g0) + 1e-8), 1e-12));
    CHECK(close_to(a[1][0], 0.5 + 1e-2 * 2.0 / (2.0 + 1e-8), 1e-12));
    for (int i = 0; i < 8; ++i) free(a[i]);

    CHECK(update_oracle_dropout_threshold(0.5) == 2147483648ULL && update_oracle_dropout_threshold(1.0) == 4294967296ULL);
    const int64_t nw = 3, ldw = 4, ldg = 5;
    const int32_t s_loc = 2;
    uint32_t *words = malloc(((size_t)ldw + (size_t)nw) * sizeof(uint32_t));
    float *mu = floats((size_t)nw), *G = floats((size_t)ldg + (size_t)nw);
    if (!words) abort();
    const uint32_t w0[3] = {0u, 0x7fffffffu, 0x80000000u}, w1[3] = {0xffffffffu, 5u, 0x40000000u};
    memcpy(words, w0, sizeof w0); memcpy(words + ldw, w1, sizeof w1);
    mu[0] = 2.0f; mu[1] = -4.0f; mu[2] = 8.0f;
    for (int i = 0; i < 3; ++i) { G[i] = (float)(i + 1); G[ldg + i] = 10.0f * (float)(i + 1); }
    double *w = doubles((size_t)(s_loc * nw)), *gm = doubles((size_t)nw);
    update_oracle_dropout_forward(nw, ldw, s_loc, 0.5, mu, words, w);
    CHECK(w[0] == 4.0 && w[1] == -8.0 && w[2] == 0.0 && w[3] == 0.0 && w[4] == -8.0 && w[5] == 16.0);
    update_oracle_dropout_backward(nw, ldg, ldw, s_loc, 4, 0, 0.5, G, words, gm);
    CHECK(gm[0] == 0.5 && gm[1] == 11.0 && gm[2] == 15.0);
    update_oracle_dropout_forward(nw, ldw, s_loc, 1.0, mu, words, w);
    CHECK(w[3] == 2.0);       /* keep = 1 keeps the largest word too */
    free(words); free(mu); free(G); free(w); free(gm);
}

int main(void)
{
    kl_closed_forms();
    sample_layer(1, 1, 1, 1);
    sample_layer(5, 5, 3, 12);
    sample_layer(1027, 1040, 4, 16);
    sample_layer(4099, 4099, 13, 52);
    generator();
    for (int bias = 0; bias < 2; ++bias)
        for (int own = 0; own < 2; ++own)
            for (int dx = 0; dx < 2; ++dx) linear_layer(bias, own, dx);
    statistics();
    update_and_dropout();
    if (failures) {
        fprintf(stderr, "oracle driver: %d check(s) failed\n", failures);
        return 1;
    }
    puts("oracle driver ok");
    return 0;
}
