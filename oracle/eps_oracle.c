/*
 * CPU oracle for the counter-based draw of eps ~ N(0, I) (Algorithm 2 of arxiv
 * 2604.04736, line "Sample eps_s ~ N(0, I)"; each GPU must draw samples that no other
 * GPU draws).  TEST INFRASTRUCTURE, not the product; shares no code with the HIP
 * library.
 *
 * The paper names no generator, so this build fixes one, as a definition both sides
 * implement independently:
 *
 *   integer stage   Philox-4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw, "Parallel
 *                   random numbers: as easy as 1, 2, 3", SC'11), written here from the
 *                   round description in that paper.
 *                     key     = (seed mod 2^32, seed div 2^32)
 *                     counter = (q mod 2^32, q div 2^32, t, step)
 *                   where q = i div 4 is the quad of weight i, t = first_sample + s is
 *                   the global index of local sample s (so GPUs with disjoint sample
 *                   ranges draw disjoint streams from one seed) and step counts
 *                   training steps.  The four output words x0..x3 belong to weights
 *                   4q .. 4q+3.
 *   float stage     Box-Muller on word pairs (x0, x1) and (x2, x3):
 *                     u = ((xa >> 8) + 1) / 2^24   in (0, 1]
 *                     f = (xb >> 8) / 2^24         in [0, 1)   (fraction of a turn)
 *                     r = sqrt(-2 ln u)
 *                     eps[4q + 2p]     = r cos(2 pi f)
 *                     eps[4q + 2p + 1] = r sin(2 pi f)         for pair p = 0, 1.
 *                   u and f are exact in fp32, so the two sides can differ only in the
 *                   rounding of ln, sqrt, cos, sin and the product.
 *
 * Pins (tests/test_eps_oracle_pins.py): the known-answer vectors published with the
 * Philox reference distribution, invertibility of the round structure, exact
 * integer-to-uniform mapping, moments / Kolmogorov-Smirnov distance / independence of the
 * normals.  Nothing here is "parity unpinned".
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

static const uint32_t PHILOX_M0 = 0xD2511F53u;
static const uint32_t PHILOX_M1 = 0xCD9E8D57u;
static const uint32_t PHILOX_W0 = 0x9E3779B9u; /* golden ratio */
static const uint32_t PHILOX_W1 = 0xBB67AE85u; /* sqrt(3) - 1 */

/* Philox-4x32-R: R rounds of { multiply two counter words by M0, M1; cross the high and
 * low halves; xor the key into the high halves }, with the key bumped by (W0, W1)
 * between rounds. */
void eps_oracle_philox4x32(const uint32_t ctr[4], const uint32_t key[2], int rounds, uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int r = 0; r < rounds; ++r) {
        if (r > 0) {
            k0 += PHILOX_W0;
            k1 += PHILOX_W1;
        }
        uint64_t p0 = (uint64_t)PHILOX_M0 * (uint64_t)c0;
        uint64_t p1 = (uint64_t)PHILOX_M1 * (uint64_t)c2;
        uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
        uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
        uint32_t n0 = hi1 ^ c1 ^ k0;
        uint32_t n1 = lo1;
        uint32_t n2 = hi0 ^ c3 ^ k1;
        uint32_t n3 = lo0;
        c0 = n0;
        c1 = n1;
        c2 = n2;
        c3 = n3;
    }
    out[0] = c0;
    out[1] = c1;
    out[2] = c2;
    out[3] = c3;
}

static void words_of(int64_t q, uint32_t t, uint64_t seed, uint32_t step, uint32_t x[4])
{
    uint32_t ctr[4] = {(uint32_t)((uint64_t)q & 0xFFFFFFFFu), (uint32_t)((uint64_t)q >> 32), t, step};
    uint32_t key[2] = {(uint32_t)(seed & 0xFFFFFFFFu), (uint32_t)(seed >> 32)};
    eps_oracle_philox4x32(ctr, key, 10, x);
}

/* Integer stage for weights col0 .. col0+n-1: bits[s, c] = word (i mod 4) of quad i div 4 of
 * sample first_sample + s, with i = col0 + c. */
void eps_oracle_bits(int64_t col0, int64_t n, int64_t ld_out, int32_t s_loc, uint64_t seed, uint32_t step,
                     uint32_t first_sample, uint32_t *bits)
{
    for (int32_t s = 0; s < s_loc; ++s)
        for (int64_t c = 0; c < n; ++c) {
            int64_t i = col0 + c;
            uint32_t x[4];
            words_of(i / 4, first_sample + (uint32_t)s, seed, step, x);
            bits[(size_t)s * (size_t)ld_out + (size_t)c] = x[i % 4];
        }
}

/* Both stages: eps[s, i] in fp64, and optionally the Box-Muller radius r[s, i] it was
 * scaled by (the natural magnitude for a tolerance on eps), for weights col0 .. col0+n-1.
 * radius may be NULL. */
void eps_oracle_normal(int64_t col0, int64_t n, int64_t ld_out, int32_t s_loc, uint64_t seed, uint32_t step,
                       uint32_t first_sample, double *eps, double *radius)
{
    const double two_pi = 6.283185307179586476925286766559;
    for (int32_t s = 0; s < s_loc; ++s)
        for (int64_t c = 0; c < n; ++c) {
            int64_t i = col0 + c;
            uint32_t x[4];
            words_of(i / 4, first_sample + (uint32_t)s, seed, step, x);
            int j = (int)(i % 4);
            int p = j / 2;
            double u = ((double)(x[2 * p] >> 8) + 1.0) / 16777216.0;
            double f = (double)(x[2 * p + 1] >> 8) / 16777216.0;
            double r = sqrt(-2.0 * log(u));
            double e = (j % 2 == 0) ? r * cos(two_pi * f) : r * sin(two_pi * f);
            eps[(size_t)s * (size_t)ld_out + (size_t)c] = e;
            if (radius) radius[(size_t)s * (size_t)ld_out + (size_t)c] = r;
        }
}
