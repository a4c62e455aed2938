"""Pins of the eps-draw oracle (Philox-4x32-10 + Box-Muller, see oracle/eps_oracle.c).

Expected values come from the Philox publication's known-answer vectors, from the
invertibility of the round structure, from exact integer arithmetic done here in Python, and
from what a standard normal sample must satisfy; none is produced by the oracle itself."""
import math
import os

import numpy as np
import pytest
from scipy import stats

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
M0, M1, W0, W1 = 0xD2511F53, 0xCD9E8D57, 0x9E3779B9, 0xBB67AE85
MASK = 0xFFFFFFFF


def test_philox_known_answers(oracle):
    rows = [l.split() for l in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) if l.strip() and l[0] != "#"]
    assert len(rows) == 3
    for r in rows:
        v = [int(x, 16) for x in r]
        assert oracle.philox4x32(v[0:4], v[4:6], 10) == v[6:10]


def _inverse(out, key, rounds):
    """Undo the rounds: the low product words give back the multiplied counter words through
    the inverses of the odd multipliers mod 2^32; the high words then unmask the other two."""
    inv0, inv1 = pow(M0, -1, 1 << 32), pow(M1, -1, 1 << 32)
    c = list(out)
    for r in reversed(range(rounds)):
        k0 = (key[0] + r * W0) & MASK
        k1 = (key[1] + r * W1) & MASK
        p0 = (c[3] * inv0) & MASK            # counter word 0 before the round
        p2 = (c[1] * inv1) & MASK            # counter word 2 before the round
        hi0 = (M0 * p0) >> 32
        hi1 = (M1 * p2) >> 32
        c = [p0, c[0] ^ hi1 ^ k0, p2, c[2] ^ hi0 ^ k1]
    return c


@pytest.mark.parametrize("rounds", [1, 2, 7, 10])
def test_philox_is_a_bijection_with_this_round_structure(oracle, rounds):
    rng = np.random.default_rng(rounds)
    for _ in range(50):
        ctr = [int(v) for v in rng.integers(0, 1 << 32, size=4)]
        key = [int(v) for v in rng.integers(0, 1 << 32, size=2)]
        assert _inverse(oracle.philox4x32(ctr, key, rounds), key, rounds) == ctr


def test_one_round_by_hand(oracle):
    # counter (1, 2, 3, 4), key (5, 6), one round, multiplied out in Python integers
    p0, p1 = M0 * 1, M1 * 3
    want = [(p1 >> 32) ^ 2 ^ 5, p1 & MASK, (p0 >> 32) ^ 4 ^ 6, p0 & MASK]
    assert oracle.philox4x32([1, 2, 3, 4], [5, 6], 1) == want


def test_counter_layout(oracle):
    seed, step = 0x0123456789ABCDEF, 7
    a = oracle.eps_bits(1003, 5, seed, step, first_sample=0)
    # the same global sample index gives the same stream whichever GPU owns it
    b = oracle.eps_bits(1003, 2, seed, step, first_sample=3)
    assert np.array_equal(a[3:5], b)
    # a shorter weight vector is a prefix
    assert np.array_equal(oracle.eps_bits(10, 5, seed, step), a[:, :10])
    # every argument matters, and both halves of the seed do
    for other in (oracle.eps_bits(1003, 5, seed, step + 1), oracle.eps_bits(1003, 5, seed ^ 1, step),
                  oracle.eps_bits(1003, 5, seed ^ (1 << 40), step), oracle.eps_bits(1003, 5, seed, step, 1)):
        assert not np.array_equal(a, other)
        assert np.mean(a == other) < 1e-3
    # quad q of sample t is Philox(counter = (q, 0, t, step), key = seed halves), words in order
    q, t = 57, 4
    want = oracle.philox4x32([q, 0, t, step], [seed & MASK, seed >> 32], 10)
    assert a[t, 4 * q:4 * q + 4].tolist() == want
    # quads beyond 2^32 carry into the second counter word
    q = (1 << 32) + 1
    hi = oracle.eps_bits(8, 1, seed, step, first_sample=2, col0=4 * q)
    assert hi[0, :4].tolist() == oracle.philox4x32([1, 1, 2, step], [seed & MASK, seed >> 32], 10)
    assert hi[0, 4:].tolist() == oracle.philox4x32([2, 1, 2, step], [seed & MASK, seed >> 32], 10)
    # a window of weights is the same as the matching columns of the whole
    assert np.array_equal(oracle.eps_bits(100, 5, seed, step, col0=37), a[:, 37:137])
    np.testing.assert_array_equal(oracle.eps_normal(100, 5, seed, step, col0=37),
                                  oracle.eps_normal(1003, 5, seed, step)[:, 37:137])
    # all words distinct enough: no repeated quads
    assert len(np.unique(a)) > 0.999 * a.size


def test_float_stage_is_box_muller_of_the_words(oracle):
    seed, n, s = 99, 4001, 3
    bits = oracle.eps_bits(n, s, seed).astype(np.int64)
    eps, rad = oracle.eps_normal(n, s, seed, with_radius=True)
    m = n - n % 4
    x = bits[:, :m].reshape(s, m // 4, 4)
    e = eps[:, :m].reshape(s, m // 4, 4)
    r = rad[:, :m].reshape(s, m // 4, 4)
    for p in (0, 1):
        u = ((x[..., 2 * p] >> 8) + 1) / 2.0 ** 24
        f = (x[..., 2 * p + 1] >> 8) / 2.0 ** 24
        assert np.all((u > 0) & (u <= 1)) and np.all((f >= 0) & (f < 1))
        np.testing.assert_allclose(np.exp(-0.5 * r[..., 2 * p] ** 2), u, rtol=1e-12)
        np.testing.assert_array_equal(r[..., 2 * p], r[..., 2 * p + 1])
        np.testing.assert_allclose(e[..., 2 * p] ** 2 + e[..., 2 * p + 1] ** 2, r[..., 2 * p] ** 2, rtol=1e-12, atol=1e-300)
        ang = np.arctan2(e[..., 2 * p + 1], e[..., 2 * p]) / (2 * math.pi) % 1.0
        ok = r[..., 2 * p] > 0
        d = np.abs(ang - f)[ok]
        assert np.all(np.minimum(d, 1 - d) < 1e-12)
    # the ragged last quad uses the leading words of its quad
    full = oracle.eps_normal(n + 3, s, seed)
    np.testing.assert_array_equal(full[:, :n], eps)


def test_draws_are_standard_normal(oracle):
    n, s = 1_000_000, 4
    e = oracle.eps_normal(n, s, seed=2024, step=1)
    x = e.ravel()
    m = x.size
    assert abs(x.mean()) < 5 / math.sqrt(m)
    assert abs(x.var() - 1) < 5 * math.sqrt(2 / m)
    assert abs(stats.skew(x)) < 5 * math.sqrt(6 / m)
    assert abs(stats.kurtosis(x)) < 5 * math.sqrt(24 / m)
    d, p = stats.kstest(x[::7], "norm")
    assert p > 1e-3, (d, p)
    assert np.max(np.abs(x)) < 5.78          # u >= 2^-24 bounds the radius by sqrt(48 ln 2)
    # tail mass beyond 3 sigma: 2.6998e-3
    tail = np.mean(np.abs(x) > 3)
    assert abs(tail - 2.6998e-3) < 5 * math.sqrt(2.6998e-3 / m)
    # independence: the two outputs of a pair, neighbouring quads, neighbouring samples
    for a, b in ((e[:, 0::4], e[:, 1::4]), (e[:, 0:-4:4], e[:, 4::4]), (e[0], e[1]), (e[:, 0::4] ** 2, e[:, 1::4] ** 2)):
        a, b = a.ravel(), b.ravel()
        c = np.corrcoef(a, b)[0, 1]
        assert abs(c) < 5 / math.sqrt(a.size)


def test_word_bits_are_uniform(oracle):
    bits = oracle.eps_bits(400_000, 2, seed=5)
    for shift in (0, 8, 16, 24):
        counts = np.bincount((bits.ravel() >> shift) & 0xFF, minlength=256)
        chi2 = np.sum((counts - counts.mean()) ** 2 / counts.mean())
        assert chi2 < 400, (shift, chi2)      # 255 degrees of freedom: mean 255, sd 22.6


def test_frozen_sample_of_the_definition(oracle):
    """tests/golden/eps_draw_seed42.txt was written by the oracle (make_eps_golden.py); it freezes the
    definition, so any later change to generator, counter layout or Box-Muller mapping shows up here."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "eps_draw_seed42.txt")) if l[0] != "#"]
    col0 = int(rows[0][1])
    n = len(rows) // 2
    bits = oracle.eps_bits(n, 2, 42, 3, 5, col0=col0)
    eps = oracle.eps_normal(n, 2, 42, 3, 5, col0=col0)
    for s, i, word, e in rows:
        s, i = int(s), int(i) - col0
        assert int(bits[s, i]) == int(word, 16)
        assert eps[s, i] == float(e)
