"""Pins of the predictive-statistics oracle (oracle/stats_oracle.c): closed forms, numpy's own
mean / std as the library special case, shift and scale laws, and the exactness of merging the
per-GPU partials, which is what the paper's "exact algorithm" with two communicated numbers per
output relies on (arxiv 2604.04736, paragraphs after Algorithm 2)."""
import math

import numpy as np
import pytest

f32 = np.float32


def test_closed_forms(oracle):
    s, m = 16, 5
    y = np.zeros((s, m), f32)
    y[:, 0] = 3.25                                   # constant: std 0
    y[:, 1] = np.arange(1, s + 1)                    # 1..S: mean (S+1)/2, population variance (S^2-1)/12
    y[:, 2] = np.where(np.arange(s) % 2 == 0, -2.0, 2.0)   # +-2 alternating: mean 0, population std 2
    y[:, 3] = [1] + [0] * (s - 1)                    # one-hot: mean 1/S, variance (1/S)(1-1/S)
    y[:, 4] = -7.5
    mean, std = oracle.stats_whole(y, ddof=0)
    np.testing.assert_allclose(mean, [3.25, (s + 1) / 2, 0.0, 1 / s, -7.5], rtol=1e-15)
    np.testing.assert_allclose(std, [0.0, math.sqrt((s * s - 1) / 12), 2.0, math.sqrt((1 / s) * (1 - 1 / s)), 0.0],
                               rtol=1e-15)
    _, std1 = oracle.stats_whole(y, ddof=1)
    np.testing.assert_allclose(std1, std * math.sqrt(s / (s - 1)), rtol=1e-15)
    pm, m2 = oracle.stats_partial(y)
    np.testing.assert_allclose(pm, mean, rtol=1e-15)
    np.testing.assert_allclose(m2, s * std ** 2, rtol=1e-14)


@pytest.mark.parametrize("ddof", [0, 1])
def test_reduces_to_numpy_mean_and_std(oracle, ddof):
    r = np.random.default_rng(1)
    y = (r.normal(size=(13, 301)) * 10 ** r.uniform(-3, 3, size=301) + r.normal(size=301) * 100).astype(f32)
    mean, std = oracle.stats_whole(y, ddof=ddof)
    y64 = y.astype(np.float64)
    np.testing.assert_allclose(mean, y64.mean(axis=0), rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(std, y64.std(axis=0, ddof=ddof), rtol=1e-10)


def test_pitch_and_padding(oracle):
    r = np.random.default_rng(2)
    y = np.full((4, 40), np.nan, f32)
    y[:, :33] = r.normal(size=(4, 33))
    a = oracle.stats_whole(y, m=33)
    b = oracle.stats_whole(np.ascontiguousarray(y[:, :33]))
    np.testing.assert_array_equal(a[0], b[0])
    np.testing.assert_array_equal(a[1], b[1])
    assert np.all(np.isfinite(a[0])) and np.all(np.isfinite(a[1]))


def test_shift_and_scale_laws(oracle):
    r = np.random.default_rng(3)
    y = r.integers(-50, 50, size=(9, 64)).astype(f32)          # small integers: shifts and scalings are exact in fp32
    mean, std = oracle.stats_whole(y)
    mean_s, std_s = oracle.stats_whole(y + f32(1024.0))
    np.testing.assert_allclose(mean_s, mean + 1024.0, rtol=1e-15)
    np.testing.assert_allclose(std_s, std, rtol=1e-13)
    mean_c, std_c = oracle.stats_whole(y * f32(-8.0))
    np.testing.assert_allclose(mean_c, -8.0 * mean, rtol=1e-15)
    np.testing.assert_allclose(std_c, 8.0 * std, rtol=1e-15)
    # permuting the samples changes nothing but rounding
    mean_p, std_p = oracle.stats_whole(y[r.permutation(9)])
    np.testing.assert_allclose(mean_p, mean, rtol=1e-14, atol=1e-14)
    np.testing.assert_allclose(std_p, std, rtol=1e-14)


@pytest.mark.parametrize("groups", [[16], [8, 8], [4, 4, 4, 4], [1] * 16, [13, 3], [1, 15], [5, 2, 9], [2] * 8])
@pytest.mark.parametrize("ddof", [0, 1])
def test_merging_partials_of_any_grouping_is_exact(oracle, groups, ddof):
    r = np.random.default_rng(4)
    s, m = 16, 257
    y = (r.normal(size=(s, m)) * 10 ** r.uniform(-4, 2, size=m) + 10 ** r.uniform(-2, 4, size=m)).astype(f32)
    whole_mean, whole_std = oracle.stats_whole(y, ddof=ddof)
    means, m2s, at = [], [], 0
    for g in groups:
        pm, pm2 = oracle.stats_partial(np.ascontiguousarray(y[at:at + g]))
        means.append(pm)
        m2s.append(pm2)
        at += g
    mean, std = oracle.stats_merge(groups, np.array(means), np.array(m2s), ddof=ddof)
    np.testing.assert_allclose(mean, whole_mean, rtol=1e-14)
    # the merged sum of squares loses digits only where the spread is far below the magnitude
    scale = np.abs(whole_mean) * 1e-15 * 10 + whole_std * 1e-12
    assert np.all(np.abs(std - whole_std) <= scale + 1e-12 * whole_std)


def test_single_sample_partials_carry_no_spread(oracle):
    y = np.array([[1.0, -2.0, 5.5]], f32)
    mean, m2 = oracle.stats_partial(y)
    np.testing.assert_array_equal(mean, [1.0, -2.0, 5.5])
    np.testing.assert_array_equal(m2, [0.0, 0.0, 0.0])


def test_exact_merge_gives_the_arithmetic_mean_of_class_probabilities(oracle):
    """The paper's example: with one sample per GPU, averaging the per-GPU cross-entropies is the
    cross-entropy of the GEOMETRIC mean of the class probabilities; the exact algorithm recovers
    the ARITHMETIC mean, on which the non-distributed loss is defined."""
    r = np.random.default_rng(5)
    s, classes = 8, 10
    logits = r.normal(size=(s, classes)) * 2
    probs = (np.exp(logits) / np.exp(logits).sum(1, keepdims=True)).astype(f32)
    label = 3
    per_gpu_ce = -np.log(probs[:, label].astype(np.float64))
    geometric = np.exp(np.mean(np.log(probs[:, label].astype(np.float64))))
    assert np.mean(per_gpu_ce) == pytest.approx(-math.log(geometric), rel=1e-13)
    means, m2s = zip(*(oracle.stats_partial(probs[i:i + 1].copy()) for i in range(s)))
    mean, _ = oracle.stats_merge([1] * s, np.array(means), np.array(m2s))
    arithmetic = probs[:, label].astype(np.float64).mean()
    assert mean[label] == pytest.approx(arithmetic, rel=1e-14)
    assert -math.log(mean[label]) < np.mean(per_gpu_ce)          # Jensen: the two losses differ
    assert mean.sum() == pytest.approx(1.0, abs=1e-6)
