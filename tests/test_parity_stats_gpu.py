"""GPU parity of the predictive statistics (hot_stats_local, hot_stats_merge) against the
two-pass fp64 oracle.

Tolerances.  Partials are fp64: the kernel works with shifted sums, whose cancellation is bounded
by the number of rows (sum (y-y0)^2 <= n * M2), so
    |mean - mean64| <= 1e-14 * max_s |y|,      |M2 - M2_64| <= 1e-12 * n * M2_64.
Final outputs are fp32:  |mean - mean64| <= 1e-6 * max_s |y|,
    |std - std64| <= 1e-6 * std64 + 1e-12 * max_s |y|   (the second term is the fp64 merge's
    own cancellation when the spread is far below the magnitude)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def hot():
    from paper_2604_04736_amd import binding
    binding.lib()
    assert torch.cuda.is_available()
    return binding


def _predictions(s, m, ld, seed):
    r = np.random.default_rng(seed)
    scale = 10 ** r.uniform(-4, 2, size=m)
    centre = 10 ** r.uniform(-2, 4, size=m) * r.choice([-1, 1], size=m)
    y = np.full((s, ld), np.nan, np.float32)
    y[:, :m] = (r.normal(size=(s, m)) * scale + centre).astype(np.float32)
    if m > 8:
        y[:, 3] = 42.0                      # constant column: spread exactly zero
        y[:, 5] = y[0, 5]                   # constant at an arbitrary fp32 value
        y[1:, 7] = 1000.0
        y[0, 7] = np.float32(1000.0) + np.float32(6.1035156e-05)   # one ulp of spread at magnitude 1000
    return y


def _local(hot, y_dev, m):
    mean = torch.full((m,), float("nan"), dtype=torch.float64, device=DEV)
    m2 = torch.full((m,), float("nan"), dtype=torch.float64, device=DEV)
    hot.hot_stats_local(y_dev[:, :m], mean, m2)
    torch.cuda.synchronize()
    return mean, m2


SHAPES = [(16, 2560, 2560, 0), (16, 1536, 1536, 0), (2, 69 * 121 * 240, 69 * 121 * 240, 0), (5, 1003, 1003, 0),
          (5, 1003, 1024, 0), (13, 70_001, 70_001, 1), (1, 7, 7, 0), (3, 1, 1, 0), (33, 4099, 4100, 3), (64, 300, 300, 0),
          # larger than the 256 MiB memory-side cache: the kernels then read with non-temporal hints
          (17, 4_000_000, 4_000_000, 0), (16, 4_200_003, 4_200_003, 1)]


@pytest.mark.parametrize("s,m,ld,offset", SHAPES)
def test_local_partials_match_oracle(oracle, hot, s, m, ld, offset):
    print("case stats local", s, m, ld, offset, flush=True)
    y = _predictions(s, m, ld, seed=s * 1000 + m)
    buf = torch.empty(s * ld + offset, device=DEV)
    yd = buf[offset:].view(s, ld)
    yd.copy_(torch.from_numpy(y))
    mean, m2 = _local(hot, yd, m)
    want_mean, want_m2 = oracle.stats_partial(y, m)
    big = np.abs(y[:, :m]).max(axis=0).astype(np.float64)
    assert np.all(np.abs(mean.cpu().numpy() - want_mean) <= 1e-14 * big)
    assert np.all(np.abs(m2.cpu().numpy() - want_m2) <= 1e-12 * s * want_m2)
    if m > 8:
        assert m2[3].item() == 0.0 and m2[5].item() == 0.0 and mean[3].item() == 42.0


@pytest.mark.parametrize("groups", [[16], [8, 8], [4] * 4, [1] * 16, [13, 3], [5, 2, 9]])
@pytest.mark.parametrize("ddof", [0, 1])
def test_merged_statistics_match_the_whole(oracle, hot, groups, ddof):
    s, m = sum(groups), 5000
    ld = 5003
    y = _predictions(s, m, ld, seed=77)
    yd = torch.from_numpy(y).to(DEV)
    parts = len(groups)
    means = torch.empty(parts, m, dtype=torch.float64, device=DEV)
    m2s = torch.empty(parts, m, dtype=torch.float64, device=DEV)
    at = 0
    for p, g in enumerate(groups):
        hot.hot_stats_local(yd[at:at + g, :m], means[p], m2s[p])
        at += g
    mean_out = torch.empty(m, device=DEV)
    std_out = torch.empty(m, device=DEV)
    hot.hot_stats_merge(means, m2s, groups, ddof, mean_out, std_out)
    torch.cuda.synchronize()
    big = np.abs(y[:, :m]).max(axis=0).astype(np.float64)
    # the merge kernel against the oracle's merge of the very same partials
    o_mean, o_std = oracle.stats_merge(groups, means.cpu().numpy(), m2s.cpu().numpy(), ddof)
    if not (ddof == 1 and s == 1):
        assert np.all(np.abs(mean_out.cpu().numpy() - o_mean) <= 1e-6 * big)
        assert np.all(np.abs(std_out.cpu().numpy() - o_std) <= 1e-6 * o_std + 1e-12 * big)
    # and the whole chain against the definition over all samples
    w_mean, w_std = oracle.stats_whole(y, m, ddof)
    assert np.all(np.abs(mean_out.cpu().numpy() - w_mean) <= 1e-6 * big)
    assert np.all(np.abs(std_out.cpu().numpy() - w_std) <= 1e-6 * w_std + 1e-12 * big)
    assert std_out[3].item() == 0.0


@pytest.mark.parametrize("s,m,ld,offset", SHAPES)
@pytest.mark.parametrize("ddof", [0, 1])
def test_one_pass_statistics_match_the_definition(oracle, hot, s, m, ld, offset, ddof):
    """hot_stats_whole (all samples on one GPU) against the two-pass definition, and bit for bit
    against hot_stats_local followed by hot_stats_merge of that single partial."""
    print("case stats whole", s, m, ld, offset, ddof, flush=True)
    y = _predictions(s, m, ld, seed=s * 1000 + m)
    buf = torch.empty(s * ld + offset, device=DEV)
    yd = buf[offset:].view(s, ld)
    yd.copy_(torch.from_numpy(y))
    mean_out = torch.full((m,), float("nan"), device=DEV)
    std_out = torch.full((m,), float("nan"), device=DEV)
    hot.hot_stats_whole(yd[:, :m], ddof, mean_out, std_out)
    mean, m2 = _local(hot, yd, m)
    mo2, so2 = torch.empty(m, device=DEV), torch.empty(m, device=DEV)
    hot.hot_stats_merge(mean.view(1, m), m2.view(1, m), [s], ddof, mo2, so2)
    torch.cuda.synchronize()
    if s == 1 and ddof == 1:
        assert torch.isnan(std_out).all()          # 0 / 0: no spread can be estimated from one sample
        return
    w_mean, w_std = oracle.stats_whole(y, m, ddof)
    big = np.abs(y[:, :m]).max(axis=0).astype(np.float64)
    assert np.all(np.abs(mean_out.cpu().numpy() - w_mean) <= 1e-6 * big)
    assert np.all(np.abs(std_out.cpu().numpy() - w_std) <= 1e-6 * w_std + 1e-12 * big)
    assert torch.equal(mean_out, mo2) and torch.equal(std_out, so2)


def test_single_gpu_finish_and_full_size_weather_shape(oracle, hot):
    # two samples of a 69 x 121 x 240 forecast: the local batch of the paper's third use case
    s, m = 2, 69 * 121 * 240
    y = _predictions(s, m, m, seed=5)
    yd = torch.from_numpy(y).to(DEV)
    mean, m2 = _local(hot, yd, m)
    mean_out, std_out = torch.empty(m, device=DEV), torch.empty(m, device=DEV)
    hot.hot_stats_merge(mean.view(1, m), m2.view(1, m), [s], 1, mean_out, std_out)
    torch.cuda.synchronize()
    w_mean, w_std = oracle.stats_whole(y, m, 1)
    big = np.abs(y).max(axis=0).astype(np.float64)
    assert np.all(np.abs(mean_out.cpu().numpy() - w_mean) <= 1e-6 * big)
    assert np.all(np.abs(std_out.cpu().numpy() - w_std) <= 1e-6 * w_std + 1e-12 * big)
    # numpy as a second witness
    np.testing.assert_allclose(std_out.cpu().numpy(), y.astype(np.float64).std(axis=0, ddof=1), rtol=2e-6, atol=1e-9)


def test_errors(hot):
    L = hot.lib()
    y = torch.zeros(4, 8, device=DEV)
    mean = torch.zeros(8, dtype=torch.float64, device=DEV)
    with pytest.raises(TypeError):
        hot.hot_stats_local(y, mean.float(), mean)
    with pytest.raises(TypeError):
        hot.hot_stats_local(y.double(), mean, mean.clone())
    means = torch.zeros(2, 8, dtype=torch.float64, device=DEV)
    out = torch.zeros(8, device=DEV)
    with pytest.raises(ValueError):
        hot.hot_stats_merge(means, means.clone(), [1], 0, out, out.clone())
    with pytest.raises(hot.HotError):
        hot.hot_stats_merge(means, means.clone(), [1, 0], 0, out, out.clone())
    with pytest.raises(hot.HotError):
        hot.hot_stats_merge(means, means.clone(), [1, 1], 2, out, out.clone())
    assert L.hot_stats_local(y.data_ptr(), 8, 4, 4, mean.data_ptr(), mean.data_ptr(), None) == hot.HOT_EINVAL   # ld < m
