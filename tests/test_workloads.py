"""The seeded input generator: integer stage against the published SplitMix64 test
vector, value distributions against the recipe, shapes against the paper's models."""
import math

import numpy as np
import torch

from paper_2604_04736_amd import workloads as W


def test_splitmix64_reference_vector():
    # first three outputs of SplitMix64 started from state 0 (Steele, Lea, Flood 2014;
    # the widely published test vector of the public-domain reference code)
    c = torch.arange(3, dtype=torch.int64)
    state = (c + 1) * W._signed(W._GOLDEN)
    got = [int(x) & W._MASK64 for x in W._mix(state)]
    assert got == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]
    assert [W._mix_int((k + 1) * W._GOLDEN) for k in range(3)] == got


def test_hash_is_a_pure_function_of_seed_stream_counter():
    k = torch.arange(1000, dtype=torch.int64)
    a = W.hash64(3, W.STREAM_EPS, k)
    b = torch.cat([W.hash64(3, W.STREAM_EPS, k[:137]), W.hash64(3, W.STREAM_EPS, k[137:])])
    assert torch.equal(a, b)
    assert not torch.equal(a, W.hash64(4, W.STREAM_EPS, k))
    assert not torch.equal(a, W.hash64(3, W.STREAM_G, k))
    assert len(set(a.tolist())) == 1000


def test_shapes_follow_the_papers_models():
    c = W.CONFIGS
    assert c["C1"].n_weights == 96 * 128 + 128 + 128 * 128 + 128 + 128 * 24 + 24 == 32_024
    assert c["C2"].n_weights == 2_693_578
    assert c["C3"].n_weights == 6 << 20 and c["C3"].s_local == c["C3"].s_total == 16
    assert c["C4"].n_weights == 200 << 20 and c["C4"].s_local == 2 and c["C4"].s_total == 16
    assert c["C5"].n_weights % 4 == 3 and c["C5"].ld == c["C5"].n_weights
    assert (c["C5"].s_local, c["C5"].s_total) == (13, 52)
    for wl in c.values():
        assert sum(l for l, _ in wl.segments) == wl.n_weights
        assert wl.ld >= wl.n_weights
    assert c["C1"].ld % 64 == 0 and c["C2"].ld % 64 == 0
    assert 0.9e5 < c["C1"].items < 2e5 and 0.9e7 < c["C2"].items < 2e7
    assert 0.9e8 < c["C3"].items < 2e8 and 0.9e8 < c["C5"].items < 2e8


def test_paper_value_distributions():
    wl = W.CONFIGS["C1"]
    d = W.make_inputs(wl)
    n = wl.n_weights
    assert d["mu"].shape == (n,) and d["eps"].shape == (wl.s_local, wl.ld)
    assert torch.isnan(d["eps"][:, n:]).all() and torch.isnan(d["G"][:, n:]).all()
    assert torch.isfinite(d["eps"][:, :n]).all() and torch.isfinite(d["G"][:, :n]).all()
    assert (d["sigma"] > 0).all()
    eps = d["eps"][:, :n].double()
    assert abs(float(eps.mean())) < 5 / math.sqrt(eps.numel())
    assert abs(float(eps.var()) - 1) < 5 * math.sqrt(2 / eps.numel())
    # first layer: 96*128 weights with fan_in 96 -> std sqrt(2/96)
    m = d["mu"][:96 * 128].double()
    assert abs(float(m.std()) / math.sqrt(2 / 96) - 1) < 0.03
    s = d["sigma"][:96 * 128].double()
    assert abs(float(s.log().mean()) - 0.5 * math.log(W.KAPPA / 96)) < 0.01
    # all elements distinct enough that an index bug cannot hide
    assert len(np.unique(d["mu"].numpy())) > 0.99 * n


def test_generation_is_reproducible_and_sliceable():
    wl = W.scaled(W.CONFIGS["C3"], 5000)
    a = W.make_inputs(wl)
    b = W.make_inputs(wl)
    for k in a:
        assert torch.equal(a[k], b[k])
    # a prefix of the full config is the same as the scaled config's mu
    z = W.normal(wl.seed, W.STREAM_MU, 100, 50, "cpu")
    fan = 192.0
    assert torch.equal((torch.sqrt(torch.tensor(2.0 / fan, dtype=torch.float64)) * z).float(), a["mu"][100:150])


def test_adversarial_recipe_and_misaligned_base():
    wl = W.scaled(W.CONFIGS["C5"], 200_003)
    d = W.make_inputs(wl, base_offset=1)
    for v in d.values():
        assert v.data_ptr() % 16 == 4
        assert torch.isfinite(v).all()
    assert wl.ld == wl.n_weights and wl.n_weights % 4 == 3
    sg = d["sigma"].double()
    assert (sg > 0).all()
    assert 0.05 < float((sg < 1e-6).double().mean()) < 0.15      # the underflowing-square class
    assert 0.003 < float(((sg - 1).abs() < 2e-3).double().mean()) < 0.03
    assert float(d["mu"].abs().max()) > 1e5 and float(d["mu"].abs().min()) < 1e-5
    e = d["eps"]
    assert int((e == 0).sum()) > 0 and int((e == 6).sum()) > 0 and int((e == -6).sum()) > 0
    # the common component makes the sum over samples cancel
    G = d["G"].double()
    assert float((G.sum(0).abs() / G.abs().sum(0)).median()) < 0.2
