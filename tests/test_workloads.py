"""The synthetic parameter sets have the stated tensor counts, sizes and value recipes."""
import math

import numpy as np
import pytest
import torch

from paper_2005_06728_amd import workloads as wl

EXPECT = {  # name: (tensors, parameters, workers)
    "lenet5": (10, 61706, 4),
    "resnet20": (65, 272474, 8),
    "resnet50": (161, 25557032, 8),
    "alexnet": (16, 61100840, 16),
    "vgg16": (32, 138357544, 16),
}


@pytest.mark.parametrize("name", list(EXPECT))
def test_shapes(name):
    w = wl.WORKLOADS[name]
    K, N, W = EXPECT[name]
    assert len(w.tensors) == K and wl.total_params(w) == N and w.num_workers == W


def test_odd_sized_tensors_present():
    assert sorted(n for n in wl.numels(wl.WORKLOADS["lenet5"]) if n % 4) == [6, 10, 150]
    assert [n for n in wl.numels(wl.WORKLOADS["resnet20"]) if n % 4] == [10]
    assert max(wl.numels(wl.WORKLOADS["vgg16"])) == 102760448


def test_generation_is_seeded_and_distributions_match():
    w = wl.WORKLOADS["resnet20"]
    a = wl.allocate(w, "cpu")
    b = wl.allocate(w, "cpu")
    for x, y in zip(a["w"], b["w"]):
        assert torch.equal(x, y)
    wl.fill_all_grads_(a, w, 3)
    wl.fill_all_grads_(b, w, 3)
    assert torch.equal(a["g"][5][10], b["g"][5][10])
    wl.fill_all_grads_(b, w, 4)
    assert not torch.equal(a["g"][5][10], b["g"][5][10])
    assert not torch.equal(a["g"][0][10], a["g"][1][10])
    # He-normal conv weights, BN scale one, biases zero, momentum zero, locals = w_0
    for t, buf in zip(w.tensors, a["w"]):
        if t.kind == "bn_scale":
            assert torch.all(buf == 1)
        elif t.kind == "bias":
            assert torch.all(buf == 0)
    big = max(range(len(w.tensors)), key=lambda k: a["w"][k].numel())
    fan_in = math.prod(w.tensors[big].shape[1:])
    assert abs(a["w"][big].std().item() / math.sqrt(2 / fan_in) - 1) < 0.05
    assert all(torch.all(v == 0) for v in a["v"])
    assert torch.equal(a["u"][3][big], a["w"][big])
    # heavy tail: about 1 % of entries are 100x larger
    g = torch.cat([x for x in a["g"][0]])
    frac = (g.abs() > 8e-3).float().mean().item()
    assert 0.005 < frac < 0.015
    assert abs(g[g.abs() < 4e-3].std().item() / 1e-3 - 1) < 0.05


def test_exact_zero_mask():
    w = wl.WORKLOADS["vgg16"]
    buf = [torch.empty(200000)]
    wl.fill_grads_(buf, w, 0, 0)
    z = (buf[0] == 0).float().mean().item()
    assert 0.0005 < z < 0.0015
    assert abs(buf[0].std().item() / 1e-4 - 1) < 0.05
