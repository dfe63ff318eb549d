"""The shared input generators: determinism, distributions, storage encodings."""
import numpy as np
import torch

import workloads
from workloads import rng


def test_counter_based_slices_agree():
    a = rng.bits64(5, 0, 1000)
    b = rng.bits64(5, 400, 100)
    assert (a[400:500] == b).all()
    assert not (rng.bits64(6, 0, 1000) == a).any()


def test_normal_moments_and_determinism():
    x = rng.normal(1, (200000,))
    assert abs(float(x.mean())) < 0.01 and abs(float(x.std()) - 1.0) < 0.01
    assert abs(float((x ** 3).mean())) < 0.03           # symmetric
    assert abs(float((x ** 4).mean()) - 3.0) < 0.1      # gaussian kurtosis
    assert (rng.normal(1, (200000,)) == x).all()
    y = rng.normal(2, (1000,), std=0.1)
    assert abs(float(y.std()) - 0.1) < 0.01


def test_uniform_int_and_geometric():
    u = rng.uniform_int(3, (30000,), 1, 4)
    assert u.min() == 1 and u.max() == 4
    for v in range(1, 5):
        assert abs(float((u == v).mean()) - 0.25) < 0.01
    g = rng.geometric(4, (50000,), 0.5)
    assert g.min() == 1
    assert abs(float((g == 1).mean()) - 0.5) < 0.01 and abs(float((g == 2).mean()) - 0.25) < 0.01


def test_bf16_and_f16_encodings_match_torch():
    x = np.concatenate([rng.normal(9, (4096,)), np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38,
                                                          1e-30, -2.5, 65504.0], dtype=np.float32)])
    ours = workloads.to_storage(x, "bf16")
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert (ours == ref).all()
    back = workloads.from_storage(ours, "bf16")
    assert (back == torch.from_numpy(x).to(torch.bfloat16).double().numpy()).all()
    x = x[np.abs(x) < 6e4]
    h = workloads.to_storage(x, "f16")
    assert (h.view(np.uint16) == torch.from_numpy(x).to(torch.float16).view(torch.int16).numpy().view(np.uint16)).all()


def test_config_shapes():
    c1 = workloads.config1()
    assert c1["X"].shape == (1, 16, 32, 32) and c1["Wt"].shape == (32, 16, 3, 3)
    assert set(np.unique(c1["g"])) <= {1, 2, 3}
    v = workloads.vgg16_shape()
    assert sum(l.kind == "gdws" for l in v) == 13 and sum(l.kind == "maxpool" for l in v) == 5
    assert (v[-1].Ho, v[-1].Wo) == (1, 1)
    r = workloads.resnet18_shape()
    assert sum(l.kind == "gdws" for l in r) == 17 and sum(l.kind == "dense" for l in r) == 3
    assert (r[-1].Ho, r[-1].M) == (4, 512)
    r50 = workloads.resnet50_shape()
    assert sum(l.kind == "gdws" for l in r50) == 16
    assert (r50[-1].Ho, r50[-1].M) == (7, 2048)
    w = workloads.wrn28_4_shape()
    assert sum(l.kind == "gdws" for l in w) == 25 and sum(l.kind == "dense" for l in w) == 3
    assert (w[-1].Ho, w[-1].M) == (8, 256) and w[0].M == 16
    g = workloads.skewed_g(77, 64, 201)
    assert g.sum() == 201 and g.min() >= 1 and g.max() <= 9
