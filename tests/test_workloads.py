"""The seeded input generators: shapes, determinism, distributions, bf16 rounding."""
import numpy as np
import torch

from paper_1810_10962_amd import workloads as wl


def test_table_of_workloads_matches_the_benchmark_shapes():
    W = wl.WORKLOADS
    assert W["tiny_bs"].shape == (8, 16, 8, 8) and W["tiny_bs"].n_s == 2
    assert W["cifar_fs"].shape == (128, 64, 32, 32) and (W["cifar_fs"].patch_h, W["cifar_fs"].patch_w) == (8, 8)
    assert W["imagenet_bs"].shape == (64, 256, 56, 56) and W["imagenet_bs"].n_s == 8
    assert (W["imagenet_fs"].patch_h, W["imagenet_fs"].patch_w) == (14, 14)
    assert W["vdn"].shape == (130, 128, 28, 28) and W["vdn"].n_s == 2
    assert W["micro_a_fs"].shape == (2, 512, 14, 14) and W["micro_b_fs"].shape == (1, 1024, 7, 7)
    assert W["imagenet_bs"].elements == 51380224
    assert W["imagenet_bs"].label() == "BS-8/64"


def test_inputs_are_seeded_and_distributed_as_stated():
    w = wl.WORKLOADS["tiny_bs"].replace(N=64, H=16, W=16)
    a, b = wl.make_inputs(w), wl.make_inputs(w)
    for k in a:
        assert a[k].dtype == np.float32 and (a[k] == b[k]).all()
    x = a["x"]
    mu = x.mean(axis=(0, 2, 3))
    sd = x.std(axis=(0, 2, 3))
    assert (-1.1 < mu).all() and (mu < 1.1).all() and (0.45 < sd).all() and (sd < 2.1).all()
    assert (0.5 <= a["gamma"]).all() and (a["gamma"] <= 1.5).all()
    assert (-0.5 <= a["beta"]).all() and (a["beta"] <= 0.5).all()
    assert abs(a["dy"].mean()) < 0.02 and abs(a["dy"].std() - 1) < 0.02
    assert (a["running_mean"] == 0).all() and (a["running_var"] == 1).all()
    sub = wl.make_inputs(w, channels=slice(3, 7))
    assert (sub["x"] == x[:, 3:7]).all() and (sub["gamma"] == a["gamma"][3:7]).all()
    other = wl.make_inputs(w.replace(data_seed=w.data_seed + 1))
    assert not (other["x"] == x).all()


def test_vdn_virtual_samples_sit_in_front_and_come_from_a_conv_of_uniform_inputs():
    w = wl.WORKLOADS["vdn"].replace(N=6, C=8, H=10, W=10)
    a = wl.make_inputs(w)
    assert a["x"].shape == (6, 8, 10, 10)
    # conv of non-negative inputs with zero-mean weights: per-channel means of the two virtual
    # samples are strongly correlated with each other, unlike the i.i.d. real samples
    v = a["x"][:2].mean(axis=(2, 3))
    assert np.corrcoef(v[0], v[1])[0, 1] > 0.9
    # the 3x3 "same" convolution against torch's
    rng = np.random.default_rng(0)
    vin = rng.uniform(0, 1, (2, 3, 7, 5))
    wgt = rng.standard_normal((4, 3, 3, 3))
    ref = torch.nn.functional.conv2d(torch.tensor(vin), torch.tensor(wgt), padding=1).numpy()
    np.testing.assert_allclose(wl._conv3x3_same(vin, wgt), ref, rtol=1e-12, atol=1e-12)


def test_bf16_rounding_matches_torch():
    rng = np.random.default_rng(0)
    a = (rng.standard_normal(100000) * 10 ** rng.uniform(-6, 6, 100000)).astype(np.float32)
    a[:4] = [0.0, -0.0, 1.00390625, 1.01171875]          # two exact ties: round to even
    r = wl.round_to_bf16(a)
    ref = torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    assert (r.view(np.uint32) == ref.view(np.uint32)).all()
    assert (wl.round_to_bf16(r) == r).all()
    w = wl.WORKLOADS["imagenet_bs_bf16"].replace(N=4, C=4, H=8, W=8)
    x = wl.make_inputs(w)["x"]
    assert (x.view(np.uint32) & 0xFFFF == 0).all()
