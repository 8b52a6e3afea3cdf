"""Pins for the oracle's forward pass (Eq. 1, Eq. 3, Eq. 8).

Checked against: numpy's mean/var on an explicitly sliced sub-tensor (the slices
printed in Alg. 1-3), torch's batch_norm for the ratio-1 case, the moments of
the normalised subset, a hand-worked example, and Eq. 9's closed form.
"""
import numpy as np
import pytest
import torch

from oracle import bns_oracle as o

EPS = 1e-5


def _data(N, C, H, W, seed=0):
    rng = np.random.default_rng(seed)
    mu = rng.uniform(-1, 1, C)
    sg = rng.uniform(0.5, 2, C)
    x = mu[None, :, None, None] + sg[None, :, None, None] * rng.standard_normal((N, C, H, W))
    gamma = rng.uniform(0.5, 1.5, C)
    beta = rng.uniform(-0.5, 0.5, C)
    return x, gamma, beta


CASES = [
    (o.FULL, {}),
    (o.NS, dict(n_s=3)),
    (o.BS, dict(n_s=2)),
    (o.FS, dict(patch_h=3, patch_w=2)),
    (o.FS, dict(patch_h=2, patch_w=5, fs_per_channel=1)),
    (o.VDN, dict(n_s=1)),
]


@pytest.mark.parametrize("mode,kw", CASES)
def test_statistics_equal_numpy_on_the_printed_slice(mode, kw):
    N, C, H, W = 7, 5, 6, 9
    x, gamma, beta = _data(N, C, H, W, seed=3)
    for epoch in range(6):
        boxes = o.sample_index(N, C, H, W, mode, seed=11, layer_id=2, epoch=epoch, **kw)
        out = o.forward(x, gamma, beta, boxes, EPS)
        for c in range(C):
            n0, nc, h0, hc, w0, wc = (int(v) for v in boxes[c])
            B_s = x[n0:n0 + nc, c, h0:h0 + hc, w0:w0 + wc]         # B_l[begin : begin+n_s-1, ...]
            assert B_s.size == o.subset_size(boxes[c])
            assert out["mean"][c] == pytest.approx(np.mean(B_s), rel=1e-13, abs=1e-14)
            assert out["var"][c] == pytest.approx(np.var(B_s, ddof=0), rel=1e-12)
            assert out["invstd"][c] == pytest.approx(1 / np.sqrt(np.var(B_s) + EPS), rel=1e-12)
            # Eq. 1 applied to every point of the feature map, sampled or not
            ref = gamma[c] * (x[:, c] - np.mean(B_s)) / np.sqrt(np.var(B_s) + EPS) + beta[c]
            np.testing.assert_allclose(out["y"][:, c], ref, rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("mode,kw", [(o.FULL, {}), (o.BS, dict(n_s=6)), (o.FS, dict(patch_h=5, patch_w=4))])
def test_ratio_one_is_plain_batch_norm(mode, kw):
    """s = m: Eq. 3 becomes Eq. 2; torch's training-mode batch_norm is the library routine."""
    N, C, H, W = 6, 4, 5, 4
    x, gamma, beta = _data(N, C, H, W, seed=5)
    boxes = o.sample_index(N, C, H, W, mode, seed=1, **kw)
    rm0 = np.linspace(-1, 1, C)
    rv0 = np.linspace(0.5, 2, C)
    out = o.forward(x, gamma, beta, boxes, EPS, momentum=0.1, running_mean=rm0, running_var=rv0)
    rm, rv = torch.tensor(rm0.copy()), torch.tensor(rv0.copy())
    y = torch.nn.functional.batch_norm(torch.tensor(x), rm, rv, torch.tensor(gamma), torch.tensor(beta),
                                       training=True, momentum=0.1, eps=EPS)
    np.testing.assert_allclose(out["y"], y.numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(out["running_mean"], rm.numpy(), rtol=1e-12, atol=1e-14)
    # torch keeps the *unbiased* variance in running_var; Eq. 8 averages Var of Eq. 3 (biased):
    m = N * H * W
    torch_biased = (rv.numpy() - 0.9 * rv0) * (m - 1) / m + 0.9 * rv0
    np.testing.assert_allclose(out["running_var"], torch_biased, rtol=1e-11)


@pytest.mark.parametrize("mode,kw", CASES)
def test_sampled_subset_is_normalised(mode, kw):
    """Over S: mean(x^) = 0 and mean(x^2) = Var / (Var + eps); gamma = 1, beta = 0 gives y = x^."""
    N, C, H, W = 9, 4, 8, 8
    x, _, _ = _data(N, C, H, W, seed=8)
    boxes = o.sample_index(N, C, H, W, mode, seed=21, layer_id=5, epoch=2, **kw)
    out = o.forward(x, np.ones(C), np.zeros(C), boxes, EPS)
    for c in range(C):
        S = o.subset_mask(N, H, W, boxes[c])
        ys = out["y"][:, c][S]
        assert abs(ys.mean()) < 1e-12
        assert (ys ** 2).mean() == pytest.approx(out["var"][c] / (out["var"][c] + EPS), rel=1e-12)
        if S.sum() < S.size:
            # the complement is not constrained: with a sampled estimate it is off by the estimation error
            assert abs(out["y"][:, c][~S].mean()) > 1e-6


def test_hand_worked_example():
    """One feature map, 2 samples of 1x2; Batch Sampling keeps sample 1 = {3, 5}.

    E = 4, Var = 1 (biased), eps = 0: x^ = (1-4, 2-4, 3-4, 5-4) = (-3, -2, -1, 1);
    gamma = 2, beta = 10 -> y = (4, 6, 8, 12).
    Moving average from (0, 1) with alpha = 0.25: mean 1.0, var 1.0; alpha = 1 -> (4, 1).
    """
    x = np.array([1.0, 2.0, 3.0, 5.0]).reshape(2, 1, 1, 2)
    box = np.array([[1, 1, 0, 1, 0, 2]])
    out = o.forward(x, [2.0], [10.0], box, 0.0, momentum=0.25, running_mean=[0.0], running_var=[1.0])
    assert out["mean"][0] == 4.0 and out["var"][0] == 1.0 and out["invstd"][0] == 1.0
    assert out["y"].ravel().tolist() == [4.0, 6.0, 8.0, 12.0]
    assert out["running_mean"][0] == 1.0 and out["running_var"][0] == 1.0
    first = o.forward(x, [2.0], [10.0], box, 0.0, momentum=1.0, running_mean=[7.0], running_var=[9.0])
    assert first["running_mean"][0] == 4.0 and first["running_var"][0] == 1.0      # Eq. 8, it = 1
    # single sampled point: Var = 0, inv-std = 1/sqrt(eps)
    one = o.forward(x, [1.0], [0.0], np.array([[0, 1, 0, 1, 1, 1]]), 0.25)
    assert one["mean"][0] == 2.0 and one["var"][0] == 0.0 and one["invstd"][0] == 2.0
    assert one["y"].ravel().tolist() == [-2.0, 0.0, 2.0, 6.0]


def test_moving_average_variance_closed_form():
    """Eq. 9: for i.i.d. estimates the moving average has variance alpha/(2-alpha) of one estimate."""
    rng = np.random.default_rng(0)
    alpha = 0.3
    chains, steps = 4000, 80
    x = np.zeros((1, chains, 1, 1))
    rm = np.zeros(chains)
    rv = np.ones(chains)
    box = np.tile(np.array([[0, 1, 0, 1, 0, 1]]), (chains, 1))
    for _ in range(steps):
        x[0, :, 0, 0] = rng.standard_normal(chains)        # one point per "feature": E = that point
        out = o.forward(x, np.ones(chains), np.zeros(chains), box, 1.0, momentum=alpha,
                        running_mean=rm, running_var=rv)
        rm, rv = out["running_mean"], out["running_var"]
    ratio = rm.var() / 1.0
    assert ratio == pytest.approx(alpha / (2 - alpha), rel=0.1)
    np.testing.assert_allclose(rv, (1 - alpha) ** steps, rtol=1e-9)      # Var of one point is 0 each step


def test_inference_is_torch_eval_batch_norm_and_continues_training_statistics():
    N, C, H, W = 5, 4, 6, 3
    x, gamma, beta = _data(N, C, H, W, seed=21)
    rng = np.random.default_rng(1)
    rm, rv = rng.standard_normal(C), rng.uniform(0.3, 2.0, C)
    y = o.inference(x, gamma, beta, rm, rv, EPS)
    ref = torch.nn.functional.batch_norm(torch.tensor(x), torch.tensor(rm), torch.tensor(rv), torch.tensor(gamma),
                                         torch.tensor(beta), training=False, eps=EPS)
    np.testing.assert_allclose(y, ref.numpy(), rtol=1e-12, atol=1e-13)
    # Eq. 8 at it = 1 copies the statistics, so inference on the same batch reproduces the training output
    boxes = o.sample_index(N, C, H, W, o.BS, n_s=2, seed=4)
    f = o.forward(x, gamma, beta, boxes, EPS, momentum=1.0, running_mean=rm, running_var=rv)
    np.testing.assert_allclose(o.inference(x, gamma, beta, f["running_mean"], f["running_var"], EPS), f["y"],
                               rtol=1e-12, atol=1e-13)


def test_moving_average_weight_gives_the_unrolled_form_of_eq8():
    """Eq. 8 unrolled by hand: X_ma(n) = (1-a)^(n-1) X_1 + a * sum_{j=2..n} (1-a)^(n-j) X_j, whatever the
    moving average held before the first iteration."""
    rng = np.random.default_rng(8)
    for alpha in (0.1, 0.3, 0.7, 1.0):
        xs = rng.standard_normal(9)
        ma = 123.456                                  # must be forgotten at it = 1
        for it, x_it in enumerate(xs, start=1):
            a = o.moving_average_weight(it, alpha)
            ma = a * x_it + (1.0 - a) * ma            # the update the forward pass applies
            n = it
            want = (1 - alpha) ** (n - 1) * xs[0] + alpha * sum((1 - alpha) ** (n - j) * xs[j - 1] for j in range(2, n + 1))
            assert abs(ma - want) < 1e-12, (alpha, it)
    assert o.moving_average_weight(1, 0.1) == 1.0 and o.moving_average_weight(2, 0.1) == 0.1
