"""Pins for the oracle's "VDN + sampling" statistics (Eq. 4) and the backward derived for them.

The paper prints no backward for Eq. 4, so the derivation is pinned by torch autograd through an
independently written expression and by finite differences; the forward by numpy on explicit
slices and by the two limits mix_beta = 1 (pure VDN) and mix_beta = 0 (pure sampling)."""
import numpy as np
import pytest
import torch

from oracle import bns_oracle as o

EPS = 1e-5
CASES = [
    (o.BS, dict(n_s=2)),
    (o.NS, dict(n_s=3)),
    (o.FS, dict(patch_h=2, patch_w=3)),
    (o.FS, dict(patch_h=3, patch_w=2, fs_per_channel=1)),
    (o.FULL, {}),
]


def _data(N, C, H, W, seed=0):
    rng = np.random.default_rng(seed)
    x = rng.uniform(-1, 1, C)[None, :, None, None] + rng.uniform(0.5, 2, C)[None, :, None, None] * \
        rng.standard_normal((N, C, H, W))
    return x, rng.uniform(0.5, 1.5, C), rng.uniform(-0.5, 0.5, C), rng.standard_normal((N, C, H, W))


@pytest.mark.parametrize("mode,kw", CASES)
def test_mixed_index_virtual_first_real_sampled_like_alg_1_2(mode, kw):
    N, C, H, W, n_v = 9, 3, 5, 6, 2
    for epoch in range(20):
        bv, bs = o.sample_index_mixed(N, C, H, W, mode, n_v, seed=5, layer_id=1, epoch=epoch, **kw)
        assert (bv == np.array([0, n_v, 0, H, 0, W])).all()                    # Alg. 3: samples 0 .. n_v-1
        ref = o.sample_index(N - n_v, C, H, W, mode, seed=5, layer_id=1, epoch=epoch, **kw)
        assert (bs[:, 1:] == ref[:, 1:]).all() and (bs[:, 0] == ref[:, 0] + n_v).all()
        assert (bs[:, 0] >= n_v).all() and (bs[:, 0] + bs[:, 1] <= N).all()    # never touches virtual samples


@pytest.mark.parametrize("mode,kw", CASES)
@pytest.mark.parametrize("mix", [0.5, 0.2, 1.0, 0.0])
def test_mixed_forward_against_numpy_slices_and_limits(mode, kw, mix):
    N, C, H, W, n_v = 8, 4, 5, 6, 2
    x, gamma, beta, _ = _data(N, C, H, W, seed=1)
    bv, bs = o.sample_index_mixed(N, C, H, W, mode, n_v, seed=8, layer_id=2, epoch=1, **kw)
    f = o.forward_mixed(x, gamma, beta, bv, bs, mix, EPS, 0.1, np.zeros(C), np.ones(C))
    for c in range(C):
        n0, nc, h0, hc, w0, wc = (int(v) for v in bs[c])
        xs = x[n0:n0 + nc, c, h0:h0 + hc, w0:w0 + wc]
        xv = x[:n_v, c]
        E = mix * xv.mean() + (1 - mix) * xs.mean()
        V = mix * xv.var() + (1 - mix) * xs.var()
        assert f["mean"][c] == pytest.approx(E, rel=1e-12, abs=1e-14)
        assert f["var"][c] == pytest.approx(V, rel=1e-12)
        assert f["mean_v"][c] == pytest.approx(xv.mean(), rel=1e-12, abs=1e-14)
        assert f["mean_s"][c] == pytest.approx(xs.mean(), rel=1e-12, abs=1e-14)
        np.testing.assert_allclose(f["y"][:, c], gamma[c] * (x[:, c] - E) / np.sqrt(V + EPS) + beta[c], rtol=1e-12,
                                   atol=1e-13)
        assert f["running_mean"][c] == pytest.approx(0.1 * E, rel=1e-12, abs=1e-14)
        assert f["running_var"][c] == pytest.approx(0.1 * V + 0.9, rel=1e-12)
    if mix == 1.0:      # statistics from the virtual samples only: Alg. 3
        pure = o.forward(x, gamma, beta, o.sample_index(N, C, H, W, o.VDN, n_s=n_v), EPS)
        np.testing.assert_allclose(f["y"], pure["y"], rtol=1e-12, atol=1e-13)
    if mix == 0.0:      # statistics from the sampled real data only: Alg. 1 / 2 with these boxes
        pure = o.forward(x, gamma, beta, bs, EPS)
        np.testing.assert_allclose(f["y"], pure["y"], rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("mode,kw", CASES)
@pytest.mark.parametrize("mix", [0.5, 0.3, 1.0, 0.0])
def test_mixed_backward_against_autograd(mode, kw, mix):
    N, C, H, W, n_v = 7, 3, 4, 5, 2
    x, gamma, beta, dy = _data(N, C, H, W, seed=3)
    bv, bs = o.sample_index_mixed(N, C, H, W, mode, n_v, seed=2, layer_id=4, epoch=3, **kw)
    f = o.forward_mixed(x, gamma, beta, bv, bs, mix, EPS)
    b = o.backward_mixed(x, dy, gamma, f["mean"], f["var"], f["mean_v"], f["mean_s"], bv, bs, mix, EPS)
    xt = torch.tensor(x, requires_grad=True)
    gt = torch.tensor(gamma, requires_grad=True)
    bt = torch.tensor(beta, requires_grad=True)
    ys = []
    for c in range(C):
        n0, nc, h0, hc, w0, wc = (int(v) for v in bs[c])
        s_ = xt[n0:n0 + nc, c, h0:h0 + hc, w0:w0 + wc]
        v_ = xt[:n_v, c]
        E = mix * v_.mean() + (1 - mix) * s_.mean()
        V = mix * v_.var(unbiased=False) + (1 - mix) * s_.var(unbiased=False)
        ys.append(gt[c] * (xt[:, c] - E) / torch.sqrt(V + EPS) + bt[c])
    y = torch.stack(ys, dim=1)
    np.testing.assert_allclose(f["y"], y.detach().numpy(), rtol=1e-11, atol=1e-12)
    y.backward(torch.tensor(dy))
    np.testing.assert_allclose(b["dx"], xt.grad.numpy(), rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(b["dgamma"], gt.grad.numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(b["dbeta"], bt.grad.numpy(), rtol=1e-11, atol=1e-12)
    if mix == 0.0:      # reduces to Eq. 6 with S = the sampled real set
        pure = o.backward(x, dy, gamma, f["mean"], f["var"], bs, EPS)
        np.testing.assert_allclose(b["dx"], pure["dx"], rtol=1e-12, atol=1e-13)


def test_mixed_backward_finite_differences():
    N, C, H, W, n_v, mix = 5, 2, 3, 4, 1, 0.5
    x, gamma, beta, w = _data(N, C, H, W, seed=6)
    bv, bs = o.sample_index_mixed(N, C, H, W, o.FS, n_v, patch_h=2, patch_w=2, seed=1)
    f = o.forward_mixed(x, gamma, beta, bv, bs, mix, EPS)
    b = o.backward_mixed(x, w, gamma, f["mean"], f["var"], f["mean_v"], f["mean_s"], bv, bs, mix, EPS)
    loss = lambda xx: float((o.forward_mixed(xx, gamma, beta, bv, bs, mix, EPS)["y"] * w).sum())
    h = 1e-6
    num = np.zeros_like(x)
    it = np.nditer(x, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        xp, xm = x.copy(), x.copy()
        xp[i] += h
        xm[i] -= h
        num[i] = (loss(xp) - loss(xm)) / (2 * h)
    assert np.abs(num - b["dx"]).max() < 1e-7 * max(np.abs(b["dx"]).max(), 1.0)
    # outside both sets only the direct term (second branch of Eq. 6)
    for c in range(C):
        outside = ~(o.subset_mask(N, H, W, bv[c]) | o.subset_mask(N, H, W, bs[c]))
        assert (b["dx"][:, c][outside] == (w[:, c] * gamma[c] * f["invstd"][c])[outside]).all()
