"""Pins for the oracle's backward pass (Eq. 5 with the Eq. 6 modification).

Checked against: central finite differences of the oracle's own forward (itself
pinned in test_oracle_forward.py), torch autograd through an independently
written slice -> mean/var -> normalise expression, torch's batch-norm backward
for the ratio-1 case, and the structure Eq. 6 prescribes outside S.
"""
import numpy as np
import pytest
import torch

from oracle import bns_oracle as o

EPS = 1e-5

CASES = [
    (o.FULL, {}),
    (o.NS, dict(n_s=2)),
    (o.BS, dict(n_s=2)),
    (o.FS, dict(patch_h=2, patch_w=3)),
    (o.FS, dict(patch_h=3, patch_w=2, fs_per_channel=1)),
    (o.VDN, dict(n_s=1)),
]


def _data(N, C, H, W, seed=0):
    rng = np.random.default_rng(seed)
    mu = rng.uniform(-1, 1, C)
    sg = rng.uniform(0.5, 2, C)
    x = mu[None, :, None, None] + sg[None, :, None, None] * rng.standard_normal((N, C, H, W))
    return x, rng.uniform(0.5, 1.5, C), rng.uniform(-0.5, 0.5, C), rng.standard_normal((N, C, H, W))


def _loss(x, gamma, beta, boxes, w):
    return float((o.forward(x, gamma, beta, boxes, EPS)["y"] * w).sum())


@pytest.mark.parametrize("mode,kw", CASES)
def test_finite_differences(mode, kw):
    N, C, H, W = 4, 2, 4, 5
    x, gamma, beta, w = _data(N, C, H, W, seed=2)
    boxes = o.sample_index(N, C, H, W, mode, seed=4, layer_id=1, epoch=3, **kw)
    f = o.forward(x, gamma, beta, boxes, EPS)
    b = o.backward(x, w, gamma, f["mean"], f["var"], boxes, EPS)      # dl/dy = w for l = sum(w * y)
    h = 1e-6
    num = np.zeros_like(x)
    it = np.nditer(x, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        xp, xm = x.copy(), x.copy()
        xp[i] += h
        xm[i] -= h
        num[i] = (_loss(xp, gamma, beta, boxes, w) - _loss(xm, gamma, beta, boxes, w)) / (2 * h)
    scale = np.abs(b["dx"]).max()
    assert np.abs(num - b["dx"]).max() < 1e-7 * max(scale, 1.0)
    for k in range(C):
        for name, vec in (("dgamma", gamma), ("dbeta", beta)):
            vp, vm = vec.copy(), vec.copy()
            vp[k] += h
            vm[k] -= h
            args_p = (vp, beta) if name == "dgamma" else (gamma, vp)
            args_m = (vm, beta) if name == "dgamma" else (gamma, vm)
            d = (_loss(x, *args_p, boxes, w) - _loss(x, *args_m, boxes, w)) / (2 * h)
            assert d == pytest.approx(b[name][k], rel=1e-7, abs=1e-7)


@pytest.mark.parametrize("mode,kw", CASES)
def test_against_torch_autograd_of_slice_mean_var_normalise(mode, kw):
    N, C, H, W = 6, 3, 5, 7
    x, gamma, beta, dy = _data(N, C, H, W, seed=7)
    boxes = o.sample_index(N, C, H, W, mode, seed=31, layer_id=3, epoch=1, **kw)
    f = o.forward(x, gamma, beta, boxes, EPS)
    b = o.backward(x, dy, gamma, f["mean"], f["var"], boxes, EPS)

    xt = torch.tensor(x, requires_grad=True)
    gt = torch.tensor(gamma, requires_grad=True)
    bt = torch.tensor(beta, requires_grad=True)
    ys = []
    for c in range(C):
        n0, nc, h0, hc, w0, wc = (int(v) for v in boxes[c])
        sub = xt[n0:n0 + nc, c, h0:h0 + hc, w0:w0 + wc]
        mean = sub.mean()
        var = sub.var(unbiased=False)
        ys.append(gt[c] * (xt[:, c] - mean) / torch.sqrt(var + EPS) + bt[c])
    y = torch.stack(ys, dim=1)
    np.testing.assert_allclose(f["y"], y.detach().numpy(), rtol=1e-11, atol=1e-12)
    y.backward(torch.tensor(dy))
    np.testing.assert_allclose(b["dx"], xt.grad.numpy(), rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(b["dgamma"], gt.grad.numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(b["dbeta"], bt.grad.numpy(), rtol=1e-11, atol=1e-12)


def test_ratio_one_is_torch_batch_norm_backward():
    N, C, H, W = 5, 4, 3, 6
    x, gamma, beta, dy = _data(N, C, H, W, seed=9)
    boxes = o.sample_index(N, C, H, W, o.FULL)
    f = o.forward(x, gamma, beta, boxes, EPS)
    b = o.backward(x, dy, gamma, f["mean"], f["var"], boxes, EPS)
    xt = torch.tensor(x, requires_grad=True)
    gt = torch.tensor(gamma, requires_grad=True)
    bt = torch.tensor(beta, requires_grad=True)
    y = torch.nn.functional.batch_norm(xt, None, None, gt, bt, training=True, eps=EPS)
    y.backward(torch.tensor(dy))
    np.testing.assert_allclose(b["dx"], xt.grad.numpy(), rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(b["dgamma"], gt.grad.numpy(), rtol=1e-11)
    np.testing.assert_allclose(b["dbeta"], bt.grad.numpy(), rtol=1e-11)
    # textbook identities of full BN: dx sums to zero, and is orthogonal to x^ up to the eps term
    # (sum x^2 = m Var / (Var + eps), so sum dx x^ = gamma r (sum g x^) eps / (Var + eps))
    for c in range(C):
        xhat = (x[:, c] - f["mean"][c]) * f["invstd"][c]
        assert abs(b["dx"][:, c].sum()) < 1e-10
        leak = gamma[c] * f["invstd"][c] * (dy[:, c] * xhat).sum() * EPS / (f["var"][c] + EPS)
        assert (b["dx"][:, c] * xhat).sum() == pytest.approx(leak, rel=1e-6, abs=1e-12)


@pytest.mark.parametrize("mode,kw", CASES[1:])
def test_outside_S_only_the_direct_term(mode, kw):
    """Eq. 6, second branch: dl/dx_i = dl/dx^_i / sqrt(Var + eps) exactly, and inside S it differs."""
    N, C, H, W = 6, 3, 6, 6
    x, gamma, beta, dy = _data(N, C, H, W, seed=12)
    boxes = o.sample_index(N, C, H, W, mode, seed=5, layer_id=9, epoch=4, **kw)
    f = o.forward(x, gamma, beta, boxes, EPS)
    b = o.backward(x, dy, gamma, f["mean"], f["var"], boxes, EPS)
    for c in range(C):
        S = o.subset_mask(N, H, W, boxes[c])
        direct = dy[:, c] * gamma[c] * f["invstd"][c]
        assert (b["dx"][:, c][~S] == direct[~S]).all()
        assert (b["dx"][:, c][S] != direct[S]).all()
        # the correction detects S: with gamma = 1, dy = 1 it is non-zero exactly on S
        ones = np.ones_like(dy)
        b1 = o.backward(x, ones, np.ones(C), f["mean"], f["var"], boxes, EPS)
        touched = b1["dx"][:, c] != f["invstd"][c]
        assert (touched == S).all()


def test_compact_form_agrees_with_three_partials():
    """dx = gamma r [ g - 1_S/s (sum g + x^ sum g x^) ], the form obtained by substituting
    dl/dE and dl/dVar of Eq. 5 into Eq. 6; evaluated here directly with numpy."""
    N, C, H, W = 8, 3, 5, 5
    x, gamma, beta, dy = _data(N, C, H, W, seed=15)
    boxes = o.sample_index(N, C, H, W, o.FS, patch_h=2, patch_w=2, seed=3)
    f = o.forward(x, gamma, beta, boxes, EPS)
    b = o.backward(x, dy, gamma, f["mean"], f["var"], boxes, EPS)
    for c in range(C):
        S = o.subset_mask(N, H, W, boxes[c]).astype(float)
        s = S.sum()
        r = f["invstd"][c]
        xhat = (x[:, c] - f["mean"][c]) * r
        g = dy[:, c]
        ref = gamma[c] * r * (g - S / s * (g.sum() + xhat * (g * xhat).sum()))
        np.testing.assert_allclose(b["dx"][:, c], ref, rtol=1e-10, atol=1e-12)
