"""Planted mistakes: each plausible slip in the oracle must fail a pin.

The oracle's source is copied, one expression is altered, and a compact battery
of the pins (library routines on explicit slices, torch autograd, brute-force
membership, end-point reachability, the hand-worked moving average) is run on
the altered copy.  The unaltered copy must pass; every mutant must fail.
Everything here runs on the CPU.
"""
import itertools
import os
import types

import numpy as np
import pytest
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = open(os.path.join(ROOT, "oracle", "bns_oracle.py")).read()
EPS = 1e-3


def _load(src):
    mod = types.ModuleType("oracle_mutant")
    exec(compile(src, "oracle_mutant", "exec"), mod.__dict__)
    return mod


def _battery(o):
    """Raises AssertionError when any pin fails."""
    rng = np.random.default_rng(1)
    N, C, H, W = 5, 2, 4, 6
    x = rng.uniform(-1, 1, C)[None, :, None, None] + rng.uniform(0.5, 2, C)[None, :, None, None] * \
        rng.standard_normal((N, C, H, W))
    gamma, beta = rng.uniform(0.5, 1.5, C), rng.uniform(-0.5, 0.5, C)
    dy = rng.standard_normal((N, C, H, W))
    # end points of randint
    seen = {o.randint(0, 3, s, 0, 0, 1, 0) for s in range(400)}
    assert seen == {0, 1, 2, 3}
    # Batch Sampling: every legal start occurs; Feature Sampling: rows and columns both move
    starts = {int(o.sample_index(N, C, H, W, o.BS, n_s=2, seed=5, epoch=e)[0, 0]) for e in range(200)}
    assert starts == set(range(N - 2 + 1))
    fs = [o.sample_index(N, C, H, W, o.FS, patch_h=2, patch_w=3, seed=5, epoch=e)[0] for e in range(200)]
    assert {int(b[2]) for b in fs} == set(range(H - 2 + 1)) and {int(b[4]) for b in fs} == set(range(W - 3 + 1))
    for mode, kw in [(o.BS, dict(n_s=2)), (o.FS, dict(patch_h=2, patch_w=3)), (o.VDN, dict(n_s=1)),
                     (o.NS, dict(n_s=2)), (o.FULL, {})]:
        for epoch in range(4):
            boxes = o.sample_index(N, C, H, W, mode, seed=3, layer_id=1, epoch=epoch, **kw)
            f = o.forward(x, gamma, beta, boxes, EPS, momentum=0.25,
                          running_mean=np.full(C, 2.0), running_var=np.full(C, 3.0))
            b = o.backward(x, dy, gamma, f["mean"], f["var"], boxes, EPS)
            xt = torch.tensor(x, requires_grad=True)
            gt = torch.tensor(gamma, requires_grad=True)
            bt = torch.tensor(beta, requires_grad=True)
            ys = []
            for c in range(C):
                n0, nc, h0, hc, w0, wc = (int(v) for v in boxes[c])
                assert 0 <= n0 and n0 + nc <= N and 0 <= h0 and h0 + hc <= H and 0 <= w0 and w0 + wc <= W
                if mode in (o.NS, o.VDN):
                    assert n0 == 0
                members = set(itertools.product(range(n0, n0 + nc), range(h0, h0 + hc), range(w0, w0 + wc)))
                mask = o.subset_mask(N, H, W, boxes[c])
                for n, h, w in itertools.product(range(N), range(H), range(W)):
                    assert o.in_subset(boxes[c], n, h, w) == ((n, h, w) in members) == bool(mask[n, h, w])
                assert o.subset_size(boxes[c]) == len(members)
                sub = x[n0:n0 + nc, c, h0:h0 + hc, w0:w0 + wc]
                np.testing.assert_allclose(f["mean"][c], sub.mean(), rtol=1e-12)
                np.testing.assert_allclose(f["var"][c], sub.var(), rtol=1e-12)
                np.testing.assert_allclose(f["invstd"][c], 1 / np.sqrt(sub.var() + EPS), rtol=1e-12)
                np.testing.assert_allclose(f["running_mean"][c], 0.25 * sub.mean() + 0.75 * 2.0, rtol=1e-12)
                np.testing.assert_allclose(f["running_var"][c], 0.25 * sub.var() + 0.75 * 3.0, rtol=1e-12)
                st = xt[n0:n0 + nc, c, h0:h0 + hc, w0:w0 + wc]
                ys.append(gt[c] * (xt[:, c] - st.mean()) / torch.sqrt(st.var(unbiased=False) + EPS) + bt[c])
            y = torch.stack(ys, dim=1)
            np.testing.assert_allclose(f["y"], y.detach().numpy(), rtol=1e-11, atol=1e-12)
            y.backward(torch.tensor(dy))
            np.testing.assert_allclose(b["dx"], xt.grad.numpy(), rtol=1e-9, atol=1e-11)
            np.testing.assert_allclose(b["dgamma"], gt.grad.numpy(), rtol=1e-10)
            np.testing.assert_allclose(b["dbeta"], bt.grad.numpy(), rtol=1e-10)
    # inference from the moving averages (Appendix D) against torch's eval-mode batch norm
    rm, rv = rng.standard_normal(C), rng.uniform(0.3, 2.0, C)
    ref = torch.nn.functional.batch_norm(torch.tensor(x), torch.tensor(rm), torch.tensor(rv), torch.tensor(gamma),
                                         torch.tensor(beta), training=False, eps=EPS)
    np.testing.assert_allclose(o.inference(x, gamma, beta, rm, rv, EPS), ref.numpy(), rtol=1e-12, atol=1e-13)
    # Eq. 8 unrolled by hand: X_ma(n) = (1-a)^(n-1) X_1 + a sum_{j=2..n} (1-a)^(n-j) X_j
    xs, alpha, ma = rng.standard_normal(5), 0.3, 99.0
    for it, x_it in enumerate(xs, start=1):
        a = o.moving_average_weight(it, alpha)
        ma = a * x_it + (1.0 - a) * ma
    want = (1 - alpha) ** 4 * xs[0] + alpha * sum((1 - alpha) ** (5 - j) * xs[j - 1] for j in range(2, 6))
    assert abs(ma - want) < 1e-12
    # VDN + sampling (Eq. 4) against autograd through explicit slices
    n_v = 2
    for mode, kw, mix in [(o.BS, dict(n_s=2), 0.5), (o.FS, dict(patch_h=2, patch_w=3), 0.3), (o.FULL, {}, 0.7)]:
        bv, bs = o.sample_index_mixed(N, C, H, W, mode, n_v, seed=3, layer_id=1, epoch=2, **kw)
        assert (bs[:, 0] >= n_v).all() and (bs[:, 0] + bs[:, 1] <= N).all() and (bv[:, :2] == [0, n_v]).all()
        f = o.forward_mixed(x, gamma, beta, bv, bs, mix, EPS, 0.25, np.full(C, 2.0), np.full(C, 3.0))
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
            np.testing.assert_allclose(f["running_mean"][c], 0.25 * float(E.detach()) + 0.75 * 2.0, rtol=1e-12)
            np.testing.assert_allclose(f["running_var"][c], 0.25 * float(V.detach()) + 0.75 * 3.0, rtol=1e-12)
        y = torch.stack(ys, dim=1)
        np.testing.assert_allclose(f["y"], y.detach().numpy(), rtol=1e-11, atol=1e-12)
        y.backward(torch.tensor(dy))
        np.testing.assert_allclose(b["dx"], xt.grad.numpy(), rtol=1e-9, atol=1e-11)
        np.testing.assert_allclose(b["dgamma"], gt.grad.numpy(), rtol=1e-10)
        np.testing.assert_allclose(b["dbeta"], bt.grad.numpy(), rtol=1e-10)


MUTANTS = [
    ("unbiased variance", "Var[k] = ((x_s - E[k]) ** 2).sum() / s", "Var[k] = ((x_s - E[k]) ** 2).sum() / (s - 1)"),
    ("mean over all points", "E[k] = x_s.sum() / s", "E[k] = xk.sum() / xk.size"),
    ("eps outside the root", "x_hat = (xk - E[k]) / math.sqrt(Var[k] + eps)", "x_hat = (xk - E[k]) / (math.sqrt(Var[k]) + eps)"),
    ("alpha on the old value", "a * E + (1.0 - a) * np.asarray(running_mean", "(1.0 - a) * E + a * np.asarray(running_mean"),
    ("alpha on the old variance", "a * Var + (1.0 - a) * np.asarray(running_var", "(1.0 - a) * Var + a * np.asarray(running_var"),
    ("sign of dl/dE", "dl_dE = (dl_dxhat * (-r)).sum()", "dl_dE = (dl_dxhat * (r)).sum()"),
    ("exponent of dl/dVar", "(V + eps) ** (-1.5)", "(V + eps) ** (-0.5)"),
    ("factor 2 of dVar/dx", "(2.0 * (xk[S] - E) / s)", "(1.0 * (xk[S] - E) / s)"),
    ("1/m instead of 1/s", "dl_dE * (1.0 / s) +", "dl_dE * (1.0 / xk.size) +"),
    ("correction everywhere", "d[S] += dl_dE * (1.0 / s) + dl_dVar * (2.0 * (xk[S] - E) / s)",
     "d += dl_dE * (1.0 / s) + dl_dVar * (2.0 * (xk - E) / s)"),
    ("reductions over S only", "dl_dE = (dl_dxhat * (-r)).sum()", "dl_dE = (dl_dxhat[S] * (-r)).sum()"),
    ("dgamma from x not x^", "dgamma[k] = (g * x_hat).sum()", "dgamma[k] = (g * xk).sum()"),
    ("dbeta over S only", "dbeta[k] = g.sum()", "dbeta[k] = g[S].sum()"),
    ("gamma dropped from dl/dx^", "dl_dxhat = g * float(gamma[k])", "dl_dxhat = g"),
    ("exclusive randint", "outcomes = hi - lo + 1", "outcomes = max(hi - lo, 1)"),
    ("mask one sample too long", "(n <= n0 + nc - 1)", "(n <= n0 + nc)"),
    ("mask rows/cols swapped", "(h >= h0) & (h <= h0 + hc - 1)", "(h >= w0) & (h <= w0 + hc - 1)"),
    ("scalar test off by one", "(w0 <= w <= w0 + wc - 1)", "(w0 < w <= w0 + wc - 1)"),
    ("BS start not random", "n0 = randint(0, N - n_s, seed, layer_id, epoch, _TAG_N, _SHARED)", "n0 = N - n_s"),
    ("FS width drawn from height", "w0 = randint(0, W - patch_w,", "w0 = randint(0, H - patch_h,"),
    ("VDN takes the last samples", "elif mode in (NS, VDN):\n            nc = n_s", "elif mode in (NS, VDN):\n            nc = n_s\n            n0 = N - n_s"),
    ("inference: eps outside the root", "/ math.sqrt(float(moving_var[k]) + eps)", "/ (math.sqrt(float(moving_var[k])) + eps)"),
    ("Eq. 8: first iteration averaged like the others", "return 1.0 if iteration <= 1 else float(alpha)", "return float(alpha)"),
    ("Eq. 8: second iteration still a copy", "return 1.0 if iteration <= 1 else float(alpha)", "return 1.0 if iteration <= 2 else float(alpha)"),
    ("mixed: real samples not shifted", "boxes_s[:, 0] += n_v", "boxes_s[:, 0] += 0"),
    ("mixed: sampling sees the virtual samples", "real = sample_index(N - n_v, C, H, W, mode,", "real = sample_index(N, C, H, W, mode,"),
    ("mixed: weights swapped", "E[k] = mix_beta * E_v[k] + (1.0 - mix_beta) * E_s[k]", "E[k] = (1.0 - mix_beta) * E_v[k] + mix_beta * E_s[k]"),
    ("mixed: variance about the blended mean", "Var_s = ((x_s - E_s[k]) ** 2).sum() / x_s.size", "Var_s = ((x_s - (mix_beta * E_v[k] + (1.0 - mix_beta) * E_s[k])) ** 2).sum() / x_s.size"),
    ("mixed: variance not blended", "Var[k] = mix_beta * Var_v + (1.0 - mix_beta) * Var_s", "Var[k] = Var_s"),
    ("mixed backward: centre on the blended mean", "(xk[S] - centre) / s)", "(xk[S] - E) / s)"),
    ("mixed backward: weight dropped", "d[S] += dl_dE * (weight / s) + dl_dVar * (weight * 2.0", "d[S] += dl_dE * (1.0 / s) + dl_dVar * (weight * 2.0"),
    ("mixed backward: virtual set ignored", "for box, weight, centre in ((boxes_v[k], mix_beta, float(mean_v[k])),\n                                    (boxes_s[k], 1.0 - mix_beta, float(mean_s[k]))):", "for box, weight, centre in ((boxes_s[k], 1.0 - mix_beta, float(mean_s[k])),):"),
]


def test_unaltered_oracle_passes_the_battery():
    _battery(_load(SRC))


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_mutant_is_caught(name, old, new):
    assert SRC.count(old) >= 1, f"mutation site for '{name}' not found"
    mutant = _load(SRC.replace(old, new, 1))          # the first occurrence: the function the name refers to
    with pytest.raises(AssertionError):
        _battery(mutant)
