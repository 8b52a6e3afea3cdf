"""CPU oracle for Batch Normalization Sampling (Chen, Deng, Li et al., arXiv 1810.10962).

THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, fp64 restatement of what the
paper defines, used only to check the HIP library and as a timed CPU baseline.
Nothing in the product path may import it, and it imports nothing from the
product: it shares no code, table or constant generator with the HIP sources.

What it follows, in the paper's notation:

* Eq. 1   normalisation  x^ = (x - E) / sqrt(Var + eps),  y = gamma * x^ + beta
* Eq. 2   full-batch statistics (biased variance, 1/m)
* Eq. 3   statistics from the s sampled points only (biased variance, 1/s)
* Alg. 1  Naive / Batch Sampling: samples begin .. begin + n_s - 1
* Alg. 2  Feature Sampling: one h_s x w_s patch at (begin_h, begin_w), all samples
* Alg. 3  Virtual Dataset Normalisation: statistics from samples 0 .. n_v - 1
* Eq. 5   BN backward, three partial derivatives
* Eq. 6   sampled backward: the 1/s mean and variance terms only on x_i in S
* Eq. 4   VDN combined with a sampling strategy: blended E and Var (backward derived, see there)
* Eq. 8   moving average, alpha weights the new value; App. D: validation uses it in Eq. 1

The paper stores activations as N x H x W x C; here tensors are N x C x H x W
(the reduction is over the same three axes: samples, height, width).

The paper does not say which random generator draws ``randint``.  The reading
taken here (and, independently, by the HIP library): a counter-based integer
hash of (seed, layer, epoch, purpose, channel), see ``index_hash``.

Every function below is pinned by tests/test_oracle_*.py against something
other than itself (library routines on explicit slices, torch autograd, finite
differences, brute-force enumeration, values the paper prints).  No function is
"parity unpinned".
"""
from __future__ import annotations

import math

import numpy as np

# Sampling modes (same numbering as the C header; restated, not imported).
FULL, NS, BS, FS, VDN = 0, 1, 2, 3, 4

_MASK64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15          # 2^64 / golden ratio, odd
_TAG_N, _TAG_H, _TAG_W = 1, 2, 3      # which integer is being drawn
_SHARED = 0xFFFFFFFF                   # "channel" slot when one index serves the layer


# --------------------------------------------------------------------------
# Index generation: Alg. 1 / Alg. 2 "randint", made concrete
# --------------------------------------------------------------------------
def mix64(z: int) -> int:
    """64-bit finaliser of the SplitMix64 generator (Steele, Lea, Flood 2014)."""
    z &= _MASK64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK64
    return z ^ (z >> 31)


def index_hash(seed: int, layer_id: int, epoch: int, tag: int, channel: int) -> int:
    """64 random bits that depend on nothing but the five integers.

    Indices are refreshed once per epoch and differ between layers
    (Section 4.1, sampling rules), so both enter the hash.
    """
    h = mix64((seed + _GOLDEN) & _MASK64)
    h = mix64(h ^ (((layer_id & 0xFFFFFFFF) << 32) | (epoch & 0xFFFFFFFF)))
    h = mix64(h ^ (((tag & 0xFFFFFFFF) << 32) | (channel & 0xFFFFFFFF)))
    return h


def randint(lo: int, hi: int, seed: int, layer_id: int, epoch: int, tag: int, channel: int) -> int:
    """``randint(lo, hi)`` of Alg. 1 and Alg. 2 with *both* ends included.

    The slices in the algorithms end at ``begin + n_s - 1`` inclusive, so
    ``begin = N - n_s`` is the last legal start and must be reachable.
    Integer only: the top 32 hash bits are scaled to hi - lo + 1 outcomes.
    """
    outcomes = hi - lo + 1
    assert outcomes >= 1
    top = index_hash(seed, layer_id, epoch, tag, channel) >> 32
    return lo + ((top * outcomes) >> 32)


def sample_index(N: int, C: int, H: int, W: int, mode: int, *, n_s: int = 0,
                 patch_h: int = 0, patch_w: int = 0, fs_per_channel: int = 0,
                 seed: int = 0, layer_id: int = 0, epoch: int = 0) -> np.ndarray:
    """Per-channel sampling box, int64 array [C, 6] = (n0, n_cnt, h0, h_cnt, w0, w_cnt).

    FULL : everything (Eq. 2).
    NS   : samples 0 .. n_s-1 (Alg. 1, begin = 0).
    BS   : samples begin .. begin+n_s-1, begin = randint(0, N - n_s), one draw per
           layer and epoch, shared by all channels (Alg. 1; Section 4.1 rule 2).
    FS   : rows begin_h .. begin_h+h_s-1, columns begin_w .. begin_w+w_s-1 of every
           sample (Alg. 2); one location per layer (Section 4.1 rule 3) or, with
           ``fs_per_channel``, an independent location per feature map.
    VDN  : the n_v = n_s virtual samples at the front of the batch (Alg. 3).
    """
    box = np.zeros((C, 6), dtype=np.int64)
    for c in range(C):
        n0, nc, h0, hc, w0, wc = 0, N, 0, H, 0, W
        if mode == FULL:
            pass
        elif mode in (NS, VDN):
            nc = n_s
        elif mode == BS:
            nc = n_s
            n0 = randint(0, N - n_s, seed, layer_id, epoch, _TAG_N, _SHARED)
        elif mode == FS:
            ch = c if fs_per_channel else _SHARED
            hc, wc = patch_h, patch_w
            h0 = randint(0, H - patch_h, seed, layer_id, epoch, _TAG_H, ch)
            w0 = randint(0, W - patch_w, seed, layer_id, epoch, _TAG_W, ch)
        else:
            raise ValueError("unknown mode")
        box[c] = (n0, nc, h0, hc, w0, wc)
    return box


def in_subset(box, n: int, h: int, w: int) -> bool:
    """Membership of activation (n, h, w) of a feature map in its location set S."""
    n0, nc, h0, hc, w0, wc = (int(v) for v in box)
    return (n0 <= n <= n0 + nc - 1) and (h0 <= h <= h0 + hc - 1) and (w0 <= w <= w0 + wc - 1)


def subset_mask(N: int, H: int, W: int, box) -> np.ndarray:
    """Boolean [N, H, W] array, True exactly on S (vectorised ``in_subset``)."""
    n0, nc, h0, hc, w0, wc = (int(v) for v in box)
    n = np.arange(N)[:, None, None]
    h = np.arange(H)[None, :, None]
    w = np.arange(W)[None, None, :]
    return ((n >= n0) & (n <= n0 + nc - 1) & (h >= h0) & (h <= h0 + hc - 1)
            & (w >= w0) & (w <= w0 + wc - 1))


def subset_size(box) -> int:
    """s, the number of sampled points per feature map."""
    return int(box[1]) * int(box[3]) * int(box[5])


def sampling_ratio(N: int, H: int, W: int, box) -> float:
    """s / m (Section 3.2)."""
    return subset_size(box) / float(N * H * W)


# --------------------------------------------------------------------------
# Forward: Eq. 3 statistics, Eq. 1 normalisation, Eq. 8 moving average
# --------------------------------------------------------------------------
def forward(x, gamma, beta, boxes, eps: float, momentum: float = 0.1,
            running_mean=None, running_var=None):
    """Sampled BN forward over an [N, C, H, W] tensor.

    Returns dict(y, mean, var, invstd, running_mean, running_var), all fp64.
    ``momentum`` is alpha of Eq. 8 (weight of the new value).  Eq. 8's first
    iteration (moving average := current value) is alpha = 1.
    """
    x = np.asarray(x)
    N, C, H, W = x.shape
    y = np.empty((N, C, H, W), dtype=np.float64)
    E = np.empty(C)
    Var = np.empty(C)
    for k in range(C):
        xk = x[:, k].astype(np.float64)                      # x^(k): all m points
        x_s = xk[subset_mask(N, H, W, boxes[k])]             # the s sampled points
        s = x_s.size
        E[k] = x_s.sum() / s                                 # Eq. 3
        Var[k] = ((x_s - E[k]) ** 2).sum() / s               # Eq. 3, biased
        x_hat = (xk - E[k]) / math.sqrt(Var[k] + eps)        # Eq. 1, every point
        y[:, k] = float(gamma[k]) * x_hat + float(beta[k])
    out = dict(y=y, mean=E, var=Var, invstd=1.0 / np.sqrt(Var + eps))
    if running_mean is not None:
        a = float(momentum)
        out["running_mean"] = a * E + (1.0 - a) * np.asarray(running_mean, dtype=np.float64)    # Eq. 8
        out["running_var"] = a * Var + (1.0 - a) * np.asarray(running_var, dtype=np.float64)
    return out


def moving_average_weight(iteration: int, alpha: float) -> float:
    """Eq. 8, weight of the current statistics at iteration it (counted from 1): the moving average
    is the statistics themselves at it = 1 and alpha * X + (1 - alpha) * X_ma afterwards."""
    return 1.0 if iteration <= 1 else float(alpha)


def inference(x, gamma, beta, moving_mean, moving_var, eps: float):
    """Validation-time normalisation (Appendix D): E and Var of Eq. 1 are replaced by the
    recorded moving averages of Eq. 8."""
    x = np.asarray(x)
    N, C, H, W = x.shape
    y = np.empty((N, C, H, W), dtype=np.float64)
    for k in range(C):
        x_hat = (x[:, k].astype(np.float64) - float(moving_mean[k])) / math.sqrt(float(moving_var[k]) + eps)
        y[:, k] = float(gamma[k]) * x_hat + float(beta[k])
    return y


# --------------------------------------------------------------------------
# Backward: Eq. 5 with the Eq. 6 modification
# --------------------------------------------------------------------------
def backward(x, dy, gamma, mean, var, boxes, eps: float):
    """Sampled BN backward.  ``mean`` / ``var`` are E and Var saved by ``forward``.

    Follows Eq. 5 term by term (dl/dx^, dl/dE, dl/dVar), then the two branches
    of Eq. 6.  The sums in Eq. 5 run over all m points of the feature map,
    sampled or not; only the 1/s terms are restricted to S.
    Returns dict(dx, dgamma, dbeta), fp64.
    """
    x = np.asarray(x)
    dy = np.asarray(dy)
    N, C, H, W = x.shape
    dx = np.empty((N, C, H, W), dtype=np.float64)
    dgamma = np.empty(C)
    dbeta = np.empty(C)
    for k in range(C):
        xk = x[:, k].astype(np.float64)
        g = dy[:, k].astype(np.float64)                      # dl/dy
        S = subset_mask(N, H, W, boxes[k])
        s = subset_size(boxes[k])
        E, V = float(mean[k]), float(var[k])
        r = 1.0 / math.sqrt(V + eps)
        x_hat = (xk - E) * r

        dl_dxhat = g * float(gamma[k])
        dl_dE = (dl_dxhat * (-r)).sum()
        dl_dVar = (dl_dxhat * (xk - E) * (-0.5) * (V + eps) ** (-1.5)).sum()

        d = dl_dxhat * r                                      # "otherwise" branch of Eq. 6
        d[S] += dl_dE * (1.0 / s) + dl_dVar * (2.0 * (xk[S] - E) / s)     # x_i in S
        dx[:, k] = d
        dgamma[k] = (g * x_hat).sum()
        dbeta[k] = g.sum()
    return dict(dx=dx, dgamma=dgamma, dbeta=dbeta)


# --------------------------------------------------------------------------
# VDN combined with a sampling strategy: Eq. 4
# --------------------------------------------------------------------------
def sample_index_mixed(N: int, C: int, H: int, W: int, mode: int, n_v: int, *, n_s: int = 0,
                       patch_h: int = 0, patch_w: int = 0, fs_per_channel: int = 0,
                       seed: int = 0, layer_id: int = 0, epoch: int = 0):
    """Location sets for "VDN + sampling" (Section 4.2, step 3; Eq. 4).

    The batch holds n_v virtual samples in front of N - n_v real ones (Alg. 3).  Returns
    (boxes_v, boxes_s): x_v = the virtual samples 0 .. n_v-1, x_s = the real samples
    sampled by ``mode`` exactly as in Alg. 1 / Alg. 2 applied to the real part of the batch
    (sample indices shifted by n_v).
    """
    real = sample_index(N - n_v, C, H, W, mode, n_s=n_s, patch_h=patch_h, patch_w=patch_w,
                        fs_per_channel=fs_per_channel, seed=seed, layer_id=layer_id, epoch=epoch)
    boxes_s = real.copy()
    boxes_s[:, 0] += n_v
    boxes_v = np.tile(np.array([[0, n_v, 0, H, 0, W]], dtype=np.int64), (C, 1))
    return boxes_v, boxes_s


def forward_mixed(x, gamma, beta, boxes_v, boxes_s, mix_beta: float, eps: float, momentum: float = 0.1,
                  running_mean=None, running_var=None):
    """Eq. 4: X = beta_mix * X[x_v] + (1 - beta_mix) * X[x_s] for X in {E, Var}, each X[.] by Eq. 3
    on its own set (Var[x_v] about E[x_v], Var[x_s] about E[x_s]); then Eq. 1 on every point."""
    x = np.asarray(x)
    N, C, H, W = x.shape
    y = np.empty((N, C, H, W), dtype=np.float64)
    E, Var, E_v, E_s = (np.empty(C) for _ in range(4))
    for k in range(C):
        xk = x[:, k].astype(np.float64)
        x_v = xk[subset_mask(N, H, W, boxes_v[k])]
        x_s = xk[subset_mask(N, H, W, boxes_s[k])]
        E_v[k] = x_v.sum() / x_v.size
        E_s[k] = x_s.sum() / x_s.size
        Var_v = ((x_v - E_v[k]) ** 2).sum() / x_v.size
        Var_s = ((x_s - E_s[k]) ** 2).sum() / x_s.size
        E[k] = mix_beta * E_v[k] + (1.0 - mix_beta) * E_s[k]            # Eq. 4, X = E
        Var[k] = mix_beta * Var_v + (1.0 - mix_beta) * Var_s            # Eq. 4, X = Var
        y[:, k] = float(gamma[k]) * (xk - E[k]) / math.sqrt(Var[k] + eps) + float(beta[k])
    out = dict(y=y, mean=E, var=Var, invstd=1.0 / np.sqrt(Var + eps), mean_v=E_v, mean_s=E_s)
    if running_mean is not None:
        a = float(momentum)
        out["running_mean"] = a * E + (1.0 - a) * np.asarray(running_mean, dtype=np.float64)
        out["running_var"] = a * Var + (1.0 - a) * np.asarray(running_var, dtype=np.float64)
    return out


def backward_mixed(x, dy, gamma, mean, var, mean_v, mean_s, boxes_v, boxes_s, mix_beta: float, eps: float):
    """Backward of ``forward_mixed``.  The paper prints no backward for Eq. 4; this is the chain
    rule in the form of Eq. 5 / Eq. 6: dl/dx^, dl/dE and dl/dVar exactly as in Eq. 5 (with the
    blended E and Var), and

        dl/dx_i = dl/dx^_i / sqrt(Var + eps) + dl/dE * dE/dx_i + dl/dVar * dVar/dx_i

    where, from Eq. 4 and Eq. 3, dE/dx_i = beta_mix / s_v and dVar/dx_i = beta_mix 2 (x_i - E_v) / s_v
    for x_i in the virtual set, (1 - beta_mix) / s_s and (1 - beta_mix) 2 (x_i - E_s) / s_s for x_i in
    the sampled real set, and zero elsewhere (the second branch of Eq. 6)."""
    x = np.asarray(x)
    dy = np.asarray(dy)
    N, C, H, W = x.shape
    dx = np.empty((N, C, H, W), dtype=np.float64)
    dgamma = np.empty(C)
    dbeta = np.empty(C)
    for k in range(C):
        xk = x[:, k].astype(np.float64)
        g = dy[:, k].astype(np.float64)
        E, V = float(mean[k]), float(var[k])
        r = 1.0 / math.sqrt(V + eps)
        dl_dxhat = g * float(gamma[k])
        dl_dE = (dl_dxhat * (-r)).sum()
        dl_dVar = (dl_dxhat * (xk - E) * (-0.5) * (V + eps) ** (-1.5)).sum()
        d = dl_dxhat * r
        for box, weight, centre in ((boxes_v[k], mix_beta, float(mean_v[k])),
                                    (boxes_s[k], 1.0 - mix_beta, float(mean_s[k]))):
            S = subset_mask(N, H, W, box)
            s = subset_size(box)
            d[S] += dl_dE * (weight / s) + dl_dVar * (weight * 2.0 * (xk[S] - centre) / s)
        dx[:, k] = d
        dgamma[k] = (g * (xk - E) * r).sum()
        dbeta[k] = g.sum()
    return dict(dx=dx, dgamma=dgamma, dbeta=dbeta)


# --------------------------------------------------------------------------
# Cost model of Appendix C.1 (used for the byte model and pinned to the
# numbers the paper prints)
# --------------------------------------------------------------------------
def adder_tree_speedup(m: int, s: int) -> float:
    """Forward speed-up of the reduction from the adder-tree depth, log_s(m)."""
    return math.log(m) / math.log(s)


def statistics_traffic_fraction(m: int, s: int) -> float:
    """Fraction of a feature map the statistics pass has to visit: s / m."""
    return s / float(m)
