"""Shared helpers of the GPU parity tests: oracle reference for a workload and the error metric."""
import numpy as np

from oracle import bns_oracle as oracle

# Tolerances stated for the build: fp32 1e-5, bf16 1e-2 (relative; see scaled_err).
TOL_F32 = 1e-5
TOL_BF16 = 1e-2


def oracle_boxes(wl, C=None):
    return oracle.sample_index(wl.N, wl.C if C is None else C, wl.H, wl.W, wl.mode, n_s=wl.n_s, patch_h=wl.patch_h,
                               patch_w=wl.patch_w, fs_per_channel=wl.fs_per_channel, seed=wl.sampling_seed,
                               layer_id=wl.layer_id, epoch=wl.epoch)


def oracle_boxes_mixed(wl):
    return oracle.sample_index_mixed(wl.N, wl.C, wl.H, wl.W, wl.mode, wl.n_v, n_s=wl.n_s, patch_h=wl.patch_h,
                                     patch_w=wl.patch_w, fs_per_channel=wl.fs_per_channel, seed=wl.sampling_seed,
                                     layer_id=wl.layer_id, epoch=wl.epoch)


def oracle_reference_mixed(wl, inp):
    """Oracle forward + backward for "VDN + sampling" (Eq. 4)."""
    bv, bs = oracle_boxes_mixed(wl)
    f = oracle.forward_mixed(inp["x"], inp["gamma"], inp["beta"], bv, bs, wl.mix_beta, wl.eps, wl.momentum,
                             inp["running_mean"], inp["running_var"])
    b = oracle.backward_mixed(inp["x"], inp["dy"], inp["gamma"], f["mean"], f["var"], f["mean_v"], f["mean_s"], bv, bs,
                              wl.mix_beta, wl.eps)
    return dict(y=f["y"], save_mean=f["mean"], save_invstd=f["invstd"], running_mean=f["running_mean"],
                running_var=f["running_var"], dx=b["dx"], dgamma=b["dgamma"], dbeta=b["dbeta"],
                save_mean_parts=np.concatenate([f["mean_v"], f["mean_s"]]))


def oracle_reference(wl, inp, channels=None):
    """Oracle forward + backward.  ``channels``: list of channel ids to evaluate (all by default);
    the returned tensors then hold only those channels, in that order."""
    if wl.n_v and wl.mode != 4:
        assert channels is None
        return oracle_reference_mixed(wl, inp)
    boxes = oracle_boxes(wl)
    if channels is not None:
        ch = np.asarray(channels)
        boxes = boxes[ch]
        sel = lambda a: a[:, ch] if a.ndim == 4 else a[ch]
        inp = {k: sel(v) for k, v in inp.items()}
    f = oracle.forward(inp["x"], inp["gamma"], inp["beta"], boxes, wl.eps, wl.momentum,
                       inp["running_mean"], inp["running_var"])
    b = oracle.backward(inp["x"], inp["dy"], inp["gamma"], f["mean"], f["var"], boxes, wl.eps)
    return dict(y=f["y"], save_mean=f["mean"], save_invstd=f["invstd"], running_mean=f["running_mean"],
                running_var=f["running_var"], dx=b["dx"], dgamma=b["dgamma"], dbeta=b["dbeta"])


def scaled_err(got, ref, floor=0.0):
    """max_i |got_i - ref_i| / (|ref_i| + max(RMS(ref), floor)).

    A purely element-wise relative error is undefined where y, dx or dbeta cross zero; adding an RMS
    to the denominator keeps it a relative measure at the output's own scale.  Every channel is a
    normalisation problem of its own, with its own scale gamma_c / sigma_c, so for the N x C x H x W
    outputs the RMS is taken per channel; per-channel vectors use the RMS over channels.
    ``floor`` (scalar or per channel) is the RMS of the terms the output is a difference of, for
    outputs that cancel."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.ndim == 4:
        rms = np.sqrt(np.mean(ref ** 2, axis=(0, 2, 3), keepdims=True))
        floor = np.asarray(floor, dtype=np.float64)
        if floor.ndim == 1:
            floor = floor[None, :, None, None]
        rms = np.maximum(rms, floor)
    else:
        rms = np.maximum(np.sqrt(np.mean(ref ** 2)), np.asarray(floor, dtype=np.float64))   # scalar or per channel
    return float(np.max(np.abs(got - ref) / (np.abs(ref) + rms + 1e-300)))


def direct_term_rms(inp, ref, channels=None):
    """Per-channel RMS of gamma * invstd * dy, the first term of both branches of Eq. 6.

    dx is that term minus the 1/s corrections.  For s of a few points the two nearly cancel
    (with s = m = 2 exactly, up to eps), and fp32 rounding of the terms then dominates the
    difference, so dx is measured against the larger of its own RMS and this one.  For the
    benchmark shapes (s in the thousands) the two are equal to within 1/s."""
    ch = slice(None) if channels is None else np.asarray(channels)
    a = (np.asarray(inp["gamma"], dtype=np.float64)[ch] * ref["save_invstd"])[None, :, None, None]
    return np.sqrt(np.mean((a * inp["dy"][:, ch].astype(np.float64)) ** 2, axis=(0, 2, 3)))


def saved_mean_rounding_scale(wl, inp, ref, tol, channels=None):
    """Per channel, the floors for y and dx that admit the error the fp32 rounding of save_mean alone causes.

    The interface hands E from the statistics to the normalisation and to the backward pass as a float, so
    x - E carries an error dE <= 2^-24 |E| whatever the kernels do.  Eq. 1 turns it into gamma r dE in y.  On
    S, Eq. 6 subtracts gamma r^2 w dgamma (x_i - E), w = 1/s (for Eq. 4 the set's weight and its own
    centre): dE moves the factor (x_i - E) by dE and, through the sum dgamma = r sum_j g_j (x_j - E) of Eq. 5, the
    factor dgamma by r |dbeta| dE, so dx_i moves by up to gamma r^2 w (|dgamma| + |dbeta| max|x^|) dE.  With few
    sampled points close together (large r) or far-away points outside S (large |dgamma|) either output can exceed
    the tolerance times its own scale.  Twice the bound, divided by the tolerance, is the scale against which
    such an error still passes.  dgamma itself moves by r |dbeta| dE (per-channel vectors: fp32 tolerance)."""
    ch = slice(None) if channels is None else np.asarray(channels)
    centre = np.abs(np.asarray(ref["save_mean"], dtype=np.float64))
    if wl.n_v and wl.mode != 4:
        bv, bs = oracle_boxes_mixed(wl)
        size = lambda b: (b[:, 1] * b[:, 3] * b[:, 5]).astype(np.float64)
        w = np.maximum(wl.mix_beta / size(bv), (1.0 - wl.mix_beta) / size(bs))[ch]
        parts = np.abs(np.asarray(ref["save_mean_parts"], dtype=np.float64)).reshape(2, -1)
        centre_sets = np.maximum(parts[0], parts[1])
    else:
        b = oracle_boxes(wl)[ch]
        w = 1.0 / (b[:, 1] * b[:, 3] * b[:, 5]).astype(np.float64)
        centre_sets = centre
    r = np.asarray(ref["save_invstd"], dtype=np.float64)
    g = np.abs(np.asarray(inp["gamma"], dtype=np.float64)[ch])
    xhat_max = np.max(np.abs(inp["x"][:, ch].astype(np.float64) - ref["save_mean"][None, :, None, None]), axis=(0, 2, 3)) * r
    return dict(y=2.0 * g * r * 2.0 ** -24 * centre / tol,
                dgamma=2.0 * r * np.abs(ref["dbeta"]) * 2.0 ** -24 * centre / TOL_F32,
                dx=2.0 * g * r * r * w * (np.abs(ref["dgamma"]) * centre_sets + np.abs(ref["dbeta"]) * xhat_max * centre)
                   * 2.0 ** -24 / tol)


def summand_scale(inp, ref, channels=None):
    """Per channel, sqrt(m) * RMS of the m summands of dbeta (dy) and of dgamma (dy * x^): the size such a
    sum has when its terms do not happen to cancel.

    dbeta and dgamma are sums of m signed terms.  With many channels the RMS over channels is that size;
    with one channel (or a few) it is whatever the one sum came to, and a sum that lands near zero by
    chance would be held to an absolute accuracy no fp32 summation of its terms has."""
    ch = slice(None) if channels is None else np.asarray(channels)
    dy = inp["dy"][:, ch].astype(np.float64)
    xh = (inp["x"][:, ch].astype(np.float64) - ref["save_mean"][None, :, None, None]) * ref["save_invstd"][None, :, None, None]
    m = dy.shape[0] * dy.shape[2] * dy.shape[3]
    return dict(dbeta=np.sqrt(m * np.mean(dy ** 2, axis=(0, 2, 3))),
                dgamma=np.sqrt(m * np.mean((dy * xh) ** 2, axis=(0, 2, 3))))


def parity_floors(wl, inp, ref, channels=None):
    """The floor of every output of ``ref`` (scalar or per channel), as assert_parity applies it when it is given
    the inputs.  0.0 = none: the output is measured against its own RMS alone."""
    tol_t = TOL_F32 if wl.dtype == "f32" else TOL_BF16
    floors = {}
    for k in ref:
        tol = tol_t if k in ("y", "dx") else TOL_F32          # per-channel vectors are fp32 in every mode
        floor = 0.0
        if inp is not None and k == "dx":
            floor = np.maximum(direct_term_rms(inp, ref, channels), saved_mean_rounding_scale(wl, inp, ref, tol, channels)["dx"])
        elif inp is not None and k == "y":
            floor = saved_mean_rounding_scale(wl, inp, ref, tol, channels)["y"]
        elif inp is not None and k in ("dgamma", "dbeta"):
            floor = summand_scale(inp, ref, channels)[k]
            if k == "dgamma":
                floor = np.maximum(floor, saved_mean_rounding_scale(wl, inp, ref, tol, channels)["dgamma"])
        elif k in ("save_mean", "running_mean"):
            # a mean is known to eps times the spread of what was averaged; with one or a few channels the RMS over
            # channels can be a mean that happens to lie near zero
            floor = (wl.momentum if k == "running_mean" else 1.0) / np.asarray(ref["save_invstd"], dtype=np.float64)
        elif k == "running_var":
            # a variance enters the method only as Var + eps (Eq. 1, and App. D for the moving average); where every
            # channel's variance is exactly zero (one sampled point) the RMS over channels is zero as well
            floor = wl.eps
        floors[k] = floor
    return floors


def plain_scale(ref_k):
    """The RMS that scaled_err adds to |ref| when there is no floor: per channel for the N x C x H x W outputs,
    over the channels for the per-channel vectors."""
    r = np.asarray(ref_k, dtype=np.float64)
    if r.ndim == 4:
        return np.sqrt(np.mean(r ** 2, axis=(0, 2, 3)))
    return np.sqrt(np.mean(r ** 2))


def assert_parity(res, ref, wl, channels=None, what="", inp=None, floors=True):
    """Every output of ``ref`` within the build's tolerance of the oracle.  floors=False: no floor on any output,
    i.e. |got - ref| / (|ref| + RMS(ref)) alone (the check for the benchmark configurations, whose outputs do
    not cancel)."""
    tol_t = TOL_F32 if wl.dtype == "f32" else TOL_BF16
    floor_of = parity_floors(wl, inp, ref, channels) if floors else {}
    errs = {}
    for k, r in ref.items():
        g = res[k]
        if channels is not None:
            g = g[:, channels] if g.ndim == 4 else g[channels]
        assert g.shape == r.shape, (k, g.shape, r.shape)
        assert np.isfinite(g).all(), f"{what} {k}: non-finite output"
        tol = tol_t if k in ("y", "dx") else TOL_F32          # per-channel vectors are fp32 in every mode
        errs[k] = scaled_err(g, r, floor_of.get(k, 0.0))
        assert errs[k] <= tol, f"{what} {k}: scaled error {errs[k]:.3e} > {tol:g}" + ("" if floors else " (no floors)")
    return errs
