"""Seeded synthetic workloads for sampled batch normalization.

This module only *produces inputs*: activation tensors, affine parameters and
upstream gradients with the shapes and value distributions of the workloads
that the Batch Normalization Sampling paper trains (ResNet/DenseNet feature
maps on CIFAR and ImageNet, Table 1 and Section 5).  Those datasets and
networks are not available, so i.i.d. Gaussian activations with a random
per-channel mean and scale stand in for them.

It holds none of the method's arithmetic (no statistics, no normalisation, no
index generation), so both the HIP library's tests and the CPU oracle's tests
may consume what it returns.  It imports neither of them.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

# Sampling modes, numbered as in include/bns.h.
FULL, NS, BS, FS, VDN = 0, 1, 2, 3, 4
MODE_NAMES = {FULL: "FULL", NS: "NS", BS: "BS", FS: "FS", VDN: "VDN"}


@dataclass(frozen=True)
class Workload:
    """One named benchmark / parity case.

    ``N`` counts every sample in the tensor.  For VDN it includes the ``n_s``
    virtual samples, which sit in front of the real ones (Algorithm 3).
    """

    name: str
    N: int
    C: int
    H: int
    W: int
    mode: int
    n_s: int = 0            # BS / NS: samples kept; VDN: number of virtual samples
    patch_h: int = 0        # FS
    patch_w: int = 0        # FS
    fs_per_channel: int = 0
    n_v: int = 0            # "VDN + sampling" (Eq. 4): virtual samples in front; mode then samples the real ones
    mix_beta: float = 0.5   # beta of Eq. 4
    dtype: str = "f32"      # "f32" | "bf16" : storage type of x, y, dy, dx
    layout: str = "nchw"    # "nchw" | "nhwc" : memory order on the device; arrays here are always [n, c, h, w]
    data_seed: int = 0
    sampling_seed: int = 0
    layer_id: int = 0
    epoch: int = 0
    eps: float = 1e-5
    momentum: float = 0.1
    extra: dict = field(default_factory=dict)

    @property
    def shape(self):
        return (self.N, self.C, self.H, self.W)

    @property
    def elements(self) -> int:
        return self.N * self.C * self.H * self.W

    def label(self) -> str:
        """Paper-style label "Approach-sampled/original" (Section 5, set-up)."""
        if self.mode in (BS, NS, VDN):
            return f"{MODE_NAMES[self.mode]}-{self.n_s}/{self.N}"
        if self.mode == FS:
            return f"FS-{self.patch_h}x{self.patch_w}/{self.H}x{self.W}"
        return f"BN-{self.N}/{self.N}"

    def replace(self, **kw) -> "Workload":
        d = self.__dict__.copy()
        d.update(kw)
        return Workload(**d)


_DATA_SEED = 1810_10962 * 10
_SAMP_SEED = 0xB45E5EED


def _wl(idx, name, N, C, H, W, mode, **kw):
    return Workload(name=name, N=N, C=C, H=H, W=W, mode=mode,
                    data_seed=_DATA_SEED + idx, sampling_seed=_SAMP_SEED + idx,
                    layer_id=idx, **kw)


WORKLOADS = {
    w.name: w for w in [
        _wl(1, "tiny_bs", 8, 16, 8, 8, BS, n_s=2),
        _wl(2, "cifar_fs", 128, 64, 32, 32, FS, patch_h=8, patch_w=8),
        _wl(3, "imagenet_bs", 64, 256, 56, 56, BS, n_s=8),
        _wl(3, "imagenet_fs", 64, 256, 56, 56, FS, patch_h=14, patch_w=14),
        _wl(3, "imagenet_full", 64, 256, 56, 56, FULL),
        _wl(3, "imagenet_bs_bf16", 64, 256, 56, 56, BS, n_s=8, dtype="bf16"),
        _wl(3, "imagenet_fs_bf16", 64, 256, 56, 56, FS, patch_h=14, patch_w=14, dtype="bf16"),
        _wl(3, "imagenet_full_bf16", 64, 256, 56, 56, FULL, dtype="bf16"),
        _wl(3, "imagenet_bs_nhwc", 64, 256, 56, 56, BS, n_s=8, layout="nhwc"),
        _wl(3, "imagenet_fs_nhwc", 64, 256, 56, 56, FS, patch_h=14, patch_w=14, layout="nhwc"),
        _wl(3, "imagenet_full_nhwc", 64, 256, 56, 56, FULL, layout="nhwc"),
        _wl(3, "imagenet_bs_nhwc_bf16", 64, 256, 56, 56, BS, n_s=8, dtype="bf16", layout="nhwc"),
        _wl(3, "imagenet_full_nhwc_bf16", 64, 256, 56, 56, FULL, dtype="bf16", layout="nhwc"),
        # the 112 x 112 maps of the first stage of the ImageNet models (Table 1): same element count as above, planes
        # four times as large, a quarter of the channels
        _wl(7, "stage1_bs", 64, 64, 112, 112, BS, n_s=8),
        _wl(7, "stage1_fs", 64, 64, 112, 112, FS, patch_h=28, patch_w=28),
        _wl(7, "stage1_full", 64, 64, 112, 112, FULL),
        _wl(4, "vdn", 130, 128, 28, 28, VDN, n_s=2),
        # "FS + VDN", the paper's best-accuracy combination (Table 2): 2 virtual + 128 real samples,
        # one 7x7 patch (1/16 of a 28x28 map) of every real sample, beta = 0.5
        _wl(4, "vdn_fs_mix", 130, 128, 28, 28, FS, patch_h=7, patch_w=7, n_v=2, mix_beta=0.5),
        _wl(4, "vdn_bs_mix", 130, 128, 28, 28, BS, n_s=4, n_v=2, mix_beta=0.5),
        _wl(5, "micro_a_fs", 2, 512, 14, 14, FS, patch_h=4, patch_w=4),
        _wl(5, "micro_a_full", 2, 512, 14, 14, FULL),
        _wl(6, "micro_b_fs", 1, 1024, 7, 7, FS, patch_h=4, patch_w=4),
        _wl(6, "micro_b_full", 1, 1024, 7, 7, FULL),
    ]
}


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even), returned as float32.

    A storage-format conversion of the *inputs*: both the oracle and the HIP path
    consume the rounded values, so neither sees more mantissa than the other.
    """
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    bias = ((u >> np.uint64(16)) & np.uint64(1)) + np.uint64(0x7FFF)
    r = ((u + bias) & np.uint64(0xFFFF0000)).astype(np.uint32)
    out = r.view(np.float32).reshape(a.shape).copy()
    nan = np.isnan(a)
    if nan.any():
        out[nan] = np.nan
    return out


def _conv3x3_same(v: np.ndarray, wgt: np.ndarray) -> np.ndarray:
    """Plain 3x3, stride-1, zero-padded convolution (cross-correlation) in fp64.

    v: [n, Cin, H, W], wgt: [Cout, Cin, 3, 3] -> [n, Cout, H, W].  Only used to
    turn virtual *inputs* into virtual *activations* for the VDN workload.
    """
    n, cin, H, W = v.shape
    cout = wgt.shape[0]
    vp = np.zeros((n, cin, H + 2, W + 2), dtype=np.float64)
    vp[:, :, 1:-1, 1:-1] = v
    out = np.zeros((n, cout, H, W), dtype=np.float64)
    for dh in range(3):
        for dw in range(3):
            patch = vp[:, :, dh:dh + H, dw:dw + W]              # [n, Cin, H, W]
            out += np.einsum("nchw,oc->nohw", patch, wgt[:, :, dh, dw])
    return out


def make_inputs(wl: Workload, channels: slice | None = None):
    """Return ``dict(x, gamma, beta, dy, running_mean, running_var)`` as float32 arrays.

    Recipe (per channel c): mu_c ~ U(-1, 1), sigma_c ~ U(0.5, 2),
    x[n, c, h, w] = mu_c + sigma_c * z with z ~ N(0, 1) i.i.d.;
    gamma ~ U(0.5, 1.5), beta ~ U(-0.5, 0.5); dy ~ N(0, 1) i.i.d.;
    running statistics start at (0, 1).

    VDN: the first ``n_s`` samples are *virtual*: inputs drawn i.i.d. U(0, 1) of
    shape [n_s, 3, H, W], passed through one seeded 3x3 convolution
    (weights ~ N(0, 2 / 27), no bias) to C channels.  The remaining samples are
    real activations drawn as above.

    For ``dtype == "bf16"`` x and dy are rounded to bfloat16 (still returned as
    float32 arrays holding the rounded values).

    ``channels`` restricts the *returned* tensors to a channel slice while
    drawing exactly the same random numbers, so that a subset of channels of a
    large workload can be regenerated cheaply for sampled parity checks.
    """
    N, C, H, W = wl.shape
    rng = np.random.Generator(np.random.PCG64(wl.data_seed))
    mu = rng.uniform(-1.0, 1.0, size=C).astype(np.float32)
    sigma = rng.uniform(0.5, 2.0, size=C).astype(np.float32)
    gamma = rng.uniform(0.5, 1.5, size=C).astype(np.float32)
    beta = rng.uniform(-0.5, 0.5, size=C).astype(np.float32)

    x = rng.standard_normal(size=(N, C, H, W), dtype=np.float32)
    x *= sigma[None, :, None, None]
    x += mu[None, :, None, None]
    dy = rng.standard_normal(size=(N, C, H, W), dtype=np.float32)

    if wl.mode == VDN or wl.n_v > 0:
        n_v = wl.n_s if wl.mode == VDN else wl.n_v
        cin = 3
        v_in = rng.uniform(0.0, 1.0, size=(n_v, cin, H, W))
        wgt = rng.standard_normal(size=(C, cin, 3, 3)) * np.sqrt(2.0 / (9 * cin))
        x[:n_v] = _conv3x3_same(v_in, wgt).astype(np.float32)

    if wl.dtype == "bf16":
        x = round_to_bf16(x)
        dy = round_to_bf16(dy)

    out = dict(
        x=x, dy=dy, gamma=gamma, beta=beta,
        running_mean=np.zeros(C, dtype=np.float32),
        running_var=np.ones(C, dtype=np.float32),
    )
    if channels is not None:
        out = dict(
            x=np.ascontiguousarray(out["x"][:, channels]),
            dy=np.ascontiguousarray(out["dy"][:, channels]),
            gamma=out["gamma"][channels].copy(), beta=out["beta"][channels].copy(),
            running_mean=out["running_mean"][channels].copy(),
            running_var=out["running_var"][channels].copy(),
        )
    return out
