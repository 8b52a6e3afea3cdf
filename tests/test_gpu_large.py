"""Tensors of more than 2^31 elements (element offsets beyond 32 bits, byte offsets beyond 2^33 in fp32).

Inputs this large are drawn on the device (seeded); a handful of channels, first, middle and last, are
copied back and the oracle evaluates exactly those (a channel is independent of the others).  Every
channel reaches the far end of the tensor through its last samples / rows, so each checked channel
exercises the large offsets."""
import numpy as np
import pytest
import torch

from oracle import bns_oracle as oracle
from paper_1810_10962_amd import bns
from paper_1810_10962_amd.workloads import BS, FS, Workload
from parity import assert_parity, oracle_boxes

pytestmark = pytest.mark.gpu

CASES = [
    # large planes: a channel is far too big for the single-launch kernels -> streaming kernels
    ("planes", (40, 1024, 240, 240), dict(mode=BS, n_s=5), "bf16"),
    ("planes", (40, 1024, 240, 240), dict(mode=FS, patch_h=60, patch_w=60), "bf16"),
    # many small channels: the single-launch kernels apply (N x C x H x W)
    ("channels", (64, 16384, 48, 48), dict(mode=BS, n_s=8), "bf16"),
    ("channels", (64, 16384, 48, 48), dict(mode=FS, patch_h=12, patch_w=12), "f32"),
]


@pytest.mark.parametrize("layout", ["nchw", "nhwc"])
@pytest.mark.parametrize("kind,shape,mkw,dtype", CASES, ids=[f"{c[0]}-{c[2]['mode']}-{c[3]}" for c in CASES])
def test_more_than_2_31_elements(kind, shape, mkw, dtype, layout):
    N, C_, H, W = shape
    assert N * C_ * H * W > 2 ** 31
    wl = Workload(name=f"large_{kind}", N=N, C=C_, H=H, W=W, dtype=dtype, layout=layout, data_seed=5, sampling_seed=11,
                  layer_id=2, epoch=3, **mkw)
    print(f"[gpu-case] large {layout} {shape} {dtype} {mkw}", flush=True)
    dev = torch.device("cuda:0")
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    g = torch.Generator(device=dev)
    g.manual_seed(wl.data_seed)
    f32 = dict(dtype=torch.float32, device=dev)
    mu = torch.rand(C_, generator=g, **f32) * 2 - 1
    sigma = torch.rand(C_, generator=g, **f32) * 1.5 + 0.5
    gamma = torch.rand(C_, generator=g, **f32) + 0.5
    beta = torch.rand(C_, generator=g, **f32) - 0.5
    stored = (N, H, W, C_) if layout == "nhwc" else (N, C_, H, W)
    per_c = (lambda v: v.view(1, 1, 1, C_)) if layout == "nhwc" else (lambda v: v.view(1, C_, 1, 1))
    x = torch.randn(stored, generator=g, dtype=tdt, device=dev)
    x.mul_(per_c(sigma).to(tdt)).add_(per_c(mu).to(tdt))
    dy = torch.randn(stored, generator=g, dtype=tdt, device=dev)
    y, dx = torch.empty_like(x), torch.empty_like(x)
    save_mean, save_invstd, dgamma, dbeta = (torch.empty(C_, **f32) for _ in range(4))
    rm, rv = torch.zeros(C_, **f32), torch.ones(C_, **f32)
    shp = bns.make_shape(N, C_, H, W, dtype, layout)
    spec = bns.make_spec(wl.mode, wl.n_s, wl.patch_h, wl.patch_w, 0, wl.layer_id, wl.epoch)
    ws = torch.empty(bns.bns_workspace_bytes(shp, spec), dtype=torch.uint8, device=dev)
    bns.bns_forward(shp, spec, wl.sampling_seed, x, gamma, beta, wl.eps, wl.momentum, y, save_mean, save_invstd, rm, rv, ws)
    bns.bns_backward(shp, spec, wl.sampling_seed, x, dy, gamma, save_mean, save_invstd, dx, dgamma, dbeta, ws)
    torch.cuda.synchronize()
    if layout == "nchw" and kind == "channels":
        assert bns.bns_get_option("last_path_backward") == 2          # the single-launch kernel ran

    ch = [0, 1, C_ // 2 - 1, C_ // 2, C_ - 2, C_ - 1]
    idx = torch.tensor(ch, device=dev)
    if layout == "nhwc":
        take = lambda t: t.index_select(3, idx).permute(0, 3, 1, 2).float().cpu().numpy()
    else:
        take = lambda t: t.index_select(1, idx).float().cpu().numpy()
    vec = lambda t: t[idx].cpu().numpy()
    inp = dict(x=take(x), dy=take(dy), gamma=vec(gamma), beta=vec(beta))
    res = dict(y=take(y), dx=take(dx), save_mean=vec(save_mean), save_invstd=vec(save_invstd), running_mean=vec(rm),
               running_var=vec(rv), dgamma=vec(dgamma), dbeta=vec(dbeta))
    del x, dy, y, dx
    torch.cuda.empty_cache()
    boxes = oracle_boxes(wl)[ch]
    assert (bns.bns_sample_index(shp, spec, wl.sampling_seed)[ch] == boxes).all()
    k = len(ch)
    f = oracle.forward(inp["x"], inp["gamma"], inp["beta"], boxes, wl.eps, wl.momentum, np.zeros(k), np.ones(k))
    b = oracle.backward(inp["x"], inp["dy"], inp["gamma"], f["mean"], f["var"], boxes, wl.eps)
    ref = dict(y=f["y"], save_mean=f["mean"], save_invstd=f["invstd"], running_mean=f["running_mean"],
               running_var=f["running_var"], dx=b["dx"], dgamma=b["dgamma"], dbeta=b["dbeta"])
    errs = assert_parity(res, ref, wl, what=f"large {layout} {shape}")
    print(f"[gpu-case] large scaled errors {errs}", flush=True)
