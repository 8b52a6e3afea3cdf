"""Seeded random sweep over shapes, modes, storage types, layouts and kernel paths: every draw is one
forward + backward through the C ABI against the oracle.  The hand-picked cases elsewhere cover the
known corners; this one is for the corners nobody thought of (patches as wide as the plane, one
sample, one channel, planes of a single vector, ...)."""
import os

import numpy as np
import pytest

from paper_1810_10962_amd import bns, workloads
from paper_1810_10962_amd.workloads import BS, FS, FULL, NS, VDN, Workload
from oracle import bns_oracle as oracle
from parity import TOL_BF16, TOL_F32, assert_parity, oracle_boxes, oracle_boxes_mixed, oracle_reference, scaled_err

pytestmark = pytest.mark.gpu


def _draw(rng):
    if rng.integers(0, 8) == 0:                 # now and then a channel that needs a team of blocks
        N = int(rng.integers(16, 49))
        C_ = int(rng.choice([8, 24, 40]))
        H = W = int(rng.choice([7, 14, 15, 28, 30, 56]))      # 7, 15: scalar accesses; 14, 30: 64-bit ones in bf16
    else:
        N = int(rng.integers(1, 14))
        C_ = int(rng.choice([1, 2, 3, 4, 7, 8, 12, 16, 33, 40, 64, 130, 260, 515]))
        H = int(rng.choice([1, 2, 3, 4, 6, 7, 8, 12, 14, 16, 20]))
        W = int(rng.choice([1, 2, 3, 4, 6, 7, 8, 12, 14, 16, 28]))
    dtype = str(rng.choice(["f32", "bf16"]))
    layout = str(rng.choice(["nchw", "nhwc"]))
    mixed = bool(rng.integers(0, 3) == 0) and N >= 3
    n_v = int(rng.integers(1, min(3, N - 2) + 1)) if mixed else 0
    real = N - n_v
    modes = [FULL, NS, BS, FS] + ([] if mixed or N < 2 else [VDN])
    mode = int(rng.choice(modes))
    kw = dict(mode=mode)
    if mode in (NS, BS):
        kw["n_s"] = int(rng.integers(1, real + 1))
    elif mode == VDN:
        kw["n_s"] = int(rng.integers(1, N))
    elif mode == FS:
        kw["patch_h"] = int(rng.integers(1, H + 1))
        kw["patch_w"] = int(rng.integers(1, W + 1))
        kw["fs_per_channel"] = int(rng.integers(0, 2)) if layout == "nchw" else 0
    path = int(rng.choice([0, 0, 1, 2]))
    return Workload(name="rnd", N=N, C=C_, H=H, W=W, dtype=dtype, layout=layout, n_v=n_v,
                    mix_beta=float(rng.choice([0.0, 0.25, 0.5, 1.0])), data_seed=int(rng.integers(0, 2 ** 31)),
                    sampling_seed=int(rng.integers(0, 2 ** 62)), layer_id=int(rng.integers(0, 2 ** 32)),
                    epoch=int(rng.integers(0, 2 ** 32)), eps=float(rng.choice([1e-5, 1e-3])),
                    momentum=float(rng.choice([0.1, 0.3, 1.0])), **kw), path


# A longer or different sweep: BNS_SWEEP_CHUNKS chunks of 40 draws, seeded from BNS_SWEEP_SEED + chunk.
SWEEP_CHUNKS = int(os.environ.get("BNS_SWEEP_CHUNKS", "20"))
SWEEP_SEED = int(os.environ.get("BNS_SWEEP_SEED", "20181026"))


@pytest.mark.parametrize("chunk", range(SWEEP_CHUNKS))
def test_random_configurations(chunk):
    rng = np.random.default_rng(SWEEP_SEED + chunk)
    done = fused_refused = 0
    for i in range(40):
        wl, path = _draw(rng)
        print(f"[gpu-case] random {chunk}/{i}: {wl.shape} {wl.dtype} {wl.layout} mode={wl.mode} n_s={wl.n_s} "
              f"patch={wl.patch_h}x{wl.patch_w} pc={wl.fs_per_channel} n_v={wl.n_v} beta={wl.mix_beta} path={path}",
              flush=True)
        inp = workloads.make_inputs(wl)
        bns.bns_set_option("path", path)
        try:
            res = bns.run_workload(wl, inp)
        except bns.BnsError as e:
            # forcing the single-launch kernels is allowed to be refused (layout, scalar Eq. 4, channel too large)
            assert path == 2 and e.status == bns.BNS_EUNSUPPORTED, (wl, path, e)
            fused_refused += 1
            continue
        finally:
            bns.bns_set_option("path", 0)
        mixed = wl.n_v and wl.mode != VDN
        boxes = oracle_boxes_mixed(wl)[1] if mixed else oracle_boxes(wl)
        assert (res["boxes"] == boxes).all()
        ref = oracle_reference(wl, inp)
        assert_parity(res, ref, wl, what=f"random {chunk}/{i} {wl}", inp=inp)
        if not mixed and i % 3 == 0:            # the four stage calls on fresh buffers give the same
            buf = bns.Buffers(wl, inp)
            bns.bns_forward_stats(buf.shape, buf.spec, buf.seed, buf.x, wl.eps, wl.momentum, buf.save_mean,
                                  buf.save_invstd, buf.running_mean, buf.running_var, buf.workspace)
            bns.bns_forward_normalize(buf.shape, buf.x, buf.gamma, buf.beta, buf.save_mean, buf.save_invstd, buf.y)
            bns.bns_backward_reduce(buf.shape, buf.x, buf.dy, buf.save_mean, buf.save_invstd, buf.dgamma, buf.dbeta,
                                    buf.workspace)
            bns.bns_backward_dx(buf.shape, buf.spec, buf.seed, buf.x, buf.dy, buf.gamma, buf.save_mean,
                                buf.save_invstd, buf.dgamma, buf.dbeta, buf.dx)
            assert_parity(buf.results(), ref, wl, what=f"random {chunk}/{i} stages {wl}", inp=inp)
        if i % 4 == 1:                          # App. D: the same tensor normalised with given moving averages
            stats = np.random.default_rng(wl.data_seed)
            rm = stats.standard_normal(wl.C).astype(np.float32)
            rv = stats.uniform(0.0, 3.0, wl.C).astype(np.float32)
            buf = bns.Buffers(wl, dict(inp, running_mean=rm, running_var=rv))
            bns.bns_inference(buf.shape, buf.x, buf.gamma, buf.beta, buf.running_mean, buf.running_var, wl.eps, buf.y)
            want = oracle.inference(inp["x"], inp["gamma"], inp["beta"], rm, rv, wl.eps)
            # y against its own scale and the floor for the fp32 moving mean (see parity.saved_mean_rounding_scale)
            tol = TOL_F32 if wl.dtype == "f32" else TOL_BF16
            r = 1.0 / np.sqrt(rv.astype(np.float64) + wl.eps)
            floor = 2.0 * np.abs(inp["gamma"].astype(np.float64)) * r * 2.0 ** -24 * np.abs(rm) / tol
            assert scaled_err(buf.results()["y"], want, floor) <= tol, f"random {chunk}/{i} inference {wl}"
        done += 1
    assert done >= 20 and fused_refused <= 20


# Launch-choice overrides (include/bns.h, bns_set_option): documented ranges, extremes included.
OVERRIDES = {
    "norm_unroll": [0, 1, 2, 4], "dx_unroll": [0, 1, 2, 4], "reduce_unroll": [0, 1, 2, 4], "norm_nt": [0, 1, 2, 3, 4],
    "dx_nt": [0, 1, 2, 3, 4], "reduce_nt": [0, 1, 2, 3, 4], "cache_reuse": [0, 1, 2], "split_statistics": [0, 1], "splits_stats": [0, 1, 2, 7, 33, 64],
    "splits_reduce": [0, 1, 3, 16, 64], "channel_group": [0, 1, 3, 16, 100], "nhwc_blocks": [0, 1, 7, 256, 3000, 8192],
    "nhwc_ew_rows": [0, 1, 2, 9, 64, 5000, 1 << 20], "nhwc_small": [0, 2], "nhwc_split_dx": [0, 1, 2], "fused_variant": [0, 0, 1, 2, 3, 4, 5, 6, 7],
    "fused_keep_x": [0, 1, 2], "fused_patch_mask": [0, 1, 2], "fused_coop": [0, 1], "path": [0, 0, 1, 2],
    "fused_pipe": [0, 0, 1, 2, 3, 4, 5, 6, 16], "fused_team": [0, 0, 1, 2, 3, 5, 8, 16, 128],
}


@pytest.mark.parametrize("chunk", range(max(SWEEP_CHUNKS // 2, 1)))
def test_random_launch_overrides_do_not_change_results(chunk):
    """Random subsets of the launch-choice overrides at random values on random shapes: whatever kernels,
    block counts and access widths they select, the results still match the oracle."""
    rng = np.random.default_rng(SWEEP_SEED + 1000003 + chunk)
    done = 0
    for i in range(40):
        wl, _ = _draw(rng)
        opts = {k: int(rng.choice(v)) for k, v in OVERRIDES.items() if rng.integers(0, 3) == 0}
        print(f"[gpu-case] overrides {chunk}/{i}: {wl.shape} {wl.dtype} {wl.layout} mode={wl.mode} n_s={wl.n_s} "
              f"patch={wl.patch_h}x{wl.patch_w} pc={wl.fs_per_channel} n_v={wl.n_v} {opts}", flush=True)
        inp = workloads.make_inputs(wl)
        for k, v in opts.items():
            bns.bns_set_option(k, v)
        try:
            res = bns.run_workload(wl, inp)
        except bns.BnsError as e:
            # a forced single-launch kernel (or variant of it) may not exist for the shape
            assert e.status == bns.BNS_EUNSUPPORTED and (opts.get("path") == 2 or opts.get("fused_variant", 0) > 0), \
                (wl, opts, e)
            continue
        finally:
            for k in opts:
                bns.bns_set_option(k, 0)
        mixed = wl.n_v and wl.mode != VDN
        boxes = oracle_boxes_mixed(wl)[1] if mixed else oracle_boxes(wl)
        assert (res["boxes"] == boxes).all()
        assert_parity(res, oracle_reference(wl, inp), wl, what=f"overrides {chunk}/{i} {wl} {opts}", inp=inp)
        done += 1
    assert done >= 20
