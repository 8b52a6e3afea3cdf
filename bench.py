#!/usr/bin/env python3
"""Benchmark of libbns on one MI355X: sampled batch normalisation, forward + backward.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload imagenet_bs] [--quick]

A step is one bns_forward + bns_backward over one synthetic batch that is already
resident in HBM.  The workload is the shape the headline metric is quoted on,
NCHW 64x256x56x56 fp32 with Batch Sampling 8/64; the other sampling modes, full BN and
the bf16 variants of the same tensor are timed after it and reported under "variants".
Buffers rotate between steps so that no step finds its inputs in the last-level cache.

Prints ONE JSON line.  `value` is the effective bandwidth in the unit the metric is defined
in: the bytes of the two-pass byte model (see algorithmic_bytes) divided by the measured time
per step.  The single-launch kernels move fewer bytes than that model; what really crosses the
HBM interface is reported beside it (`measured_hbm_GBs`, `measured_pct_of_peak`, from hardware
counters), and `roofline` prices the dominant kernel by the bytes that kernel has to move.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X HBM3E, published peak
METRIC = "BN fwd+bwd effective HBM GB/s (% peak) and speedup vs full BN, 64x256x56x56"

# HBM traffic per launch measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE), scaled by what the same counters
# read for bns_copy_reference of known size: profiles/hbm_traffic.json (the summaries beside it give the commands).
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")


def load_traffic():
    try:
        with open(TRAFFIC_FILE) as f:
            return json.load(f)
    except (OSError, ValueError):
        return {"bytes_per_launch": {}, "measured_at_commit": None}


def default_path_kernels(wl, dirs, bns):
    """Names of the kernels one default forward + backward launches for this workload (as in the counter table)."""
    pre = "nhwc_" if wl.layout == "nhwc" else ""
    fwd = {"fused": ["fused_forward_kernel"], "one-launch": [pre + "small_forward_kernel"],
           "streaming": ([pre + "stats_partial_kernel", pre + "stats_finalize_kernel"] if wl.layout == "nhwc" else
                         ["stats_one_block_kernel"]) + [pre + "normalize_kernel"]}[dirs["forward_path"]]
    fused_bwd = {1: "fused_backward_kernel", 2: "fused_backward_kernel", 3: "fused_backward_pipe_kernel"}
    bwd = {"fused": [fused_bwd.get(bns.bns_get_option("last_fused_backward"), "fused_backward_kernel")],
           "one-launch": [pre + "small_backward_kernel"],
           "streaming": [pre + "reduce_partial_kernel", pre + "reduce_finalize_kernel", pre + "dx_kernel"],
           # N x H x W x C: dx outside S written by the reduction kernel, the rows of S by a kernel of their own
           "streaming-split": ["nhwc_reduce_outside_kernel", "nhwc_reduce_finalize_kernel", "nhwc_dx_rows_kernel"],
           }[dirs["backward_path"]]
    return fwd, bwd


def sampling_ratio(wl, boxes) -> float:
    b = boxes[0]
    return float(b[1]) * float(b[3]) * float(b[5]) / float(wl.N * wl.H * wl.W)


def algorithmic_bytes(wl, r: float) -> dict:
    """Bytes each stage has to move, per step (e = element size).

    statistics  : read x on S only                      r e E
    normalise   : read x, write y                       2 e E
    bwd reduce  : read dy and x, all m points           2 e E
    dx          : read dy, write dx, read x on S    (2 + r) e E
    Per-channel vectors and the partial-sum workspace are O(C) and left out.
    """
    e = 4 if wl.dtype == "f32" else 2
    E = wl.elements
    st = dict(stats=r * e * E, normalize=2 * e * E, reduce=2 * e * E, dx=(2 + r) * e * E)
    st["fwd+bwd"] = sum(st.values())
    return st


class DeviceSet:
    """`nset` rotating buffer sets for one workload plus the shared per-channel tensors."""

    def __init__(self, wl, inputs, nset, torch, bns):
        self.wl = wl
        self.bufs = [bns.Buffers(wl, inputs)]
        for _ in range(nset - 1):
            b = bns.Buffers.__new__(bns.Buffers)
            b.__dict__.update(self.bufs[0].__dict__)
            b._fwd_args = b._bwd_args = None
            for name in ("x", "dy"):
                setattr(b, name, getattr(self.bufs[0], name).clone())
            for name in ("y", "dx"):
                setattr(b, name, torch.empty_like(self.bufs[0].x))
            self.bufs.append(b)
        self.i = 0

    def next(self):
        b = self.bufs[self.i % len(self.bufs)]
        self.i += 1
        return b


def time_steps(ds, steps, warmup, torch):
    for _ in range(warmup):
        b = ds.next()
        b.forward()
        b.backward()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        b = ds.next()
        b.forward()
        b.backward()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def time_stages(ds, steps, torch, bns):
    """Average duration of every stage, HIP events on the stream the kernels run on."""
    wl = ds.wl
    names = ["stats", "normalize", "reduce", "dx"]
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(steps)]
    for s in range(steps):
        b = ds.next()
        e = evs[s]
        e[0].record()
        bns.bns_forward_stats(b.shape, b.spec, b.seed, b.x, wl.eps, wl.momentum, b.save_mean, b.save_invstd,
                              b.running_mean, b.running_var, b.workspace)
        e[1].record()
        bns.bns_forward_normalize(b.shape, b.x, b.gamma, b.beta, b.save_mean, b.save_invstd, b.y)
        e[2].record()
        bns.bns_backward_reduce(b.shape, b.x, b.dy, b.save_mean, b.save_invstd, b.dgamma, b.dbeta, b.workspace)
        e[3].record()
        bns.bns_backward_dx(b.shape, b.spec, b.seed, b.x, b.dy, b.gamma, b.save_mean, b.save_invstd, b.dgamma,
                            b.dbeta, b.dx)
        e[4].record()
    torch.cuda.synchronize()
    out = {}
    for k, name in enumerate(names):
        out[name] = float(np.mean([evs[s][k].elapsed_time(evs[s][k + 1]) for s in range(steps)])) * 1e-3
    return out


def time_directions(ds, steps, torch, bns):
    """Average duration of bns_forward and of bns_backward as the library runs them by default
    (event pairs on the launch stream), and which kernels each took."""
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
    for s in range(steps):
        b = ds.next()
        e = evs[s]
        e[0].record()
        b.forward()
        e[1].record()
        b.backward()
        e[2].record()
    torch.cuda.synchronize()
    paths = {1: "streaming", 2: "fused", 3: "one-launch", 4: "streaming-split"}
    c0 = bns.bns_get_option("launch_count")
    ds.bufs[0].forward()
    c1 = bns.bns_get_option("launch_count")
    ds.bufs[0].backward()
    c2 = bns.bns_get_option("launch_count")
    torch.cuda.synchronize()
    launches = ((c1 - c0) % (1 << 31), (c2 - c1) % (1 << 31))
    fwd = np.array([e[0].elapsed_time(e[1]) for e in evs]) * 1e-3
    bwd = np.array([e[1].elapsed_time(e[2]) for e in evs]) * 1e-3
    both = fwd + bwd
    stat = lambda a: {"mean": round(float(a.mean()) * 1e6, 2), "median": round(float(np.median(a)) * 1e6, 2),
                      "min": round(float(a.min()) * 1e6, 2)}
    return dict(forward=float(fwd.mean()), backward=float(bwd.mean()), launches=launches,
                spread_us={"forward": stat(fwd), "backward": stat(bwd), "forward+backward": stat(both)},
                forward_path=paths.get(bns.bns_get_option("last_path_forward"), "?"),
                backward_path=paths.get(bns.bns_get_option("last_path_backward"), "?"))


def time_copy(ds, steps, torch, bns):
    for _ in range(3):
        b = ds.next()
        bns.bns_copy_reference(b.y, b.x)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for a, z in evs:
        b = ds.next()
        a.record()
        bns.bns_copy_reference(b.y, b.x)
        z.record()
    torch.cuda.synchronize()
    return float(np.mean([a.elapsed_time(z) for a, z in evs])) * 1e-3


def cpu_baseline(wl, inputs, res, budget_s=12.0):
    """The fp64 oracle, as it stands, timed on this host on a bounded sample of channels.

    Channels are independent, so the sample is whole channels of the same tensor; it is also
    compared with what the GPU produced for them."""
    from oracle import bns_oracle as oracle

    boxes = oracle.sample_index(wl.N, wl.C, wl.H, wl.W, wl.mode, n_s=wl.n_s, patch_h=wl.patch_h, patch_w=wl.patch_w,
                                fs_per_channel=wl.fs_per_channel, seed=wl.sampling_seed, layer_id=wl.layer_id,
                                epoch=wl.epoch)
    tol = {"f32": 1e-5, "bf16": 1e-2}[wl.dtype]
    done, spent, worst = 0, 0.0, {}
    order = list(range(0, wl.C, 8)) + [c for c in range(wl.C) if c % 8]
    while done < len(order) and spent < budget_s:
        ch = np.asarray(order[done:done + 4])
        x, dy = inputs["x"][:, ch], inputs["dy"][:, ch]
        t0 = time.perf_counter()
        f = oracle.forward(x, inputs["gamma"][ch], inputs["beta"][ch], boxes[ch], wl.eps, wl.momentum,
                           inputs["running_mean"][ch], inputs["running_var"][ch])
        b = oracle.backward(x, dy, inputs["gamma"][ch], f["mean"], f["var"], boxes[ch], wl.eps)
        spent += time.perf_counter() - t0
        ref = dict(y=f["y"], dx=b["dx"], save_mean=f["mean"], save_invstd=f["invstd"], dgamma=b["dgamma"],
                   dbeta=b["dbeta"])
        for k, rv in ref.items():
            g = res[k][:, ch] if res[k].ndim == 4 else res[k][ch]
            rms = np.sqrt(np.mean(rv ** 2, axis=(0, 2, 3), keepdims=True)) if rv.ndim == 4 else np.sqrt(np.mean(rv ** 2))
            err = float(np.max(np.abs(g - rv) / (np.abs(rv) + rms)))     # per-channel scale for the 4-D outputs
            worst[k] = max(worst.get(k, 0.0), err)
            assert err <= (tol if k in ("y", "dx") else 1e-5), f"GPU result differs from the oracle: {k} {err:.3e}"
        done += len(ch)
    r = sampling_ratio(wl, boxes)
    bytes_per_channel = algorithmic_bytes(wl, r)["fwd+bwd"] / wl.C

    # The same channels again, groups of four handed to a pool of threads (numpy releases the interpreter lock
    # inside its loops); the oracle itself is unchanged.
    def one_group(ch):
        x, dy = inputs["x"][:, ch], inputs["dy"][:, ch]
        f = oracle.forward(x, inputs["gamma"][ch], inputs["beta"][ch], boxes[ch], wl.eps, wl.momentum,
                           inputs["running_mean"][ch], inputs["running_var"][ch])
        oracle.backward(x, dy, inputs["gamma"][ch], f["mean"], f["var"], boxes[ch], wl.eps)

    threads = max(1, min(16, os.cpu_count() or 1))
    groups = [np.asarray(order[i:i + 4]) for i in range(0, done, 4)]
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=threads) as pool:
        t0 = time.perf_counter()
        list(pool.map(one_group, groups))
        spent_all = time.perf_counter() - t0
    return dict(value=round(bytes_per_channel * done / spent / 1e9, 4), unit="GB/s", cores=1, kind="oracle",
                all_cores=dict(value=round(bytes_per_channel * done / spent_all / 1e9, 4), unit="GB/s", cores=threads,
                               seconds=round(spent_all, 2)),
                sample=f"{done} of {wl.C} channels of the same tensor, oracle forward+backward in fp64 (numpy, "
                       f"one thread), {spent:.1f} s", elements_per_s=round(wl.elements / wl.C * done / spent, 1),
                max_scaled_error_vs_gpu={k: float(f"{v:.3e}") for k, v in worst.items()})


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="imagenet_bs")
    ap.add_argument("--quick", action="store_true", help="primary workload only, no variants, no CPU baseline")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (sampled BN keeps its statistics local to a GPU; "
              "no exchange between GPUs is part of the method); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_1810_10962_amd import bns, workloads

    bns.load()                                            # raises if libbns.so is missing: no fallback
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    K, W = args.steps, args.warmup

    wl = workloads.WORKLOADS[args.workload]
    inputs = workloads.make_inputs(wl)
    tensor_bytes = wl.elements * (4 if wl.dtype == "f32" else 2)
    nset = max(3, min(8, int(np.ceil(1.5e9 / (4 * tensor_bytes)))))       # rotate over >= 1.5 GB, at least 3 sets
    ds = DeviceSet(wl, inputs, nset, torch, bns)
    boxes = bns.bns_sample_index(ds.bufs[0].shape, ds.bufs[0].spec, wl.sampling_seed)
    r = sampling_ratio(wl, boxes)
    alg = algorithmic_bytes(wl, r)

    sec = time_steps(ds, K, W, torch)
    # the same steps on ONE buffer set: whatever the caches keep between forward, backward and the next step helps
    warm = DeviceSet.__new__(DeviceSet)
    warm.wl, warm.bufs, warm.i = wl, ds.bufs[:1], 0
    warm_sec = time_steps(warm, K, W, torch)
    dirs = time_directions(ds, K, torch, bns)
    stages = time_stages(ds, K, torch, bns)          # the streaming kernels one by one, for reference
    copy_s = time_copy(ds, min(K, 50), torch, bns)

    # Dominant kernel of the default path.  A fused direction is ONE kernel covering two rows of the
    # byte model (reduction + element-wise pass); a streaming direction is several kernels, of which
    # the longest single-kernel stage is taken (the statistics and reduce stages also contain a
    # one-block finalize kernel, so their event pair covers two launches).
    traffic_table = load_traffic()
    table = traffic_table.get("bytes_per_launch", {}).get(wl.name, {})
    fwd_kernels, bwd_kernels = default_path_kernels(wl, dirs, bns)
    # Candidates: (kernel, seconds per launch, bytes the kernel has to move, bytes of the same work in the two-pass
    # model, note).  A single-launch kernel keeps its channel on chip: forward reads x and writes y once (2e per
    # element); backward reads dy and x and writes dx once (3e; the plain flavour reads x again on S: (3+r)e).
    e_bytes = 4 if wl.dtype == "f32" else 2
    tensor = e_bytes * wl.elements
    cands = []
    if dirs["backward_path"] == "fused":
        plain = bns.bns_get_option("last_fused_backward") == 1
        cands.append((bwd_kernels[0], dirs["backward"], (3 + r if plain else 3) * tensor, alg["reduce"] + alg["dx"],
                      "single-launch backward: dy and x read once, dx written once, 3e bytes per element"
                      + (" + x again on S, r e" if plain else "")))
    elif dirs["backward_path"] == "streaming-split":
        # three launches timed as one (the event pair is around bns_backward): sums + dx outside S, finalize, dx on S
        cands.append((bwd_kernels[0], dirs["backward"], (3 + 2 * r) * tensor, alg["reduce"] + alg["dx"],
                      "backward in three launches, timed together: dy and x read once and dx written outside S by the "
                      "reduction kernel (3 - r) e, then dy, x, dx on the rows of S, 3 r e: (3 + 2r) e per element"))
    else:
        cands += [(bwd_kernels[0], stages["reduce"], alg["reduce"], alg["reduce"], "dy and x read once: 2e per element"),
                  (bwd_kernels[-1], stages["dx"], alg["dx"], alg["dx"], "dy read, dx written, x read on S: (2+r)e per element")]
    if dirs["forward_path"] == "fused":
        cands.append((fwd_kernels[0], dirs["forward"], 2 * tensor, alg["stats"] + alg["normalize"],
                      "single-launch forward: x read once, y written once, 2e bytes per element"))
    else:
        cands.append((fwd_kernels[-1], stages["normalize"], alg["normalize"], alg["normalize"],
                      "x read, y written: 2e per element"))
    kernel_name, dom_s, dom_bytes, two_pass_bytes, dom_note = max(cands, key=lambda c: c[1])
    achieved = dom_bytes / dom_s / 1e9
    traffic = table.get(kernel_name)
    if dirs["backward_path"] == "streaming-split" and kernel_name == bwd_kernels[0]:
        traffic = sum(table[k] for k in bwd_kernels) if all(k in table for k in bwd_kernels) else None
    roofline = dict(bound="hbm", kernel=kernel_name, achieved=round(achieved, 1), peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=round(achieved / HBM_PEAK_GBS, 4), traffic=traffic,
                    achieved_by_counters=round(traffic / dom_s / 1e9, 1) if traffic else None,
                    frac_by_counters=round(traffic / dom_s / 1e9 / HBM_PEAK_GBS, 4) if traffic else None,
                    stale=traffic is None, counters_measured_at_commit=traffic_table.get("measured_at_commit"),
                    algorithmic_bytes_per_launch=int(dom_bytes), algorithmic_bytes_note=dom_note,
                    effective_two_pass={"bytes_per_launch": int(two_pass_bytes),
                                        "GBs": round(two_pass_bytes / dom_s / 1e9, 1),
                                        "frac": round(two_pass_bytes / dom_s / 1e9 / HBM_PEAK_GBS, 4),
                                        "note": "the same work priced by the two-pass byte model that `value` uses "
                                                "(reductions 2e + dx (2+r)e, statistics r e + normalise 2e): bytes a "
                                                "kernel that keeps its channel on chip does not move, so not a bandwidth"},
                    avg_launch_us=round(dom_s * 1e6, 2),
                    timing="HIP events on the launch stream around the call, mean over the timed steps")
    # the whole default step by the counters: what forward + backward really moved through HBM
    step_kernels = fwd_kernels + bwd_kernels
    measured_step = sum(table[k] for k in step_kernels) if all(k in table for k in step_kernels) else None

    out = {
        "metric": METRIC, "value": round(alg["fwd+bwd"] / sec / 1e9, 1), "unit": "GB/s", "n_gpus": 1, "steps": K,
        "warmup": W, "ms_per_step": round(sec * 1e3, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32" if wl.dtype == "f32" else "bf16 storage, f32 arithmetic",
        "data": "synthetic",
        "config": {"workload": f"{wl.name}: {wl.layout.upper()} {wl.N}x{wl.C}x{wl.H}x{wl.W} {wl.dtype}, {wl.label()} "
                               f"(sampling ratio {r:.4f}), forward+backward, eps={wl.eps}, momentum={wl.momentum}",
                   "buffer_sets_rotated": nset},
        "pct_of_hbm_peak": round(100 * alg["fwd+bwd"] / sec / 1e9 / HBM_PEAK_GBS, 2),
        "elements_per_s": round(wl.elements / sec, 1),
        "algorithmic_bytes_per_step": int(alg["fwd+bwd"]),
        "hbm_bytes_measured_per_step": measured_step,
        "measured_hbm_GBs": round(measured_step / sec / 1e9, 1) if measured_step else None,
        "measured_pct_of_peak": round(100 * measured_step / sec / 1e9 / HBM_PEAK_GBS, 2) if measured_step else None,
        "measured_note": "FETCH_SIZE + WRITE_SIZE of the default path's kernels (profiles/hbm_traffic.json) over the time "
                         "per step; `value` counts the bytes of the two-pass byte model instead, which the single-launch "
                         "backward kernel undercuts by keeping a channel on chip",
        "warm": {"us_per_step": round(warm_sec * 1e6, 2), "GBs": round(alg["fwd+bwd"] / warm_sec / 1e9, 1),
                 "note": "one buffer set reused every step (value and ms_per_step rotate over buffer_sets_rotated sets)"},
        "default_path": {"forward": dirs["forward_path"], "backward": dirs["backward_path"],
                         "kernels": step_kernels, "launches": {"forward": dirs["launches"][0], "backward": dirs["launches"][1]},
                         "forward_us": round(dirs["forward"] * 1e6, 2), "backward_us": round(dirs["backward"] * 1e6, 2),
                         "event_pairs_us": dirs["spread_us"]},
        "streaming_stages_us": {k: round(v * 1e6, 2) for k, v in stages.items()},
        "streaming_stages_GBs": {k: round(alg[k] / stages[k] / 1e9, 1) for k in stages},
        "copy_reference": {"us": round(copy_s * 1e6, 2), "GBs": round(2 * tensor_bytes / copy_s / 1e9, 1)},
        "roofline": roofline,
    }

    if not args.quick:
        ds.bufs[0].forward()
        ds.bufs[0].backward()
        res = ds.bufs[0].results()
        out["cpu_baseline"] = cpu_baseline(wl, inputs, res)
        del ds
        torch.cuda.empty_cache()
        variants = {}
        base = wl.name.split("_")[0]
        for name in [f"{base}_bs", f"{base}_fs", f"{base}_full", f"{base}_bs_bf16", f"{base}_fs_bf16",
                     f"{base}_full_bf16", f"{base}_bs_nhwc", f"{base}_fs_nhwc", f"{base}_full_nhwc",
                     f"{base}_bs_nhwc_bf16", f"{base}_full_nhwc_bf16"]:
            if name not in workloads.WORKLOADS:
                continue
            v = workloads.WORKLOADS[name]
            vin = inputs
            if v.dtype == "bf16":
                vin = dict(inputs)
                vin["x"] = workloads.round_to_bf16(inputs["x"])
                vin["dy"] = workloads.round_to_bf16(inputs["dy"])
            vb = v.elements * (4 if v.dtype == "f32" else 2)
            vds = DeviceSet(v, vin, max(2, min(8, int(np.ceil(1.5e9 / (4 * vb))))), torch, bns)
            vr = sampling_ratio(v, bns.bns_sample_index(vds.bufs[0].shape, vds.bufs[0].spec, v.sampling_seed))
            vsec = time_steps(vds, K, W, torch)
            va = algorithmic_bytes(v, vr)["fwd+bwd"]
            variants[name] = dict(label=v.label(), dtype=v.dtype, layout=v.layout, ratio=round(vr, 4), us_per_step=round(vsec * 1e6, 2),
                                  effective_GBs=round(va / vsec / 1e9, 1),
                                  pct_of_hbm_peak=round(100 * va / vsec / 1e9 / HBM_PEAK_GBS, 2),
                                  elements_per_s=round(v.elements / vsec, 1))
            # the two kernel families side by side: streaming (several kernels, HBM re-read) and
            # fused (one launch per direction, channel kept on chip); `us_per_step` above is the default
            for label, path in (("streaming_us", 1), ("fused_us", 2)):
                bns.bns_set_option("path", path)
                try:
                    variants[name][label] = round(time_steps(vds, max(K // 2, 10), max(W // 2, 5), torch) * 1e6, 2)
                except bns.BnsError:
                    variants[name][label] = None
                finally:
                    bns.bns_set_option("path", 0)
            # each direction on its own (event pairs around the calls), default choice and streaming kernels:
            # the paper expects the forward pass to gain most (App. C.1)
            for prefix, path in (("", 0), ("streaming_", 1)):
                bns.bns_set_option("path", path)
                try:
                    d = time_directions(vds, max(K // 2, 10), torch, bns)
                finally:
                    bns.bns_set_option("path", 0)
                variants[name][prefix + "forward_us"] = round(d["forward"] * 1e6, 2)
                variants[name][prefix + "backward_us"] = round(d["backward"] * 1e6, 2)
            del vds
            torch.cuda.empty_cache()
        for name, v in variants.items():
            full = variants.get(name.replace("_bs", "_full").replace("_fs", "_full"))
            if full:
                v["speedup_vs_full_bn"] = round(full["us_per_step"] / v["us_per_step"], 4)
                if full.get("streaming_us") and v.get("streaming_us"):
                    # both sides with the streaming kernels only: the two-pass cost model of the paper (App. C.1)
                    v["speedup_vs_full_bn_streaming_kernels"] = round(full["streaming_us"] / v["streaming_us"], 4)
                v["forward_speedup_vs_full_bn"] = round(full["forward_us"] / v["forward_us"], 4)
                v["forward_speedup_vs_full_bn_streaming_kernels"] = round(
                    full["streaming_forward_us"] / v["streaming_forward_us"], 4)
        out["variants"] = variants
        if wl.name in variants and "speedup_vs_full_bn" in variants[wl.name]:
            out["speedup_vs_full_bn"] = variants[wl.name]["speedup_vs_full_bn"]
            out["speedup_vs_full_bn_streaming_kernels"] = variants[wl.name].get("speedup_vs_full_bn_streaming_kernels")
            out["forward_speedup_vs_full_bn_streaming_kernels"] = variants[wl.name][
                "forward_speedup_vs_full_bn_streaming_kernels"]
        # planes four times as large (the first-stage maps of the ImageNet models, Table 1): same element count
        big = {}
        big_inputs = None
        for name in ("stage1_bs", "stage1_fs", "stage1_full"):
            v = workloads.WORKLOADS[name]
            big_inputs = workloads.make_inputs(v) if big_inputs is None else big_inputs
            vds = DeviceSet(v, big_inputs, 2, torch, bns)
            vr = sampling_ratio(v, bns.bns_sample_index(vds.bufs[0].shape, vds.bufs[0].spec, v.sampling_seed))
            vsec = time_steps(vds, max(K // 2, 10), max(W // 2, 5), torch)
            vd = time_directions(vds, max(K // 2, 10), torch, bns)
            bns.bns_set_option("path", 1)
            try:
                ssec = time_steps(vds, max(K // 2, 10), max(W // 2, 5), torch)
            finally:
                bns.bns_set_option("path", 0)
            va = algorithmic_bytes(v, vr)["fwd+bwd"]
            big[name] = dict(shape="x".join(map(str, v.shape)), label=v.label(), ratio=round(vr, 4),
                             us_per_step=round(vsec * 1e6, 2), streaming_us=round(ssec * 1e6, 2),
                             forward_us=round(vd["forward"] * 1e6, 2), backward_us=round(vd["backward"] * 1e6, 2),
                             paths=f'{vd["forward_path"]}/{vd["backward_path"]}', effective_GBs=round(va / vsec / 1e9, 1),
                             ideal_speedup_two_pass_model=round(32.0 / (24.0 + 8.0 * vr), 4))
            del vds
            torch.cuda.empty_cache()
        for name, v in big.items():
            v["speedup_vs_full_bn"] = round(big["stage1_full"]["us_per_step"] / v["us_per_step"], 4)
            v["speedup_vs_full_bn_streaming_kernels"] = round(big["stage1_full"]["streaming_us"] / v["streaming_us"], 4)
            v["forward_speedup_vs_full_bn"] = round(big["stage1_full"]["forward_us"] / v["forward_us"], 4)
        out["large_plane_variants"] = big
        del big_inputs
        others = {}
        for name in ("tiny_bs", "cifar_fs", "vdn", "vdn_fs_mix", "vdn_bs_mix", "micro_a_fs", "micro_a_full", "micro_b_fs",
                     "micro_b_full"):
            v = workloads.WORKLOADS[name]
            vin = workloads.make_inputs(v)
            vb = v.elements * 4
            vds = DeviceSet(v, vin, max(2, min(8, int(np.ceil(1.5e9 / (4 * vb))))), torch, bns)
            if v.n_v and v.mode != workloads.VDN:         # Eq. 4: the virtual samples and the sampled real set
                vr = sampling_ratio(v, bns.bns_sample_index_mixed(vds.bufs[0].shape, vds.bufs[0].spec, v.sampling_seed,
                                                                  v.n_v)) + v.n_v / v.N
            else:
                vr = sampling_ratio(v, bns.bns_sample_index(vds.bufs[0].shape, vds.bufs[0].spec, v.sampling_seed))
            vsec = time_steps(vds, K, W, torch)
            va = algorithmic_bytes(v, vr)["fwd+bwd"]
            vd = time_directions(vds, K, torch, bns)
            others[name] = dict(shape="x".join(map(str, v.shape)), label=v.label(), us_per_step=round(vsec * 1e6, 2),
                                effective_GBs=round(va / vsec / 1e9, 1), elements_per_s=round(v.elements / vsec, 1),
                                # device side: event pairs around the two calls (kernels and the gap between them), and
                                # how many kernels they launch; us_per_step above also holds the host's call overhead
                                device_us=round((vd["forward"] + vd["backward"]) * 1e6, 2),
                                launches_per_step=vd["launches"][0] + vd["launches"][1],
                                paths=f'{vd["forward_path"]}/{vd["backward_path"]}')
            del vds
            torch.cuda.empty_cache()
        out["other_configs"] = others
        out["paper_context"] = ("paper reports up to 2x BN-layer speedup and up to 20% end-to-end (TensorFlow, "
                                "Titan Xp / V100, Sec. 5.2, Table 3); no kernel-level bandwidth is published")
    print(json.dumps(out))


if __name__ == "__main__":
    main()
