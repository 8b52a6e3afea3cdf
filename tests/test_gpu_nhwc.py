"""GPU parity of the N x H x W x C layout: the same oracle, the same logical [n, c, h, w] inputs; only
the memory order of x, y, dy, dx on the device differs (the binding transposes on upload / download)."""
import numpy as np
import pytest
import torch

from oracle import bns_oracle as oracle
from paper_1810_10962_amd import bns, workloads
from paper_1810_10962_amd.workloads import BS, FS, FULL, NS, VDN, Workload
from parity import assert_parity, oracle_boxes, oracle_boxes_mixed, oracle_reference, scaled_err

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True, params=["auto", "streaming"])
def kernel_choice(request):
    """Every test runs twice: with the default choice (small tensors take the one-launch kernels) and with the
    streaming kernels forced for every size."""
    bns.bns_set_option("nhwc_small", 0 if request.param == "auto" else 2)
    yield request.param
    bns.bns_set_option("nhwc_small", 0)


def _announce(msg):
    print(f"[gpu-case] nhwc {msg}", flush=True)


def _run(wl, inp=None):
    assert wl.layout == "nhwc"
    inp = workloads.make_inputs(wl) if inp is None else inp
    _announce(f"{wl.name} {wl.shape} {wl.dtype} mode={wl.mode} n_s={wl.n_s} patch={wl.patch_h}x{wl.patch_w} "
              f"epoch={wl.epoch}")
    return inp, bns.run_workload(wl, inp)


# channel counts: multiples of 8 (8-wide bf16), of 4 only, odd (scalar columns), more than one
# 64-access tile with a ragged last tile; row counts from 2 to tens of thousands
SMALL_SHAPES = [
    (8, 16, 8, 8),
    (5, 7, 7, 7),
    (3, 12, 6, 6),
    (4, 3, 10, 14),
    (2, 9, 1, 1),
    (1, 8, 24, 24),
    (17, 4, 40, 52),
    (6, 300, 4, 4),
    (3, 520, 5, 5),
    (2, 1, 9, 9),
]
MODES = [
    ("full", dict(mode=FULL)),
    ("ns", dict(mode=NS, n_s=1)),
    ("bs", dict(mode=BS, n_s=2)),
    ("fs", dict(mode=FS, patch_h=2, patch_w=3)),
    ("vdn", dict(mode=VDN, n_s=1)),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("mname,mkw", MODES, ids=[m[0] for m in MODES])
@pytest.mark.parametrize("shape", SMALL_SHAPES, ids=["x".join(map(str, s)) for s in SMALL_SHAPES])
def test_small_shapes_all_modes(shape, mname, mkw, dtype):
    N, C_, H, W = shape
    kw = dict(mkw)
    if kw.get("n_s", 0) > N or (kw["mode"] == VDN and N < 2) or (kw["mode"] == BS and N < 2):
        pytest.skip("mode not defined for this batch size")
    kw["patch_h"] = min(kw.get("patch_h", 0), H)
    kw["patch_w"] = min(kw.get("patch_w", 0), W)
    for epoch in range(3):
        wl = Workload(name=f"small_{mname}", N=N, C=C_, H=H, W=W, dtype=dtype, layout="nhwc", data_seed=100 + epoch,
                      sampling_seed=77, layer_id=3, epoch=epoch, **kw)
        inp, res = _run(wl)
        assert (res["boxes"] == oracle_boxes(wl)).all()
        assert_parity(res, oracle_reference(wl, inp), wl, what=f"nhwc {shape} {mname} {dtype} epoch {epoch}", inp=inp)


def test_extreme_offsets_are_exercised():
    N, C_, H, W = 8, 12, 12, 12
    seen_bs, seen_fs = set(), set()
    for epoch in range(200):
        wl = Workload(name="ext_bs", N=N, C=C_, H=H, W=W, mode=BS, n_s=3, sampling_seed=5, epoch=epoch, data_seed=epoch,
                      layout="nhwc")
        b = int(oracle_boxes(wl)[0, 0])
        if b in (0, N - 3) and b not in seen_bs:
            seen_bs.add(b)
            inp, res = _run(wl)
            assert_parity(res, oracle_reference(wl, inp), wl, what=f"BS begin {b}")
        wl = Workload(name="ext_fs", N=N, C=C_, H=H, W=W, mode=FS, patch_h=5, patch_w=4, sampling_seed=5, epoch=epoch,
                      data_seed=epoch, layout="nhwc")
        bx = oracle_boxes(wl)[0]
        key = (int(bx[2]), int(bx[4]))
        if key[0] in (0, H - 5) and key[1] in (0, W - 4) and key not in seen_fs:
            seen_fs.add(key)
            inp, res = _run(wl)
            assert_parity(res, oracle_reference(wl, inp), wl, what=f"FS corner {key}")
    assert seen_bs == {0, N - 3}
    assert len(seen_fs) >= 2


@pytest.mark.parametrize("shape,mkw", [
    ((65535, 2, 1, 1), dict(mode=BS, n_s=4096)),            # the largest N, two scalar columns
    ((65535, 8, 1, 3), dict(mode=FS, patch_h=1, patch_w=2)),
    ((2, 70000, 2, 2), dict(mode=BS, n_s=1)),               # many channel tiles, eight rows
    ((3, 40001, 1, 1), dict(mode=FULL)),                    # odd channel count: scalar columns, three rows
    ((1, 4, 1024, 1024), dict(mode=FS, patch_h=256, patch_w=128)),   # a million rows of one access each
    ((2, 1, 1500, 1400), dict(mode=BS, n_s=1)),             # a single column
], ids=lambda v: "x".join(map(str, v)) if isinstance(v, tuple) else None)
def test_extents_at_the_edges_of_the_supported_range(shape, mkw):
    N, C_, H, W = shape
    wl = Workload(name="edge", N=N, C=C_, H=H, W=W, data_seed=77, sampling_seed=5, layer_id=9, epoch=1, layout="nhwc",
                  **mkw)
    inp, res = _run(wl)
    assert (res["boxes"] == oracle_boxes(wl)).all()
    assert_parity(res, oracle_reference(wl, inp), wl, what=f"nhwc edge {shape}", inp=inp)


def test_degenerate_subsets_and_large_mean():
    wl = Workload(name="one_point", N=1, C=5, H=6, W=6, mode=FS, patch_h=1, patch_w=1, sampling_seed=3, layout="nhwc")
    inp, res = _run(wl)
    assert_parity(res, oracle_reference(wl, inp), wl, what="s = 1", inp=inp)
    np.testing.assert_allclose(res["save_invstd"], 1 / np.sqrt(np.float32(1e-5)), rtol=1e-6)
    wl = wl.replace(N=4)
    inp = workloads.make_inputs(wl)
    inp["x"] = np.full_like(inp["x"], 3.25)
    _, res = _run(wl, inp)
    assert_parity(res, oracle_reference(wl, inp), wl, what="constant x")
    # |mean| = 1e3 std: the pivoted sums must not cancel (bounds as in the N x C x H x W test of the same name)
    wl = Workload(name="offset", N=16, C=8, H=16, W=16, mode=BS, n_s=4, sampling_seed=2, layout="nhwc")
    inp = workloads.make_inputs(wl)
    inp["x"] = (inp["x"] * 1e-2 + 10.0).astype(np.float32)
    _, res = _run(wl, inp)
    ref = oracle_reference(wl, inp)
    for k in ("save_mean", "save_invstd", "running_mean", "running_var", "dbeta"):
        assert scaled_err(res[k], ref[k]) <= 1e-5, k
    cond = float(np.max(np.abs(ref["save_mean"]) * ref["save_invstd"]))
    assert cond > 300
    for k in ("y", "dx", "dgamma"):
        assert scaled_err(res[k], ref[k]) <= 4 * 2.0 ** -24 * cond, k


@pytest.mark.parametrize("name", ["cifar_fs", "vdn", "micro_a_fs", "micro_a_full", "micro_b_fs"])
def test_benchmark_configs_full_tensor(name):
    wl = workloads.WORKLOADS[name].replace(layout="nhwc")
    inp, res = _run(wl)
    assert (res["boxes"] == oracle_boxes(wl)).all()
    errs = assert_parity(res, oracle_reference(wl, inp), wl, what=f"nhwc {name}")
    _announce(f"{name} scaled errors {errs}")


@pytest.fixture(scope="module")
def imagenet_inputs():
    _announce("generating 64x256x56x56 inputs")
    return workloads.make_inputs(workloads.WORKLOADS["imagenet_bs_nhwc"])


@pytest.mark.parametrize("name", ["imagenet_bs_nhwc", "imagenet_fs_nhwc", "imagenet_full_nhwc",
                                  "imagenet_bs_nhwc_bf16"])
def test_imagenet_shape_all_channels(name, imagenet_inputs):
    """Full 64x256x56x56 tensor in the launch configuration the benchmark times, every channel."""
    wl = workloads.WORKLOADS[name]
    inp = imagenet_inputs
    if wl.dtype == "bf16":
        inp = dict(inp)
        inp["x"] = workloads.round_to_bf16(inp["x"])
        inp["dy"] = workloads.round_to_bf16(inp["dy"])
    _, res = _run(wl, inp)
    assert (res["boxes"] == oracle_boxes(wl)).all()
    worst = {}
    step = 32
    for c0 in range(0, wl.C, step):
        ch = list(range(c0, min(c0 + step, wl.C)))
        errs = assert_parity(res, oracle_reference(wl, inp, channels=ch), wl, channels=ch, what=f"{name} ch {c0}")
        for k, v in errs.items():
            worst[k] = max(worst.get(k, 0.0), v)
    _announce(f"{name} worst scaled errors {worst}")


def test_bit_identical_reruns_and_stage_calls():
    wl = workloads.WORKLOADS["cifar_fs"].replace(N=16, layout="nhwc")
    inp = workloads.make_inputs(wl)
    a = bns.run_workload(wl, inp)
    b = bns.run_workload(wl, inp)
    for k in a:
        assert (a[k].view(np.uint32) == b[k].view(np.uint32)).all() if a[k].dtype == np.float32 else (a[k] == b[k]).all()
    buf = bns.Buffers(wl, inp)
    bns.bns_forward_stats(buf.shape, buf.spec, buf.seed, buf.x, wl.eps, wl.momentum, buf.save_mean, buf.save_invstd,
                          buf.running_mean, buf.running_var, buf.workspace)
    bns.bns_forward_normalize(buf.shape, buf.x, buf.gamma, buf.beta, buf.save_mean, buf.save_invstd, buf.y)
    bns.bns_backward_reduce(buf.shape, buf.x, buf.dy, buf.save_mean, buf.save_invstd, buf.dgamma, buf.dbeta,
                            buf.workspace)
    bns.bns_backward_dx(buf.shape, buf.spec, buf.seed, buf.x, buf.dy, buf.gamma, buf.save_mean, buf.save_invstd,
                        buf.dgamma, buf.dbeta, buf.dx)
    s = buf.results()
    for k in a:
        assert (a[k] == s[k]).all(), k
    assert bns.bns_get_option("last_path_forward") == 1 and bns.bns_get_option("last_path_backward") == 1
    # the whole call with dx outside S written by its reduction kernel (the stage calls cannot): same bits again
    bns.bns_set_option("nhwc_split_dx", 1)
    try:
        c = bns.run_workload(wl, inp)
        assert bns.bns_get_option("last_path_backward") == 4
    finally:
        bns.bns_set_option("nhwc_split_dx", 0)
    for k in a:
        assert (a[k] == c[k]).all(), k


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape,mkw", [
    ((16, 40, 12, 12), dict(mode=BS, n_s=3)),                       # S a run of rows in the middle
    ((16, 40, 12, 12), dict(mode=FS, patch_h=5, patch_w=3)),        # S short runs of rows in every sample
    ((9, 7, 7, 7), dict(mode=NS, n_s=8)),                           # S most of the rows, scalar columns
    ((6, 300, 20, 20), dict(mode=VDN, n_s=1)),                      # more than one tile of channels
    ((5, 16, 6, 6), dict(mode=FULL)),                               # nothing outside S
    ((40, 64, 28, 28), dict(mode=FS, patch_h=1, patch_w=1)),        # one row per sample
])
def test_backward_with_dx_split_by_the_branches_of_eq_6(shape, mkw, dtype, kernel_choice):
    """Backward with dx on the rows outside S written by the reduction kernel and the rows of S by a kernel of their
    own: the same expressions as the one-kernel dx pass, so the same bits, whichever way the split is forced."""
    if kernel_choice != "streaming":
        pytest.skip("the streaming kernels are the subject")
    N, C_, H, W = shape
    wl = Workload(name="split_dx", N=N, C=C_, H=H, W=W, dtype=dtype, layout="nhwc", data_seed=31, sampling_seed=32,
                  layer_id=4, epoch=1, **mkw)
    inp = workloads.make_inputs(wl)
    try:
        bns.bns_set_option("nhwc_split_dx", 1)
        _, split = _run(wl, inp)
        bns.bns_set_option("nhwc_split_dx", 2)
        whole = bns.run_workload(wl, inp)
    finally:
        bns.bns_set_option("nhwc_split_dx", 0)
    assert_parity(split, oracle_reference(wl, inp), wl, what=f"split dx {shape} {mkw} {dtype}", inp=inp)
    for k in ("dx", "dgamma", "dbeta"):
        assert (split[k] == whole[k]).all(), f"{k}: split and one-kernel dx differ"


def test_same_results_as_the_other_layout():
    """Both layouts compute the same function of the logical tensor: equal index, results equal up to rounding order."""
    wl = workloads.WORKLOADS["vdn"].replace(N=12, C=40)
    inp = workloads.make_inputs(wl)
    a = bns.run_workload(wl, inp)
    b = bns.run_workload(wl.replace(layout="nhwc"), inp)
    assert (a["boxes"] == b["boxes"]).all()
    for k in a:
        assert scaled_err(b[k], a[k]) <= (2e-5 if a[k].dtype == np.float32 else 0), k


@pytest.mark.parametrize("shape,dtype", [((6, 10, 12, 12), "f32"), ((3, 16, 7, 7), "f32"), ((8, 64, 28, 28), "bf16"),
                                         ((4, 9, 6, 6), "bf16")])
def test_inference_mode(shape, dtype):
    N, C_, H, W = shape
    wl = Workload(name="infer", N=N, C=C_, H=H, W=W, mode=FULL, dtype=dtype, data_seed=9, layout="nhwc")
    inp = workloads.make_inputs(wl)
    rng = np.random.default_rng(3)
    rm = rng.standard_normal(C_).astype(np.float32)
    rv = rng.uniform(0.2, 3.0, C_).astype(np.float32)
    inp["running_mean"], inp["running_var"] = rm, rv
    buf = bns.Buffers(wl, inp)
    bns.bns_inference(buf.shape, buf.x, buf.gamma, buf.beta, buf.running_mean, buf.running_var, wl.eps, buf.y)
    got = buf.results()["y"]
    ref = oracle.inference(inp["x"], inp["gamma"], inp["beta"], rm, rv, wl.eps)
    assert scaled_err(got, ref) <= (1e-5 if dtype == "f32" else 1e-2)


def test_unsupported_combinations_are_refused_on_the_device_too():
    wl = Workload(name="pc", N=4, C=8, H=6, W=6, mode=FS, patch_h=2, patch_w=2, fs_per_channel=1, layout="nhwc")
    buf = bns.Buffers(wl, workloads.make_inputs(wl))
    for call in (buf.forward, buf.backward):
        with pytest.raises(bns.BnsError) as e:
            call()
        assert e.value.status == bns.BNS_EUNSUPPORTED
    bns.bns_set_option("path", 2)                   # fused kernels exist for N x C x H x W only
    try:
        ok = bns.Buffers(wl.replace(fs_per_channel=0), workloads.make_inputs(wl))
        with pytest.raises(bns.BnsError) as e:
            ok.forward()
        assert e.value.status == bns.BNS_EUNSUPPORTED
    finally:
        bns.bns_set_option("path", 0)


def test_hip_graph_capture_and_replay():
    wl = workloads.WORKLOADS["cifar_fs"].replace(N=16, layout="nhwc")
    inp = workloads.make_inputs(wl)
    eager = bns.run_workload(wl, inp)
    buf = bns.Buffers(wl, inp)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        buf.forward()
        buf.backward()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        buf.forward()
        buf.backward()
    for replay in range(3):
        buf.running_mean.copy_(torch.from_numpy(inp["running_mean"]))
        buf.running_var.copy_(torch.from_numpy(inp["running_var"]))
        buf.y.fill_(float("nan"))
        buf.dx.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        got = buf.results()
        for k in eager:
            assert (got[k] == eager[k]).all(), f"replay {replay}: {k}"


def test_small_tensors_take_one_launch_per_direction(kernel_choice):
    wl = workloads.WORKLOADS["micro_a_fs"].replace(layout="nhwc")
    inp = workloads.make_inputs(wl)
    res = bns.run_workload(wl, inp)
    want = 3 if kernel_choice == "auto" else 1
    want_b = 3 if kernel_choice == "auto" else 1
    assert bns.bns_get_option("last_path_forward") == want and bns.bns_get_option("last_path_backward") == want_b
    assert_parity(res, oracle_reference(wl, inp), wl, what="micro_a_fs nhwc", inp=inp)
    big = workloads.WORKLOADS["cifar_fs"].replace(layout="nhwc", N=16)
    bns.run_workload(big, workloads.make_inputs(big))
    assert bns.bns_get_option("last_path_forward") == 1 and bns.bns_get_option("last_path_backward") == 1


MIXED_MODES = [
    ("full", dict(mode=FULL)),
    ("ns", dict(mode=NS, n_s=2)),
    ("bs", dict(mode=BS, n_s=2)),
    ("fs", dict(mode=FS, patch_h=3, patch_w=2)),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("mname,mkw", MIXED_MODES, ids=[m[0] for m in MIXED_MODES])
@pytest.mark.parametrize("shape", [(6, 16, 8, 8), (5, 7, 7, 7), (9, 36, 6, 6), (12, 4, 40, 52)],
                         ids=lambda s: "x".join(map(str, s)))
def test_vdn_plus_sampling_small_shapes(shape, mname, mkw, dtype):
    """Eq. 4 in this layout: virtual samples in front, the strategy applied to the real ones, several blends."""
    N, C_, H, W = shape
    for epoch, (n_v, mix_beta) in enumerate(((1, 0.5), (2, 0.3), (2, 1.0), (1, 0.0))):
        wl = Workload(name=f"mix_{mname}", N=N, C=C_, H=H, W=W, dtype=dtype, layout="nhwc", n_v=n_v, mix_beta=mix_beta,
                      data_seed=300 + epoch, sampling_seed=41, layer_id=6, epoch=epoch, **mkw)
        inp, res = _run(wl)
        bv, bs = oracle_boxes_mixed(wl)
        assert (res["boxes"] == bs).all()
        assert_parity(res, oracle_reference(wl, inp), wl,
                      what=f"nhwc mixed {shape} {mname} {dtype} n_v={n_v} beta={mix_beta}", inp=inp)


def test_row_subsets_that_split_into_more_blocks_than_the_whole_tensor():
    """Dealing rows out evenly is not monotonic: the 924 rows of a 33x28x1 tensor go to 55 blocks, the 896 rows of
    32 of its samples to 56.  The workspace regions must hold the larger count (the partial sums of the
    sampled set once ran into the region of the virtual set), for Eq. 4 and for plain Batch Sampling."""
    mixed = Workload(name="regions", N=33, C=260, H=28, W=1, mode=FULL, dtype="f32", layout="nhwc", n_v=1, mix_beta=0.5,
                     data_seed=817383120, sampling_seed=2850669091811702665, layer_id=3462304091, epoch=2332354607)
    inp, res = _run(mixed)
    assert_parity(res, oracle_reference(mixed, inp), mixed, what="nhwc regions, Eq. 4", inp=inp)
    virtual_large = mixed.replace(n_v=32, mix_beta=0.3)          # now the virtual set is the one with 56 blocks
    inp, res = _run(virtual_large)
    assert_parity(res, oracle_reference(virtual_large, inp), virtual_large, what="nhwc regions, large virtual set", inp=inp)
    plain = mixed.replace(n_v=0, mode=BS, n_s=32)
    inp, res = _run(plain)
    assert_parity(res, oracle_reference(plain, inp), plain, what="nhwc regions, Batch Sampling", inp=inp)


@pytest.mark.parametrize("name", ["vdn_fs_mix", "vdn_bs_mix"])
def test_vdn_plus_sampling_benchmark_shape(name):
    wl = workloads.WORKLOADS[name].replace(layout="nhwc")
    inp, res = _run(wl)
    errs = assert_parity(res, oracle_reference(wl, inp), wl, what=f"nhwc {name}", inp=inp)
    _announce(f"{name} scaled errors {errs}")
    nchw = bns.run_workload(wl.replace(layout="nchw"), inp)
    for k in ("save_mean", "save_invstd", "save_mean_parts", "dgamma", "dbeta"):
        assert scaled_err(res[k], nchw[k]) <= 2e-5, k
