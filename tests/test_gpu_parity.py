"""GPU parity: libbns (through the C ABI) against the fp64 CPU oracle, element by element."""
import numpy as np
import pytest
import torch

from oracle import bns_oracle as oracle
from paper_1810_10962_amd import bns, workloads
from paper_1810_10962_amd.workloads import BS, FS, FULL, NS, VDN, Workload
from parity import assert_parity, oracle_boxes, oracle_boxes_mixed, oracle_reference, scaled_err

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True, params=["auto", "streaming"])
def kernel_path(request):
    """Every test runs twice: with the default choice of kernels (the fused single-launch kernels
    whenever a channel fits on chip) and with the streaming multi-kernel path forced."""
    bns.bns_set_option("path", 0 if request.param == "auto" else 1)
    yield request.param
    bns.bns_set_option("path", 0)


def _announce(msg):
    print(f"[gpu-case] {msg}", flush=True)


def _run(wl, inp=None):
    inp = workloads.make_inputs(wl) if inp is None else inp
    _announce(f"{wl.name} {wl.shape} {wl.dtype} mode={wl.mode} n_s={wl.n_s} patch={wl.patch_h}x{wl.patch_w} "
              f"pc={wl.fs_per_channel} epoch={wl.epoch}")
    res = bns.run_workload(wl, inp)
    return inp, res


# ---------------------------------------------------------------------------------------
# sampling index: device generator = host generator = oracle, bit for bit
# ---------------------------------------------------------------------------------------
def test_index_device_equals_host_equals_oracle():
    """More than 10^4 random (shape, spec, seed, layer, epoch) tuples: the first few hundred with many channels
    (several blocks of the index kernel), the rest with a handful, so that the oracle's loop stays short."""
    rng = np.random.default_rng(1)
    for i in range(10500):
        N, H, W = (int(v) for v in rng.integers(1, 80, 3))
        C_ = int(rng.integers(1, 700)) if i < 300 else int(rng.integers(1, 7))
        mode = int(rng.integers(0, 5))
        if mode == VDN and N == 1:
            continue
        n_s = int(rng.integers(1, N)) if mode == VDN else int(rng.integers(1, N + 1))
        ph, pw = int(rng.integers(1, H + 1)), int(rng.integers(1, W + 1))
        pc = int(rng.integers(0, 2))
        seed = int(rng.integers(0, 2 ** 63)) * 2 + 1
        layer, epoch = int(rng.integers(0, 2 ** 32)), int(rng.integers(0, 2 ** 32))
        shape = bns.make_shape(N, C_, H, W)
        spec = bns.make_spec(mode, n_s, ph, pw, pc, layer, epoch)
        host = bns.bns_sample_index(shape, spec, seed)
        devc = bns.bns_sample_index_device(shape, spec, seed)
        ref = oracle.sample_index(N, C_, H, W, mode, n_s=n_s, patch_h=ph, patch_w=pw, fs_per_channel=pc,
                                  seed=seed, layer_id=layer, epoch=epoch)
        assert (host == ref).all() and (devc == ref).all(), (i, N, C_, H, W, mode)


# ---------------------------------------------------------------------------------------
# small shapes: every mode, ragged plane sizes (scalar, 4-wide and 8-wide paths), several
# blocks per channel, channel counts that do not divide a block
# ---------------------------------------------------------------------------------------
SMALL_SHAPES = [
    (8, 16, 8, 8),       # HW = 64
    (5, 7, 7, 7),        # HW = 49: scalar path, unaligned planes
    (3, 5, 6, 6),        # HW = 36: 4-wide, rows of 6 straddle vectors
    (4, 3, 10, 14),      # HW = 140: 4-wide fp32 and bf16
    (2, 9, 1, 1),        # fully-connected case, HW = 1
    (1, 6, 24, 24),      # single sample
    (17, 4, 40, 52),     # planes larger than one block's tile (2080 elements)
    (6, 300, 4, 4),      # many channels, tiny planes
]
MODES = [
    ("full", dict(mode=FULL)),
    ("ns", dict(mode=NS, n_s=1)),
    ("bs", dict(mode=BS, n_s=2)),
    ("fs", dict(mode=FS, patch_h=2, patch_w=3)),
    ("fs_pc", dict(mode=FS, patch_h=3, patch_w=2, fs_per_channel=1)),
    ("vdn", dict(mode=VDN, n_s=1)),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("mname,mkw", MODES, ids=[m[0] for m in MODES])
@pytest.mark.parametrize("shape", SMALL_SHAPES, ids=["x".join(map(str, s)) for s in SMALL_SHAPES])
def test_small_shapes_all_modes(shape, mname, mkw, dtype):
    N, C_, H, W = shape
    kw = dict(mkw)
    if kw.get("n_s", 0) > N or (kw["mode"] == VDN and N < 2):
        pytest.skip("mode not defined for this batch size")
    if kw["mode"] in (BS,) and N < 2:
        pytest.skip("needs two samples")
    kw["patch_h"] = min(kw.get("patch_h", 0), H)
    kw["patch_w"] = min(kw.get("patch_w", 0), W)
    for epoch in range(3):
        wl = Workload(name=f"small_{mname}", N=N, C=C_, H=H, W=W, dtype=dtype, data_seed=100 + epoch,
                      sampling_seed=77, layer_id=3, epoch=epoch, **kw)
        inp, res = _run(wl)
        assert (res["boxes"] == oracle_boxes(wl)).all()
        assert_parity(res, oracle_reference(wl, inp), wl, what=f"{shape} {mname} {dtype} epoch {epoch}", inp=inp)


def test_extreme_offsets_are_exercised():
    """begin = 0 and begin = N - n_s (Batch Sampling), patch in both corners (Feature Sampling)."""
    N, C_, H, W = 8, 6, 12, 12
    seen_bs, seen_fs = set(), set()
    for epoch in range(200):
        wl = Workload(name="ext_bs", N=N, C=C_, H=H, W=W, mode=BS, n_s=3, sampling_seed=5, epoch=epoch, data_seed=epoch)
        b = int(oracle_boxes(wl)[0, 0])
        if b in (0, N - 3) and b not in seen_bs:
            seen_bs.add(b)
            inp, res = _run(wl)
            assert_parity(res, oracle_reference(wl, inp), wl, what=f"BS begin {b}")
        wl = Workload(name="ext_fs", N=N, C=C_, H=H, W=W, mode=FS, patch_h=5, patch_w=4, sampling_seed=5, epoch=epoch,
                      data_seed=epoch)
        bx = oracle_boxes(wl)[0]
        key = (int(bx[2]), int(bx[4]))
        if key[0] in (0, H - 5) and key[1] in (0, W - 4) and key not in seen_fs:
            seen_fs.add(key)
            inp, res = _run(wl)
            assert_parity(res, oracle_reference(wl, inp), wl, what=f"FS corner {key}")
    assert seen_bs == {0, N - 3}
    assert len(seen_fs) >= 2


@pytest.mark.parametrize("shape,mkw", [
    ((65535, 2, 1, 1), dict(mode=BS, n_s=4096)),            # the largest N: fully-connected style, m = 65535
    ((65535, 1, 1, 3), dict(mode=FS, patch_h=1, patch_w=2)),
    ((2, 70000, 2, 2), dict(mode=BS, n_s=1)),               # many channels, tiny planes
    ((3, 40000, 1, 1), dict(mode=FULL)),
    ((1, 2, 1024, 1024), dict(mode=FS, patch_h=256, patch_w=128)),   # one very large plane per channel
    ((2, 1, 1500, 1400), dict(mode=BS, n_s=1)),             # a single channel: every block works on it
    ((5, 3, 333, 17), dict(mode=FS, patch_h=100, patch_w=5, fs_per_channel=1)),   # odd plane size, scalar path
], ids=lambda v: "x".join(map(str, v)) if isinstance(v, tuple) else None)
def test_extents_at_the_edges_of_the_supported_range(shape, mkw):
    N, C_, H, W = shape
    wl = Workload(name="edge", N=N, C=C_, H=H, W=W, data_seed=77, sampling_seed=5, layer_id=9, epoch=1, **mkw)
    inp, res = _run(wl)
    assert (res["boxes"] == oracle_boxes(wl)).all()
    assert_parity(res, oracle_reference(wl, inp), wl, what=f"edge {shape}", inp=inp)


def test_degenerate_subsets():
    """One sampled point per channel (Var = 0, inv-std = 1/sqrt(eps)); constant input; ratio 1 via BS and FS."""
    wl = Workload(name="one_point", N=4, C=5, H=6, W=6, mode=FS, patch_h=1, patch_w=1, sampling_seed=3)
    inp = workloads.make_inputs(wl)
    one = wl.replace(N=1)
    inp1 = {k: (v[:1] if v.ndim == 4 else v) for k, v in inp.items()}
    _, res = _run(one, inp1)
    assert_parity(res, oracle_reference(one, inp1), one, what="s = 1", inp=inp1)
    np.testing.assert_allclose(res["save_invstd"], 1 / np.sqrt(np.float32(1e-5)), rtol=1e-6)
    const = dict(inp)
    const["x"] = np.full_like(inp["x"], 3.25)
    _, res = _run(wl, const)
    assert_parity(res, oracle_reference(wl, const), wl, what="constant x")
    for kw in (dict(mode=BS, n_s=4), dict(mode=FS, patch_h=6, patch_w=6), dict(mode=NS, n_s=4)):
        full = Workload(name="ratio1", N=4, C=5, H=6, W=6, sampling_seed=9, **kw)
        _, r1 = _run(full, inp)
        _, r0 = _run(full.replace(mode=FULL, n_s=0, patch_h=0, patch_w=0), inp)
        assert_parity(r1, oracle_reference(full, inp), full, what="ratio 1")
        for k in ("y", "dx", "dgamma", "dbeta", "save_mean", "save_invstd"):
            np.testing.assert_allclose(r1[k], r0[k], rtol=2e-6, atol=2e-6)


def test_large_mean_small_spread_keeps_variance_accurate():
    """|mean| = 1e3 std: the shifted sums must not cancel, so inv-std keeps fp32 accuracy.
    y itself cannot: save_mean is an fp32 output, and rounding it moves every x^ by up to
    2^-24 |mean| invstd, which bounds what any fp32 implementation of this interface reaches."""
    wl = Workload(name="offset", N=16, C=8, H=16, W=16, mode=BS, n_s=4, sampling_seed=2)
    inp = workloads.make_inputs(wl)
    inp["x"] = (inp["x"] * 1e-2 + 10.0).astype(np.float32)
    _, res = _run(wl, inp)
    ref = oracle_reference(wl, inp)
    for k in ("save_mean", "save_invstd", "running_mean", "running_var", "dbeta"):
        assert scaled_err(res[k], ref[k]) <= 1e-5, k
    cond = float(np.max(np.abs(ref["save_mean"]) * ref["save_invstd"]))          # ~1e3
    assert cond > 300
    for k in ("y", "dx", "dgamma"):
        assert scaled_err(res[k], ref[k]) <= 4 * 2.0 ** -24 * cond, k


# ---------------------------------------------------------------------------------------
# the benchmark configurations
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("name", ["tiny_bs", "cifar_fs", "vdn", "micro_a_fs", "micro_a_full", "micro_b_fs",
                                  "micro_b_full"])
def test_benchmark_configs_full_tensor(name):
    wl = workloads.WORKLOADS[name]
    inp, res = _run(wl)
    assert (res["boxes"] == oracle_boxes(wl)).all()
    ref = oracle_reference(wl, inp)
    errs = assert_parity(res, ref, wl, what=name, inp=inp)
    plain = assert_parity(res, ref, wl, what=name, floors=False)       # |got - ref| / (|ref| + RMS) alone
    _announce(f"{name} scaled errors with floors {errs}")
    _announce(f"{name} scaled errors without   {plain}")


def test_cifar_fs_per_channel_patches():
    wl = workloads.WORKLOADS["cifar_fs"].replace(fs_per_channel=1, N=32)
    inp, res = _run(wl)
    assert len({tuple(b) for b in res["boxes"]}) > 20
    assert_parity(res, oracle_reference(wl, inp), wl, what="cifar_fs per-channel")


@pytest.fixture(scope="module")
def imagenet_inputs():
    wl = workloads.WORKLOADS["imagenet_bs"]
    _announce("generating 64x256x56x56 inputs")
    return workloads.make_inputs(wl)


@pytest.mark.parametrize("name", ["imagenet_bs", "imagenet_fs", "imagenet_full", "imagenet_bs_bf16",
                                  "imagenet_fs_bf16", "imagenet_full_bf16"])
def test_imagenet_shape_all_channels(name, imagenet_inputs):
    """Full 64x256x56x56 tensor in the launch configuration the benchmark times; the oracle
    evaluates every channel (a channel is independent of the others)."""
    wl = workloads.WORKLOADS[name]
    inp = imagenet_inputs
    if wl.dtype == "bf16":
        inp = dict(inp)
        inp["x"] = workloads.round_to_bf16(inp["x"])
        inp["dy"] = workloads.round_to_bf16(inp["dy"])
    _, res = _run(wl, inp)
    assert (res["boxes"] == oracle_boxes(wl)).all()
    worst, worst_plain = {}, {}
    step = 32
    for c0 in range(0, wl.C, step):
        ch = list(range(c0, min(c0 + step, wl.C)))
        ref = oracle_reference(wl, inp, channels=ch)
        errs = assert_parity(res, ref, wl, channels=ch, what=f"{name} ch {c0}", inp=inp)
        plain = assert_parity(res, ref, wl, channels=ch, what=f"{name} ch {c0}", floors=False)
        for k, v in errs.items():
            worst[k] = max(worst.get(k, 0.0), v)
            worst_plain[k] = max(worst_plain.get(k, 0.0), plain[k])
    _announce(f"{name} worst scaled errors with floors {worst}")
    _announce(f"{name} worst scaled errors without   {worst_plain}")


@pytest.fixture(scope="module")
def stage1_inputs():
    wl = workloads.WORKLOADS["stage1_bs"]
    _announce("generating 64x64x112x112 inputs")
    return workloads.make_inputs(wl)


@pytest.mark.parametrize("name", ["stage1_bs", "stage1_fs", "stage1_full"])
def test_first_stage_shape_all_channels(name, stage1_inputs):
    """64x64x112x112, the first-stage maps of the ImageNet models (Table 1): a channel is 3.2 MB, which a team of
    several dozen blocks still holds on chip; every channel against the oracle."""
    wl = workloads.WORKLOADS[name]
    _, res = _run(wl, stage1_inputs)
    assert (res["boxes"] == oracle_boxes(wl)).all()
    worst = {}
    for c0 in range(0, wl.C, 16):
        ch = list(range(c0, min(c0 + 16, wl.C)))
        errs = assert_parity(res, oracle_reference(wl, stage1_inputs, channels=ch), wl, channels=ch, what=f"{name} ch {c0}")
        for k, v in errs.items():
            worst[k] = max(worst.get(k, 0.0), v)
    _announce(f"{name} worst scaled errors {worst}")


# ---------------------------------------------------------------------------------------
# determinism, stages, channel groups
# ---------------------------------------------------------------------------------------
def test_bit_identical_reruns_and_stage_calls(kernel_path):
    wl = workloads.WORKLOADS["cifar_fs"].replace(N=16)
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
        if kernel_path == "streaming":
            assert (a[k] == s[k]).all(), k               # the whole-call path is exactly these stages
        else:
            np.testing.assert_allclose(a[k], s[k], rtol=2e-5, atol=2e-5, err_msg=k)   # fused kernels sum in another order


def test_channel_groups_and_split_overrides_give_the_same_answer():
    wl = workloads.WORKLOADS["vdn"].replace(N=10, C=37)
    inp = workloads.make_inputs(wl)
    ref = oracle_reference(wl, inp)
    try:
        for group, ss, sr in [(0, 0, 0), (8, 0, 0), (1, 3, 5), (36, 64, 64), (37, 1, 1)]:
            bns.bns_set_option("channel_group", group)
            bns.bns_set_option("splits_stats", ss)
            bns.bns_set_option("splits_reduce", sr)
            _, res = _run(wl, inp)
            assert_parity(res, ref, wl, what=f"group {group} splits {ss}/{sr}")
    finally:
        for k in ("channel_group", "splits_stats", "splits_reduce"):
            bns.bns_set_option(k, 0)


@pytest.mark.parametrize("variant,shape,mkw", [
    (1, (16, 300, 16, 16), dict(mode=BS, n_s=4)),                      # 64-thread blocks, teams of 16, several rounds
    (1, (16, 300, 16, 16), dict(mode=FS, patch_h=5, patch_w=7)),
    (1, (17, 4, 40, 52), dict(mode=FS, patch_h=9, patch_w=13, fs_per_channel=1)),   # teams wider than a wave
    (2, (5, 7, 7, 7), dict(mode=BS, n_s=2)),                           # scalar path, unaligned planes
    (3, (64, 96, 28, 28), dict(mode=VDN, n_s=2)),
    (4, (32, 40, 56, 56), dict(mode=BS, n_s=4)),
    (5, (32, 40, 56, 56), dict(mode=FULL)),
    (7, (64, 24, 56, 56), dict(mode=FS, patch_h=14, patch_w=14)),      # 50 vectors per thread
    (5, (32, 300, 28, 28), dict(mode=BS, n_s=4)),                      # several rounds, two blocks per unit
    (4, (5, 700, 7, 7), dict(mode=BS, n_s=2)),                         # scalar path, many channels
])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_fused_kernels_every_variant(variant, shape, mkw, dtype, kernel_path):
    """Forces the single-launch kernels (and a block-size / registers-per-thread variant), including
    team sizes and round counts that the automatic choice would not pick for these shapes."""
    if kernel_path != "auto":
        pytest.skip("forced-fused test runs once")
    N, C_, H, W = shape
    wl = Workload(name=f"fused_v{variant}", N=N, C=C_, H=H, W=W, dtype=dtype, data_seed=5, sampling_seed=11,
                  layer_id=2, epoch=variant, **mkw)
    inp = workloads.make_inputs(wl)
    try:
        bns.bns_set_option("path", 2)
        bns.bns_set_option("fused_variant", variant)
        _, res = _run(wl, inp)
        again = bns.run_workload(wl, inp)
    finally:
        bns.bns_set_option("fused_variant", 0)
        bns.bns_set_option("path", 0)
    assert_parity(res, oracle_reference(wl, inp), wl, what=f"fused variant {variant} {shape} {dtype}", inp=inp)
    for k in res:
        assert (res[k] == again[k]).all(), f"{k}: fused kernels are not bit-identical from run to run"


@pytest.mark.parametrize("variant,shape,mkw", [
    (1, (16, 300, 16, 16), dict(mode=BS, n_s=4)),                      # 64-thread blocks, large teams, several rounds
    (1, (16, 300, 16, 16), dict(mode=FS, patch_h=5, patch_w=7)),
    (2, (5, 7, 7, 7), dict(mode=FULL)),                                # scalar path, unaligned planes
    (3, (64, 96, 28, 28), dict(mode=FS, patch_h=7, patch_w=9, fs_per_channel=1)),
    (4, (32, 40, 56, 56), dict(mode=FULL)),
    (4, (32, 300, 28, 28), dict(mode=VDN, n_s=3)),                     # several rounds
])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_fused_backward_with_x_kept_on_chip(variant, shape, mkw, dtype, kernel_path):
    """The backward flavour that keeps x in registers beside dy, forced for every variant it is built for
    and for location sets the automatic choice would not give it."""
    if kernel_path != "auto":
        pytest.skip("forced-fused test runs once")
    N, C_, H, W = shape
    wl = Workload(name=f"keepx_v{variant}", N=N, C=C_, H=H, W=W, dtype=dtype, data_seed=6, sampling_seed=12,
                  layer_id=3, epoch=variant, **mkw)
    inp = workloads.make_inputs(wl)
    try:
        bns.bns_set_option("path", 2)
        bns.bns_set_option("fused_variant", variant)
        bns.bns_set_option("fused_keep_x", 1)
        _, res = _run(wl, inp)
        again = bns.run_workload(wl, inp)
        bns.bns_set_option("fused_keep_x", 2)
        plain = bns.run_workload(wl, inp)
    finally:
        bns.bns_set_option("fused_keep_x", 0)
        bns.bns_set_option("fused_variant", 0)
        bns.bns_set_option("path", 0)
    assert_parity(res, oracle_reference(wl, inp), wl, what=f"keep-x variant {variant} {shape} {dtype}", inp=inp)
    for k in res:
        assert (res[k] == again[k]).all(), f"{k}: not bit-identical from run to run"
    for k in res:       # the flavour that reads x again: same function, team sizes (hence rounding order) may differ
        assert scaled_err(res[k], plain[k]) <= (2e-5 if k not in ("y", "dx") or dtype == "f32" else 1e-2), k


@pytest.mark.parametrize("shape,dtype,patch,per_channel,variant,masked", [
    ((24, 6, 56, 56), "bf16", (14, 14), 0, 6, True),    # 9408 vectors of 8 in (512 threads, 32 vectors): one block a channel
    ((24, 6, 56, 56), "bf16", (5, 3), 1, 6, True),      # a patch inside one vector, a location per channel
    ((44, 5, 56, 56), "bf16", (56, 9), 0, 7, True),     # (512, 50); every row sampled, columns masked
    ((24, 40, 56, 56), "bf16", (14, 14), 0, 7, True),   # (512, 50) with room to spare: several blocks a channel
    ((12, 7, 56, 56), "f32", (14, 14), 0, 6, True),     # vectors of 4
    ((12, 7, 56, 56), "f32", (1, 56), 1, 6, True),      # whole rows: every vector of a sampled row unmasked
    ((30, 5, 10, 60), "bf16", (3, 7), 0, 6, False),     # rows of 7.5 vectors: the patch elements are read on their own
    ((24, 6, 56, 56), "bf16", (14, 14), 0, 5, False),   # a variant the flavour is not built for
])
def test_patch_statistics_from_the_registers(shape, dtype, patch, per_channel, variant, masked, kernel_path):
    """Feature Sampling forward where one block holds a channel: the statistics come from the vectors in registers under
    a column mask (when a row is a whole number of vectors).  Against the oracle, and against the flavour that reads
    the patch elements on their own."""
    if kernel_path != "auto":
        pytest.skip("forced-fused test runs once")
    N, C_, H, W = shape
    wl = Workload(name="patch_mask", N=N, C=C_, H=H, W=W, dtype=dtype, mode=FS, patch_h=patch[0], patch_w=patch[1],
                  fs_per_channel=per_channel, data_seed=21, sampling_seed=22, layer_id=2, epoch=5)
    inp = workloads.make_inputs(wl)
    try:
        bns.bns_set_option("path", 2)
        bns.bns_set_option("fused_variant", variant)    # (few channels: the planner would take smaller blocks)
        bns.bns_set_option("fused_patch_mask", 1)
        _, res = _run(wl, inp)
        flavour = bns.bns_get_option("last_fused_forward")
        bns.bns_set_option("fused_patch_mask", 2)
        other = bns.run_workload(wl, inp)
        assert bns.bns_get_option("last_fused_forward") == 1
    finally:
        bns.bns_set_option("fused_patch_mask", 0)
        bns.bns_set_option("fused_variant", 0)
        bns.bns_set_option("path", 0)
    assert flavour == (2 if masked else 1)
    ref = oracle_reference(wl, inp)
    assert_parity(res, ref, wl, what=f"patch from registers {shape} {dtype} {patch}", inp=inp)
    assert_parity(other, ref, wl, what=f"patch read on its own {shape} {dtype} {patch}", inp=inp)


def test_missing_team_mate_ends_in_nan_not_in_a_hang(kernel_path):
    """The give-up path of the single-launch kernels, forced from the host: with publishing switched off every
    wait for a team-mate's sums expires after `test_spin_limit` polls.  The sums are then NaN (never a finite
    wrong value), the kernels end normally, and the next ordinary call on the same buffers and workspace is right."""
    if kernel_path != "auto":
        pytest.skip("forced-fused test runs once")
    wl = Workload(name="give_up", N=16, C=300, H=16, W=16, dtype="f32", mode=BS, n_s=4, data_seed=9, sampling_seed=15,
                  layer_id=1, epoch=0)
    inp = workloads.make_inputs(wl)
    buf = bns.Buffers(wl, inp)

    def forward_backward():
        bns.bns_forward(buf.shape, buf.spec, buf.seed, buf.x, buf.gamma, buf.beta, wl.eps, wl.momentum, buf.y,
                        buf.save_mean, buf.save_invstd, buf.running_mean, buf.running_var, buf.workspace)
        bns.bns_backward(buf.shape, buf.spec, buf.seed, buf.x, buf.dy, buf.gamma, buf.save_mean, buf.save_invstd, buf.dx,
                         buf.dgamma, buf.dbeta, buf.workspace)
        torch.cuda.synchronize()
        return buf.results()

    try:
        bns.bns_set_option("path", 2)
        bns.bns_set_option("fused_variant", 1)           # 64-thread blocks: a channel takes a team of 16
        bns.bns_set_option("test_spin_limit", 64)
        bns.bns_set_option("test_mute_exchange", 1)
        _announce("give-up path: no block publishes, 64 polls per wait")
        bad = forward_backward()
        expired_bad = bns.bns_expired_waits(buf.workspace)      # reads the count and clears it
        bns.bns_set_option("test_mute_exchange", 0)
        bns.bns_set_option("test_spin_limit", 0)
        good = forward_backward()
        expired_good = bns.bns_expired_waits(buf.workspace)
    finally:
        for name in ("test_mute_exchange", "test_spin_limit", "fused_variant", "path"):
            bns.bns_set_option(name, 0)
    for k in ("y", "save_mean", "save_invstd", "dx", "dgamma", "dbeta"):
        assert np.isnan(bad[k]).all(), f"{k}: finite values after a wait that expired"
    for k in ("running_mean", "running_var"):           # the moving averages keep their values
        assert np.array_equal(bad[k], inp[k].astype(np.float32)), f"{k} changed although the statistics were lost"
    assert expired_bad > 0 and expired_good == 0, (expired_bad, expired_good)
    assert_parity(good, oracle_reference(wl, inp), wl, what="after the give-up run", inp=inp)


def test_missing_team_mate_in_the_pipelined_backward_kernel(kernel_path):
    """The same for the backward kernel that works on two channels at a time, with teams of four blocks forced."""
    if kernel_path != "auto":
        pytest.skip("forced-fused test runs once")
    wl = Workload(name="give_up_pipe", N=24, C=40, H=32, W=32, dtype="f32", mode=FS, patch_h=9, patch_w=5, data_seed=10,
                  sampling_seed=16, layer_id=2, epoch=1)
    inp = workloads.make_inputs(wl)
    buf = bns.Buffers(wl, inp)
    buf.forward()
    try:
        bns.bns_set_option("fused_pipe", 1)             # 512 threads, 4 vectors: 6144 vectors per channel take 3 blocks
        bns.bns_set_option("fused_team", 4)
        bns.bns_set_option("test_spin_limit", 64)
        bns.bns_set_option("test_mute_exchange", 1)
        _announce("give-up path of the pipelined backward kernel")
        buf.backward()
        bad = buf.results()
        expired_bad = bns.bns_expired_waits(buf.workspace)
        bns.bns_set_option("test_mute_exchange", 0)
        bns.bns_set_option("test_spin_limit", 0)
        buf.backward()
        good = buf.results()
        expired_good = bns.bns_expired_waits(buf.workspace)
        assert bns.bns_get_option("last_path_backward") == 2
    finally:
        for name in ("test_mute_exchange", "test_spin_limit", "fused_pipe", "fused_team"):
            bns.bns_set_option(name, 0)
    for k in ("dgamma", "dbeta"):
        assert np.isnan(bad[k]).all(), f"{k}: finite values after a wait that expired"
    # Eq. 6: the sums enter dx on S only (the statistics of the forward pass were fine), and there dx is NaN
    mask = oracle.subset_mask(wl.N, wl.H, wl.W, oracle_boxes(wl)[0])          # one patch location for the layer
    in_s = np.broadcast_to(mask[:, None], bad["dx"].shape)
    assert np.isnan(bad["dx"][in_s]).all() and np.isfinite(bad["dx"][~in_s]).all()
    assert expired_bad > 0 and expired_good == 0, (expired_bad, expired_good)
    assert_parity(good, oracle_reference(wl, inp), wl, what="pipelined kernel after the give-up run", inp=inp)


def test_host_threads_on_their_own_streams_with_the_streaming_kernels():
    """Several host threads call the library at once, each on a stream of its own with buffers of its own.  The
    streaming kernels have no waits between blocks, so they may share the device (the single-launch kernels
    size their grid to the whole device; include/bns.h, Concurrency)."""
    import threading
    results, errors = {}, []

    def worker(k):
        try:
            wl = Workload(name=f"thread{k}", N=6 + k, C=24 + 8 * k, H=12, W=8 + 4 * k, mode=(BS, FS, NS, FULL)[k % 4], n_s=2,
                          patch_h=5, patch_w=3, dtype=("f32", "bf16")[k % 2], layout=("nchw", "nhwc")[(k // 2) % 2],
                          data_seed=60 + k, sampling_seed=70 + k, layer_id=k, epoch=1)
            inp = workloads.make_inputs(wl)
            with torch.cuda.stream(torch.cuda.Stream()):
                for _ in range(25):
                    res = bns.run_workload(wl, inp)
            results[k] = (wl, inp, res)
        except Exception as e:          # noqa: BLE001  (reported below, in the main thread)
            errors.append((k, repr(e)))

    bns.bns_set_option("path", 1)
    try:
        threads = [threading.Thread(target=worker, args=(k,)) for k in range(8)]
        for t in threads:
            t.start()
        for t in threads:
            t.join()
    finally:
        bns.bns_set_option("path", 0)
    assert not errors, errors
    assert len(results) == 8
    for k, (wl, inp, res) in sorted(results.items()):
        assert_parity(res, oracle_reference(wl, inp), wl, what=f"thread {k} {wl}", inp=inp)


def test_single_launch_kernels_from_several_threads_and_streams(kernel_path):
    """Several host threads, each on a stream of its own, call the single-launch kernels at once.  Blocks of such
    a kernel wait for each other, so two of them must not share the device; the library chains them with an event
    (include/bns.h, Concurrency).  Every result is right, no wait runs out."""
    if kernel_path != "auto":
        pytest.skip("single-launch kernels only")
    import threading
    results, errors = {}, []

    def worker(k):
        try:
            wl = Workload(name=f"overlap{k}", N=64, C=96, H=28, W=28, mode=(BS, FS)[k % 2], n_s=8, patch_h=7, patch_w=7,
                          dtype=("f32", "bf16")[(k // 2) % 2], data_seed=80 + k, sampling_seed=90 + k, layer_id=k, epoch=2)
            inp = workloads.make_inputs(wl)
            with torch.cuda.stream(torch.cuda.Stream()):
                buf = bns.Buffers(wl, inp)
                for _ in range(8):
                    buf.forward()
                    buf.backward()
                res = buf.results()
                expired = bns.bns_expired_waits(buf.workspace)
            results[k] = (wl, inp, res, expired)
        except Exception as e:          # noqa: BLE001  (reported below, in the main thread)
            errors.append((k, repr(e)))

    bns.bns_set_option("path", 2)
    bns.bns_set_option("test_spin_limit", 1 << 16)          # a wait that ran out would cost tens of milliseconds
    try:
        threads = [threading.Thread(target=worker, args=(k,)) for k in range(4)]
        for t in threads:
            t.start()
        for t in threads:
            t.join()
    finally:
        bns.bns_set_option("test_spin_limit", 0)
        bns.bns_set_option("path", 0)
    assert not errors, errors
    assert len(results) == 4
    for k, (wl, inp, res, expired) in sorted(results.items()):
        assert expired == 0, f"thread {k}: {expired} waits ran out"
        ref = oracle_reference(wl, inp)
        ref.pop("running_mean"), ref.pop("running_var")          # eight iterations went into them
        assert_parity({n: v for n, v in res.items() if n in ref}, ref, wl, what=f"overlap {k} {wl}", inp=inp)


def test_running_statistics_over_iterations_and_null_running_buffers():
    wl = workloads.WORKLOADS["tiny_bs"]
    inp = workloads.make_inputs(wl)
    buf = bns.Buffers(wl, inp)
    boxes = oracle_boxes(wl)
    rm, rv = inp["running_mean"].astype(np.float64), inp["running_var"].astype(np.float64)
    for it in range(4):
        mom = bns.bns_moving_average_weight(it + 1, wl.momentum)   # Eq. 8: the first iteration copies
        bns.bns_forward(buf.shape, buf.spec, buf.seed, buf.x, buf.gamma, buf.beta, wl.eps, mom, buf.y, buf.save_mean,
                        buf.save_invstd, buf.running_mean, buf.running_var, buf.workspace)
        f = oracle.forward(inp["x"], inp["gamma"], inp["beta"], boxes, wl.eps,
                           oracle.moving_average_weight(it + 1, wl.momentum), rm, rv)
        rm, rv = f["running_mean"], f["running_var"]
    r = buf.results()
    np.testing.assert_allclose(r["running_mean"], rm, rtol=1e-5, atol=1e-6)
    np.testing.assert_allclose(r["running_var"], rv, rtol=1e-5, atol=1e-6)
    before = buf.running_mean.clone()
    bns.bns_forward(buf.shape, buf.spec, buf.seed, buf.x, buf.gamma, buf.beta, wl.eps, 0.1, buf.y, buf.save_mean,
                    buf.save_invstd, None, None, buf.workspace)
    torch.cuda.synchronize()
    assert torch.equal(before, buf.running_mean)


def test_bf16_stores_round_to_nearest_even():
    """The bf16 path does the same fp32 arithmetic as the fp32 path on the same (bf16-representable)
    inputs, so its outputs must be the fp32 outputs rounded to nearest-even: bit-equal almost
    everywhere, and never more than one bf16 step apart (the statistics are summed in a different
    order, which can move an fp32 result across a rounding boundary)."""
    wl16 = workloads.WORKLOADS["cifar_fs"].replace(N=8, dtype="bf16")
    inp = workloads.make_inputs(wl16)
    r16 = bns.run_workload(wl16, inp)
    r32 = bns.run_workload(wl16.replace(dtype="f32"), inp)
    for k in ("y", "dx"):
        want = torch.from_numpy(r32[k]).to(torch.bfloat16).view(torch.int16).numpy().astype(np.int32)
        got = torch.from_numpy(r16[k]).to(torch.bfloat16).view(torch.int16).numpy().astype(np.int32)
        diff = np.abs(want - got)
        assert diff.max() <= 1, k
        assert (diff == 0).mean() > 0.999, (k, (diff == 0).mean())


MIXED_MODES = [
    ("bs", dict(mode=BS, n_s=2)),
    ("ns", dict(mode=NS, n_s=1)),
    ("fs", dict(mode=FS, patch_h=3, patch_w=2)),
    ("fs_pc", dict(mode=FS, patch_h=2, patch_w=3, fs_per_channel=1)),
    ("full", dict(mode=FULL)),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("mname,mkw", MIXED_MODES, ids=[m[0] for m in MIXED_MODES])
@pytest.mark.parametrize("shape", [(6, 10, 8, 8), (5, 7, 7, 7), (9, 33, 6, 6), (12, 4, 40, 52)],
                         ids=lambda s: "x".join(map(str, s)))
def test_vdn_plus_sampling_small_shapes(shape, mname, mkw, dtype, kernel_path):
    """Eq. 4: statistics blended from the virtual samples and the sampled real samples."""
    N, C_, H, W = shape
    for n_v, mix in ((1, 0.5), (2, 0.3), (2, 1.0), (1, 0.0)):
        wl = Workload(name=f"mix_{mname}", N=N, C=C_, H=H, W=W, dtype=dtype, n_v=n_v, mix_beta=mix, data_seed=40 + n_v,
                      sampling_seed=13, layer_id=6, epoch=n_v, **mkw)
        inp, res = _run(wl)
        bv, bs = oracle_boxes_mixed(wl)
        assert (res["boxes"] == bs).all()
        assert_parity(res, oracle_reference(wl, inp), wl, what=f"mixed {shape} {mname} {dtype} n_v={n_v} beta={mix}",
                      inp=inp)


@pytest.mark.parametrize("variant,shape,mkw", [
    (1, (16, 300, 16, 16), dict(mode=BS, n_s=4)),                      # 64-thread blocks, large teams, several rounds
    (1, (16, 300, 16, 16), dict(mode=FS, patch_h=5, patch_w=7)),
    (2, (9, 36, 6, 6), dict(mode=FULL)),
    (3, (64, 96, 28, 28), dict(mode=FS, patch_h=7, patch_w=9, fs_per_channel=1)),
    (4, (32, 40, 56, 56), dict(mode=NS, n_s=5)),
    (5, (32, 300, 28, 28), dict(mode=BS, n_s=3)),                      # several rounds, two exchanges per round
    (5, (34, 24, 56, 56), dict(mode=FS, patch_h=14, patch_w=14)),
])
@pytest.mark.parametrize("keep_x", [2, 1])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_vdn_plus_sampling_fused_variants(variant, shape, mkw, dtype, keep_x, kernel_path):
    """Eq. 4 through the single-launch kernels, every variant they are built for, backward with and without x
    kept on chip (the latter exists up to variant 4)."""
    if kernel_path != "auto":
        pytest.skip("forced-fused test runs once")
    N, C_, H, W = shape
    wl = Workload(name=f"mix_fused_v{variant}", N=N, C=C_, H=H, W=W, dtype=dtype, n_v=2, mix_beta=0.5, data_seed=7,
                  sampling_seed=14, layer_id=4, epoch=variant, **mkw)
    inp = workloads.make_inputs(wl)
    try:
        bns.bns_set_option("path", 2)
        bns.bns_set_option("fused_variant", variant)
        bns.bns_set_option("fused_keep_x", keep_x)
        _, res = _run(wl, inp)
        again = bns.run_workload(wl, inp)
    finally:
        bns.bns_set_option("fused_keep_x", 0)
        bns.bns_set_option("fused_variant", 0)
        bns.bns_set_option("path", 0)
    assert_parity(res, oracle_reference(wl, inp), wl, what=f"mixed fused variant {variant} {shape} {dtype}", inp=inp)
    for k in res:
        assert (res[k] == again[k]).all(), f"{k}: not bit-identical from run to run"


@pytest.mark.parametrize("name", ["vdn_fs_mix", "vdn_bs_mix"])
def test_vdn_plus_sampling_benchmark_shape(name, kernel_path):
    wl = workloads.WORKLOADS[name]
    inp, res = _run(wl)
    want = 2 if kernel_path == "auto" else 1         # this shape fits on chip: one launch per direction by default
    assert bns.bns_get_option("last_path_forward") == want and bns.bns_get_option("last_path_backward") == want
    errs = assert_parity(res, oracle_reference(wl, inp), wl, what=name, inp=inp)
    _announce(f"{name} scaled errors {errs}")
    again = bns.run_workload(wl, inp)
    for k in res:
        assert (res[k] == again[k]).all(), k


@pytest.mark.parametrize("shape,dtype", [((6, 10, 12, 12), "f32"), ((3, 5, 7, 7), "f32"), ((8, 64, 28, 28), "bf16"),
                                         ((4, 9, 6, 6), "bf16")])
def test_inference_mode(shape, dtype, kernel_path):
    if kernel_path != "auto":
        pytest.skip("one kernel only")
    N, C_, H, W = shape
    wl = Workload(name="infer", N=N, C=C_, H=H, W=W, mode=FULL, dtype=dtype, data_seed=9)
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


@pytest.mark.parametrize("name", ["micro_a_fs", "tiny_bs", "cifar_fs", "vdn_fs_mix", "vdn_bs_mix"])
def test_hip_graph_capture_and_replay(name, kernel_path):
    """The library allocates nothing and never synchronises, so a forward + backward can be captured
    into a HIP graph.  Every replay is checked against the eager result, with eager work and
    synchronisation between replays."""
    wl = workloads.WORKLOADS[name]
    if name == "cifar_fs":
        wl = wl.replace(N=16)
    if name.startswith("vdn_"):                         # Eq. 4: bns_forward_mixed / bns_backward_mixed
        wl = wl.replace(C=32)
    inp = workloads.make_inputs(wl)
    eager = bns.run_workload(wl, inp)
    eager_paths = (bns.bns_get_option("last_path_forward"), bns.bns_get_option("last_path_backward"))
    buf = bns.Buffers(wl, inp)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        buf.forward()                                   # warm-up outside capture (first-use queries)
        buf.backward()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    buf.running_mean.copy_(torch.from_numpy(inp["running_mean"]))
    buf.running_var.copy_(torch.from_numpy(inp["running_var"]))
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        buf.forward()
        buf.backward()
    # the same kernels are recorded as run eagerly, teams of several blocks included
    assert (bns.bns_get_option("last_path_forward"), bns.bns_get_option("last_path_backward")) == eager_paths
    for replay in range(4):
        buf.running_mean.copy_(torch.from_numpy(inp["running_mean"]))
        buf.running_var.copy_(torch.from_numpy(inp["running_var"]))
        buf.y.fill_(float("nan"))                       # eager work between replays
        buf.dx.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        got = buf.results()
        first = got if replay == 0 else first
        for k in eager:
            assert (got[k] == eager[k]).all(), f"replay {replay}: {k} differs from the eager result"
            assert (got[k] == first[k]).all(), f"replay {replay}: {k} differs from the first replay"
    assert bns.bns_expired_waits(buf.workspace) == 0


def test_copy_reference():
    src = torch.arange(0, 1 << 20, dtype=torch.int32, device="cuda:0")
    for n in (4, 1024, 4096 + 4, 1 << 20):
        dst = torch.zeros(n, dtype=torch.int32, device="cuda:0")
        bns.bns_copy_reference(dst, src[:n])
        torch.cuda.synchronize()
        assert torch.equal(dst, src[:n])
