"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol
include/bns.h declares, generates the same sampling index as the oracle bit for bit, and
rejects bad arguments before anything is enqueued."""
import ctypes as C

import numpy as np
import pytest

from oracle import bns_oracle as o
from paper_1810_10962_amd import bns


def test_library_loads_and_exports_every_declared_symbol():
    bns.load()
    names = bns.declared_symbols()
    assert {"bns_forward", "bns_backward", "bns_sample_index", "bns_workspace_bytes"} <= set(names)
    assert bns.missing_symbols() == []
    assert "BNS_OK" in bns.bns_status_string(0)
    for code in range(1, 5):
        assert bns.bns_status_string(code).startswith("BNS_E")


def _oracle_boxes(N, C_, H, W, mode, seed, **kw):
    return o.sample_index(N, C_, H, W, mode, seed=seed, **kw)


def test_host_index_is_bit_identical_to_the_oracle():
    """More than 10^5 random (shape, spec, seed, layer, epoch) tuples through the C ABI against the oracle."""
    rng = np.random.default_rng(0)
    checked = 0
    for _ in range(110000):
        N, H, W = (int(v) for v in rng.integers(1, 70, 3))
        C_ = int(rng.integers(1, 5))
        seed = int(rng.integers(0, 2 ** 63)) * 2 + int(rng.integers(0, 2))
        layer, epoch = int(rng.integers(0, 2 ** 32)), int(rng.integers(0, 2 ** 32))
        mode = int(rng.integers(0, 5))
        n_s = int(rng.integers(1, N + 1))
        if mode == o.VDN and N == 1:
            continue
        if mode == o.VDN:
            n_s = int(rng.integers(1, N))
        ph, pw = int(rng.integers(1, H + 1)), int(rng.integers(1, W + 1))
        pc = int(rng.integers(0, 2))
        shape = bns.make_shape(N, C_, H, W)
        spec = bns.make_spec(mode, n_s, ph, pw, pc, layer, epoch)
        got = bns.bns_sample_index(shape, spec, seed)
        ref = _oracle_boxes(N, C_, H, W, mode, seed, n_s=n_s, patch_h=ph, patch_w=pw, fs_per_channel=pc,
                            layer_id=layer, epoch=epoch)
        assert (got == ref).all(), (N, C_, H, W, mode, seed, layer, epoch, got, ref)
        checked += 1
    assert checked > 100000


def test_host_index_many_channels_and_large_extents():
    # per-channel FS over many channels, and extents near the documented limits
    shape = bns.make_shape(3, 4096, 60, 30)
    spec = bns.make_spec(bns.BNS_FS, 0, 17, 9, 1, 77, 5)
    got = bns.bns_sample_index(shape, spec, 2 ** 64 - 1)
    ref = _oracle_boxes(3, 4096, 60, 30, o.FS, 2 ** 64 - 1, patch_h=17, patch_w=9, fs_per_channel=1,
                        layer_id=77, epoch=5)
    assert (got == ref).all() and len({tuple(r) for r in got}) > 500
    for epoch in range(20):
        shape = bns.make_shape(1, 1, 60000, 30000)
        spec = bns.make_spec(bns.BNS_FS, 0, 1, 1, 0, 2 ** 32 - 1, epoch)
        got = bns.bns_sample_index(shape, spec, 2 ** 63)
        ref = _oracle_boxes(1, 1, 60000, 30000, o.FS, 2 ** 63, patch_h=1, patch_w=1, layer_id=2 ** 32 - 1, epoch=epoch)
        assert (got == ref).all()
    shape = bns.make_shape(65535, 2, 1, 1)
    got = bns.bns_sample_index(shape, bns.make_spec(bns.BNS_BS, 1, layer_id=1), 42)
    ref = _oracle_boxes(65535, 2, 1, 1, o.BS, 42, n_s=1, layer_id=1)
    assert (got == ref).all()


def _expect(status, fn, *args):
    with pytest.raises(bns.BnsError) as e:
        fn(*args)
    assert e.value.status == status


def test_invalid_shapes_and_specs_are_rejected():
    ok_shape = bns.make_shape(8, 4, 6, 6)
    bs = lambda n: bns.make_spec(bns.BNS_BS, n)
    for bad in [bns.make_shape(0, 4, 6, 6), bns.make_shape(8, -1, 6, 6), bns.make_shape(8, 4, 0, 6),
                bns.make_shape(8, 4, 6, 6, dtype=7)]:
        _expect(bns.BNS_EINVAL, bns.bns_sample_index, bad, bs(2), 0)
    for bad in [bns.make_shape(70000, 4, 6, 6), bns.make_shape(2, 4, 50000, 50000),
                bns.make_shape(2, 2 ** 25, 1, 1)]:
        _expect(bns.BNS_EUNSUPPORTED, bns.bns_sample_index, bad, bs(2), 0)
    for bad in [bs(0), bs(9), bs(-3), bns.make_spec(bns.BNS_NS, 0), bns.make_spec(bns.BNS_VDN, 8),
                bns.make_spec(bns.BNS_VDN, 0), bns.make_spec(bns.BNS_FS, 0, 0, 3), bns.make_spec(bns.BNS_FS, 0, 7, 3),
                bns.make_spec(bns.BNS_FS, 0, 3, 7), bns.make_spec(bns.BNS_FS, 0, 3, 3, fs_per_channel=2),
                bns.make_spec(9), bns.make_spec(-1)]:
        _expect(bns.BNS_EINVAL, bns.bns_sample_index, ok_shape, bad, 0)
    assert bns.bns_workspace_bytes(bns.make_shape(0, 4, 6, 6), bs(2)) == 0
    assert bns.bns_workspace_bytes(ok_shape, bs(2)) >= 4 * 2 * 4


def test_null_misaligned_overlapping_and_small_workspace_are_rejected_without_a_gpu():
    """Validation runs before any launch, so fake (never dereferenced) addresses suffice."""
    lib = bns.load()
    shape, spec = bns.make_shape(8, 4, 6, 6), bns.make_spec(bns.BNS_BS, 2)
    need = bns.bns_workspace_bytes(shape, spec)
    tb = 8 * 4 * 36 * 4
    P = lambda a: C.c_void_p(a)
    x, y, dy, dx, ws = 0x10000, 0x20000, 0x30000, 0x40000, 0x50000
    v = 0x60000                                                   # per-channel vectors

    def fwd(x=x, y=y, ws=ws, wsb=need, eps=1e-5, mom=0.1, gamma=v, sm=v + 256):
        return lib.bns_forward(C.byref(shape), C.byref(spec), 1, P(x), P(gamma), P(v + 128), C.c_float(eps),
                               C.c_float(mom), P(y), P(sm), P(v + 384), None, None, P(ws), wsb, None)

    def bwd(x=x, dy=dy, dx=dx, ws=ws, wsb=need):
        return lib.bns_backward(C.byref(shape), C.byref(spec), 1, P(x), P(dy), P(v), P(v + 128), P(v + 256),
                                P(dx), P(v + 384), P(v + 512), P(ws), wsb, None)

    assert fwd(x=0) == bns.BNS_EINVAL and fwd(y=0) == bns.BNS_EINVAL and fwd(ws=0) == bns.BNS_EINVAL
    assert fwd(gamma=0) == bns.BNS_EINVAL and fwd(sm=0) == bns.BNS_EINVAL
    assert fwd(x=x + 4) == bns.BNS_EINVAL and fwd(y=y + 8) == bns.BNS_EINVAL          # misaligned
    assert fwd(y=x) == bns.BNS_EINVAL and fwd(y=x + tb - 16) == bns.BNS_EINVAL        # overlap
    assert fwd(wsb=need - 1) == bns.BNS_EWORKSPACE
    assert fwd(eps=-1.0) == bns.BNS_EINVAL and fwd(mom=1.5) == bns.BNS_EINVAL
    assert fwd(eps=float("nan")) == bns.BNS_EINVAL
    assert bwd(x=0) == bns.BNS_EINVAL and bwd(dy=0) == bns.BNS_EINVAL and bwd(dx=0) == bns.BNS_EINVAL
    assert bwd(dx=dy) == bns.BNS_EINVAL and bwd(dx=x + 16) == bns.BNS_EINVAL
    assert bwd(wsb=0) == bns.BNS_EWORKSPACE
    assert lib.bns_forward(None, C.byref(spec), 1, P(x), P(v), P(v), 0.0, 0.0, P(y), P(v), P(v), None, None,
                           P(ws), need, None) == bns.BNS_EINVAL
    assert lib.bns_copy_reference(P(x), P(x + 8), 64, None) == bns.BNS_EINVAL
    assert lib.bns_copy_reference(P(x), P(y), 60, None) == bns.BNS_EINVAL
    assert lib.bns_copy_reference(P(x), P(x + 32), 64, None) == bns.BNS_EINVAL


def test_builtin_workspace_call_validates_before_it_touches_a_device():
    """bns_backward_builtin_workspace: bns_backward's argument checks, then the 4 MiB limit, all on the host."""
    lib = bns.load()
    shape, spec = bns.make_shape(8, 4, 6, 6), bns.make_spec(bns.BNS_BS, 2)
    P = lambda a: C.c_void_p(a)
    x, dy, dx, v = 0x10000, 0x30000, 0x40000, 0x60000

    def call(shape=shape, spec=spec, x=x, dy=dy, dx=dx, gamma=v):
        return lib.bns_backward_builtin_workspace(C.byref(shape), C.byref(spec), 1, P(x), P(dy), P(gamma), P(v + 128),
                                                  P(v + 256), P(dx), P(v + 384), P(v + 512), None)

    assert call(x=0) == bns.BNS_EINVAL and call(dx=0) == bns.BNS_EINVAL and call(gamma=0) == bns.BNS_EINVAL
    assert call(dy=dy + 4) == bns.BNS_EINVAL and call(dx=dy) == bns.BNS_EINVAL
    assert call(spec=bns.make_spec(bns.BNS_BS, 9)) == bns.BNS_EINVAL
    big = bns.make_shape(2, 3841, 2, 2)
    limit = (4 << 20) + 256                                        # 4 MiB and the workspace header
    assert bns.bns_workspace_bytes(big, spec) > limit
    assert call(shape=big, x=0x1000000, dy=0x2000000, dx=0x3000000) == bns.BNS_EWORKSPACE
    assert bns.bns_workspace_bytes(bns.make_shape(2, 3840, 2, 2), spec) <= limit


def test_expired_waits_query_validates_on_the_host():
    lib = bns.load()
    out = C.c_int32(7)
    P = lambda a: C.c_void_p(a)
    assert lib.bns_expired_waits(P(0x10000), 4096, None, None) == bns.BNS_EINVAL          # nowhere to write the count
    assert lib.bns_expired_waits(P(0x10004), 4096, None, C.byref(out)) == bns.BNS_EINVAL  # misaligned
    assert lib.bns_expired_waits(P(0x10000), 255, None, C.byref(out)) == bns.BNS_EWORKSPACE
    assert out.value == 7


def test_mixed_index_and_argument_checks():
    rng = np.random.default_rng(4)
    for _ in range(400):
        N, H, W = int(rng.integers(2, 40)), int(rng.integers(1, 30)), int(rng.integers(1, 30))
        C_ = int(rng.integers(1, 6))
        n_v = int(rng.integers(1, N))
        mode = int(rng.choice([o.FULL, o.NS, o.BS, o.FS]))
        n_s = int(rng.integers(1, N - n_v + 1))
        ph, pw, pc = int(rng.integers(1, H + 1)), int(rng.integers(1, W + 1)), int(rng.integers(0, 2))
        seed, layer, epoch = int(rng.integers(0, 2 ** 62)), int(rng.integers(0, 2 ** 32)), int(rng.integers(0, 2 ** 32))
        got = bns.bns_sample_index_mixed(bns.make_shape(N, C_, H, W), bns.make_spec(mode, n_s, ph, pw, pc, layer, epoch),
                                         seed, n_v)
        _, ref = o.sample_index_mixed(N, C_, H, W, mode, n_v, n_s=n_s, patch_h=ph, patch_w=pw, fs_per_channel=pc,
                                      seed=seed, layer_id=layer, epoch=epoch)
        assert (got == ref).all()
    shape = bns.make_shape(8, 4, 6, 6)
    _expect(bns.BNS_EINVAL, bns.bns_sample_index_mixed, shape, bns.make_spec(bns.BNS_BS, 2), 0, 0)      # no virtual sample
    _expect(bns.BNS_EINVAL, bns.bns_sample_index_mixed, shape, bns.make_spec(bns.BNS_BS, 2), 0, 8)      # no real sample
    _expect(bns.BNS_EINVAL, bns.bns_sample_index_mixed, shape, bns.make_spec(bns.BNS_BS, 7), 0, 2)      # n_s > real samples
    _expect(bns.BNS_EINVAL, bns.bns_sample_index_mixed, shape, bns.make_spec(bns.BNS_VDN, 2), 0, 2)
    lib = bns.load()
    spec = bns.make_spec(bns.BNS_BS, 2)
    P = lambda a: C.c_void_p(a)
    need = bns.bns_workspace_bytes(shape, spec)
    args = lambda n_v, mix, wsb=need, parts=0x70000: (C.byref(shape), C.byref(spec), 1, n_v, C.c_float(mix), P(0x10000),
                                                      P(0x60000), P(0x60100), C.c_float(1e-5), C.c_float(0.1),
                                                      P(0x20000), P(0x60200), P(0x60300), P(parts), None, None,
                                                      P(0x50000), wsb, None)
    assert lib.bns_forward_mixed(*args(2, 1.5)) == bns.BNS_EINVAL
    assert lib.bns_forward_mixed(*args(2, -0.1)) == bns.BNS_EINVAL
    assert lib.bns_forward_mixed(*args(0, 0.5)) == bns.BNS_EINVAL
    assert lib.bns_forward_mixed(*args(2, 0.5, parts=0)) == bns.BNS_EINVAL
    assert lib.bns_forward_mixed(*args(2, 0.5, wsb=need - 1)) == bns.BNS_EWORKSPACE


def test_options():
    assert bns.bns_get_option("splits_stats") == 0 and bns.bns_get_option("nonsense") == -1
    bns.bns_set_option("splits_reduce", 8)
    assert bns.bns_get_option("splits_reduce") == 8 and bns.bns_get_option("splits_stats") == 0
    bns.bns_set_option("splits_reduce", 0)
    _expect(bns.BNS_EINVAL, bns.bns_set_option, "splits_stats", 65)
    _expect(bns.BNS_EINVAL, bns.bns_set_option, "nonsense", 1)
    _expect(bns.BNS_EINVAL, bns.bns_set_option, "channel_group", -1)
    # every documented override reads back as it was set, 0 again after the reset, and rejects values out of range
    ranges = {"path": 2, "fused_variant": 7, "fused_coop": 1, "fused_keep_x": 2, "fused_patch_mask": 2, "test_spin_limit": 1 << 21,
              "test_mute_exchange": 1, "split_statistics": 1, "nhwc_blocks": 8192, "nhwc_split_dx": 2,
              "nhwc_ew_rows": 1 << 20, "norm_unroll": 4, "dx_unroll": 4, "reduce_unroll": 4, "norm_nt": 4, "dx_nt": 4,
              "reduce_nt": 4, "cache_reuse": 2}
    for name, hi in ranges.items():
        assert bns.bns_get_option(name) == 0, name
        for v in (1, hi):
            bns.bns_set_option(name, v)
            assert bns.bns_get_option(name) == v, name
        _expect(bns.BNS_EINVAL, bns.bns_set_option, name, hi + 1)
        bns.bns_set_option(name, 0)
        assert bns.bns_get_option(name) == 0, name
    _expect(bns.BNS_EINVAL, bns.bns_set_option, "norm_unroll", 3)


def test_layout_field_is_validated_and_nhwc_limits_are_reported():
    """N x H x W x C: same index as N x C x H x W; an unknown layout is invalid; per-channel Feature
    Sampling is refused as unsupported before anything is enqueued."""
    spec = bns.make_spec(bns.BNS_FS, 0, 3, 2, 0, 7, 1)
    a = bns.bns_sample_index(bns.make_shape(6, 5, 9, 8), spec, 99)
    b = bns.bns_sample_index(bns.make_shape(6, 5, 9, 8, layout="nhwc"), spec, 99)
    assert (a == b).all()
    bad = bns.make_shape(6, 5, 9, 8, layout=2)
    _expect(bns.BNS_EINVAL, bns.bns_sample_index, bad, spec, 99)
    assert bns.bns_workspace_bytes(bad, spec) == 0
    nhwc = bns.make_shape(64, 256, 56, 56, layout="nhwc")
    need = bns.bns_workspace_bytes(nhwc, spec)
    assert 0 < need <= 64 << 20 and need % 256 == 0
    assert bns.bns_workspace_bytes(bns.make_shape(2, 1 << 20, 2, 2, layout="nhwc"), spec) >= (1 << 20) * 8
    mixed = bns.bns_sample_index_mixed(bns.make_shape(6, 5, 9, 8, layout="nhwc"), spec, 99, 2)
    assert (mixed == bns.bns_sample_index_mixed(bns.make_shape(6, 5, 9, 8), spec, 99, 2)).all()

    # fake (never dereferenced) addresses: the refusal comes before any launch
    lib = bns.load()
    pc = bns.make_spec(bns.BNS_FS, 0, 3, 2, 1, 7, 1)
    shape = bns.make_shape(6, 8, 9, 8, layout="nhwc")
    P = lambda a: C.c_void_p(a)
    x, y, dy, dx, ws, v = 0x100000, 0x200000, 0x300000, 0x400000, 0x500000, 0x600000
    assert lib.bns_forward(C.byref(shape), C.byref(pc), 1, P(x), P(v), P(v + 128), C.c_float(1e-5), C.c_float(0.1),
                           P(y), P(v + 256), P(v + 384), None, None, P(ws), 1 << 30, None) == bns.BNS_EUNSUPPORTED
    assert lib.bns_backward(C.byref(shape), C.byref(pc), 1, P(x), P(dy), P(v), P(v + 128), P(v + 256), P(dx),
                            P(v + 384), P(v + 512), P(ws), 1 << 30, None) == bns.BNS_EUNSUPPORTED
    shared = bns.make_spec(bns.BNS_FS, 0, 3, 2, 0, 7, 1)
    assert lib.bns_forward(C.byref(shape), C.byref(shared), 1, P(x), P(v), P(v + 128), C.c_float(1e-5), C.c_float(0.1),
                           P(y), P(v + 256), P(v + 384), None, None, P(ws),
                           bns.bns_workspace_bytes(shape, shared) - 1, None) == bns.BNS_EWORKSPACE


def test_header_is_plain_c(tmp_path):
    """include/bns.h compiles as C99 with warnings as errors, and every declared function can be named from C."""
    import os
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    names = bns.declared_symbols()
    src = tmp_path / "use_bns.c"
    body = "\n".join(f"    table[{i}] = (void (*)(void)){n};" for i, n in enumerate(names))
    src.write_text('#include "bns.h"\n'
                   f"void (*table[{len(names)}])(void);\n"
                   "void fill(void) {\n" + body + "\n}\n"
                   "int sizes[3] = {sizeof(bns_shape), sizeof(bns_spec), sizeof(bns_box)};\n")
    out = subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(root, "include"),
                          "-c", str(src), "-o", str(tmp_path / "use_bns.o")], capture_output=True, text=True)
    assert out.returncode == 0, out.stderr
    # the ctypes mirrors of the structs have the C sizes
    assert C.sizeof(bns.bns_shape) == 24 and C.sizeof(bns.bns_spec) == 28 and C.sizeof(bns.bns_box) == 24


def test_moving_average_weight_is_eq8_and_matches_the_oracle():
    from oracle import bns_oracle as oracle
    assert bns.bns_moving_average_weight(1, 0.1) == 1.0                       # Eq. 8, it = 1: a copy
    assert bns.bns_moving_average_weight(0, 0.25) == 1.0                      # nothing recorded yet either
    for it in (2, 3, 1000, 2 ** 40):
        for alpha in (0.0, 0.1, 0.7, 1.0):
            got = bns.bns_moving_average_weight(it, alpha)
            assert got == np.float32(alpha) == np.float32(oracle.moving_average_weight(it, alpha))
