"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer, on a machine without a GPU.

Two programs under tests/host_checks/ are built here and run as child processes:

* index_harness (g++ -fsanitize=address,undefined): the sampling-index generator and the shape / spec validation,
  which are plain C++ headers.  It rebuilds the boxes of more than 10^5 random tuples, which are then compared
  with the oracle's, and pushes every combination of extreme extents, enums and counts through the validation.
* api_harness: the real extern "C" entry points, from bns_api.hip compiled with hipcc with the sanitizers on the
  host side only (the kernels come from the built libbns.so), called a few thousand times with one bad argument
  each, plus the host-only functions with exactly sized buffers.

A sanitizer report ends the child with a non-zero status (-fno-sanitize-recover), which fails the test.
"""
import os
import shutil
import subprocess

import numpy as np
import pytest

import oracle.bns_oracle as o

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CHECKS = os.path.join(ROOT, "tests", "host_checks")
PKG = os.path.join(ROOT, "paper_1810_10962_amd")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


def _run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert r.returncode == 0, f"{' '.join(cmd)}\nexit {r.returncode}\n{r.stdout[-3000:]}\n{r.stderr[-6000:]}"
    return r.stdout


@pytest.fixture(scope="module")
def index_harness(tmp_path_factory):
    gxx = shutil.which("g++")
    if not gxx:
        pytest.skip("g++ not found")
    exe = str(tmp_path_factory.mktemp("san") / "index_harness")
    _run([gxx, "-std=c++17", "-O1", "-g", "-Wall", "-Werror", *SAN, os.path.join(CHECKS, "index_harness.cpp"), "-o", exe])
    return exe


def test_validation_and_index_survive_extreme_arguments_under_sanitizers(index_harness):
    out = _run([index_harness, "extremes"], env=ENV)
    accepted, rejected = (int(v) for v in out.split()[1::2])
    assert accepted > 10 ** 6 and rejected > 10 ** 7


def _random_tuples(rng, count):
    """int64 [count, 13]: N, C, H, W, mode, n_s, patch_h, patch_w, fs_per_channel, layer_id, epoch, seed, n_v."""
    t = np.zeros((count, 13), dtype=np.int64)
    t[:, 0] = rng.integers(2, 70, count)                                  # N (at least one virtual + one real sample)
    t[:, 1] = rng.integers(1, 5, count)
    t[:, 2] = rng.integers(1, 70, count)
    t[:, 3] = rng.integers(1, 70, count)
    mixed = rng.integers(0, 4, count) == 0
    t[:, 12] = np.where(mixed, rng.integers(1, 1 << 30, count) % (t[:, 0] - 1) + 1, 0)     # n_v in [1, N - 1]
    real = t[:, 0] - t[:, 12]
    t[:, 4] = np.where(mixed, rng.integers(0, 4, count), rng.integers(0, 5, count))         # no VDN inside the mix
    vdn = t[:, 4] == o.VDN
    t[:, 5] = np.where(vdn, rng.integers(0, 1 << 30, count) % (real - 1).clip(1) + 1,
                       rng.integers(0, 1 << 30, count) % real + 1)                           # n_s in [1, N] ([1, N) for VDN)
    t[:, 6] = rng.integers(0, 1 << 30, count) % t[:, 2] + 1
    t[:, 7] = rng.integers(0, 1 << 30, count) % t[:, 3] + 1
    t[:, 8] = rng.integers(0, 2, count)
    t[:, 9] = rng.integers(0, 1 << 32, count)
    t[:, 10] = rng.integers(0, 1 << 32, count)
    t[:, 11] = rng.integers(-(1 << 63), (1 << 63) - 1, count, dtype=np.int64)               # the seed's 64 bits
    return t


def test_index_sweep_under_sanitizers_equals_the_oracle(index_harness, tmp_path):
    count = 120000
    t = _random_tuples(np.random.default_rng(7), count)
    src, dst = str(tmp_path / "tuples.bin"), str(tmp_path / "boxes.bin")
    t.tofile(src)
    assert _run([index_harness, "sweep", src, dst], env=ENV).split() == ["records", str(count)]
    got = np.fromfile(dst, dtype=np.int32).reshape(count, 1 + 4 * 6)
    assert (got[:, 0] == 0).all(), "every generated tuple is a valid one"
    modes_seen = set()
    for row, g in zip(t.tolist(), got):
        N, C_, H, W, mode, n_s, ph, pw, pc, layer, epoch, seed, n_v = row
        kw = dict(n_s=n_s, patch_h=ph, patch_w=pw, fs_per_channel=pc, seed=seed % (1 << 64), layer_id=layer, epoch=epoch)
        ref = o.sample_index_mixed(N, C_, H, W, mode, n_v, **kw)[1] if n_v else o.sample_index(N, C_, H, W, mode, **kw)
        assert (g[1:1 + 6 * C_].reshape(C_, 6) == ref).all(), row
        modes_seen.add((mode, bool(n_v)))
    assert len(modes_seen) == 9


def test_entry_points_reject_bad_arguments_under_sanitizers(tmp_path):
    hipcc = next((c for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", shutil.which("hipcc")) if c and os.path.exists(c)), None)
    clang = "/opt/rocm/lib/llvm/bin/clang++"
    lib = os.path.join(PKG, "libbns.so")
    if not hipcc or not os.path.exists(clang):
        pytest.skip("hipcc / its clang++ not found")
    assert os.path.exists(lib), "libbns.so is not built: run __graft_entry__.build() first"
    api_o, har_o, exe = (str(tmp_path / n) for n in ("bns_api_san.o", "api_harness.o", "api_harness"))
    host_san = [f for s in SAN for f in ("-Xarch_host", s)]
    _run([hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", "-fno-gpu-rdc", "-Xclang", "-target-feature",
          "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument", *host_san, "-c",
          os.path.join(PKG, "csrc", "bns_api.hip"), "-o", api_o])
    _run([clang, "-std=c++17", "-O1", "-g", "-Wall", "-Werror", *SAN, "-c", os.path.join(CHECKS, "api_harness.cpp"), "-o", har_o])
    # the harness's own bns_api object comes first, so its (instrumented) entry points are the ones called;
    # the kernels and their launchers come from the library
    _run([hipcc, "--offload-arch=gfx950", "-fno-gpu-rdc", *SAN, har_o, api_o, "-L" + PKG, "-lbns", "-Wl,-rpath," + PKG, "-o", exe])
    out = _run([exe], env=ENV).split()
    assert out[0] == "calls" and int(out[1]) > 3000 and out[2:] == ["failures", "0"]
