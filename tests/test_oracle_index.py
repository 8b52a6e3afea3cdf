"""Pins for the oracle's sampling-index generator and location sets (Alg. 1-3).

None of these re-types the oracle's formula: they check it against a published
test vector, against brute-force enumeration of the definitions in the
algorithms, and against the properties the algorithms demand.
"""
import itertools

import numpy as np
import pytest

from conftest import read_golden
from oracle import bns_oracle as o


def test_mix64_matches_published_splitmix64_vector():
    g = read_golden("splitmix64_seed1234567.txt")
    state = 1234567
    for k in range(1, 6):
        state = (state + 0x9E3779B97F4A7C15) % (1 << 64)
        assert o.mix64(state) == int(g[f"out{k}"])


def test_hash_depends_on_every_argument():
    base = (7, 3, 2, 1, 5)
    h0 = o.index_hash(*base)
    assert 0 <= h0 < (1 << 64)
    for pos in range(5):
        args = list(base)
        args[pos] += 1
        assert o.index_hash(*args) != h0
    # layer and epoch must not be interchangeable (they share one 64-bit word)
    assert o.index_hash(7, 3, 2, 1, 5) != o.index_hash(7, 2, 3, 1, 5)
    assert o.index_hash(7, 3, 2, 1, 5) != o.index_hash(7, 3, 2, 5, 1)


@pytest.mark.parametrize("K", [0, 1, 2, 6, 42, 255])
def test_randint_is_inclusive_and_reaches_both_ends(K):
    seen = set()
    for seed in range(4000):
        v = o.randint(0, K, seed, 1, 0, 1, 0xFFFFFFFF)
        assert 0 <= v <= K
        seen.add(v)
    assert 0 in seen and K in seen                     # Alg. 1: begin = N - n_s must be reachable
    if K <= 42:
        assert seen == set(range(K + 1))


def test_randint_is_close_to_uniform():
    K = 6                                               # N - n_s for 2 of 8 samples
    n = 70000
    counts = np.zeros(K + 1)
    for epoch in range(n):
        counts[o.randint(0, K, 12345, 4, epoch, 1, 0xFFFFFFFF)] += 1
    expect = n / (K + 1)
    chi2 = ((counts - expect) ** 2 / expect).sum()
    assert chi2 < 30.0                                  # 6 dof: P(chi2 > 30) < 1e-4


def test_ns_vdn_start_at_zero_and_full_batch_has_one_outcome():
    N, C, H, W = 8, 4, 6, 5
    for seed in range(50):
        for mode in (o.NS, o.VDN):
            b = o.sample_index(N, C, H, W, mode, n_s=3, seed=seed, layer_id=seed, epoch=seed)
            assert (b == np.array([0, 3, 0, H, 0, W])).all()
        b = o.sample_index(N, C, H, W, o.BS, n_s=N, seed=seed)
        assert (b == np.array([0, N, 0, H, 0, W])).all()        # randint(0, 0) = 0
        b = o.sample_index(N, C, H, W, o.FS, patch_h=H, patch_w=W, seed=seed)
        assert (b == np.array([0, N, 0, H, 0, W])).all()
        b = o.sample_index(N, C, H, W, o.FULL, seed=seed)
        assert (b == np.array([0, N, 0, H, 0, W])).all()


def test_bs_shared_across_channels_fs_shared_or_independent():
    N, C, H, W = 16, 32, 12, 12
    b = o.sample_index(N, C, H, W, o.BS, n_s=4, seed=9, layer_id=2, epoch=1)
    assert (b == b[0]).all()                                    # rule (2): shared by channels
    f = o.sample_index(N, C, H, W, o.FS, patch_h=3, patch_w=5, seed=9, layer_id=2, epoch=1)
    assert (f == f[0]).all()                                    # rule (3): shared by channels
    fpc = o.sample_index(N, C, H, W, o.FS, patch_h=3, patch_w=5, fs_per_channel=1,
                         seed=9, layer_id=2, epoch=1)
    assert len({tuple(r) for r in fpc}) > 8                     # independent per feature map
    assert ((fpc[:, 2] >= 0) & (fpc[:, 2] + 3 <= H) & (fpc[:, 4] >= 0) & (fpc[:, 4] + 5 <= W)).all()
    # indices change with layer and with epoch (Section 4.1: refreshed once per epoch)
    starts_by_layer = {int(o.sample_index(N, C, H, W, o.BS, n_s=4, seed=9, layer_id=l)[0, 0]) for l in range(64)}
    starts_by_epoch = {int(o.sample_index(N, C, H, W, o.BS, n_s=4, seed=9, epoch=e)[0, 0]) for e in range(64)}
    assert len(starts_by_layer) > 6 and len(starts_by_epoch) > 6
    # ... and are a pure function of their arguments
    again = o.sample_index(N, C, H, W, o.BS, n_s=4, seed=9, layer_id=2, epoch=1)
    assert (again == b).all()


@pytest.mark.parametrize("mode,kw", [
    (o.FULL, {}),
    (o.NS, dict(n_s=2)),
    (o.BS, dict(n_s=2)),
    (o.BS, dict(n_s=5)),
    (o.FS, dict(patch_h=2, patch_w=3)),
    (o.FS, dict(patch_h=4, patch_w=1, fs_per_channel=1)),
    (o.VDN, dict(n_s=1)),
])
def test_location_set_by_brute_force(mode, kw):
    """S built by walking every (n, h, w) and applying the algorithms' slice bounds."""
    N, C, H, W = 5, 3, 4, 6
    for seed in range(12):
        boxes = o.sample_index(N, C, H, W, mode, seed=seed, layer_id=1, epoch=seed % 3, **kw)
        for c in range(C):
            n0, nc, h0, hc, w0, wc = (int(v) for v in boxes[c])
            # the slice of the algorithm, written as explicit Python ranges
            members = set(itertools.product(range(n0, n0 + nc), range(h0, h0 + hc), range(w0, w0 + wc)))
            assert all(0 <= n < N and 0 <= h < H and 0 <= w < W for n, h, w in members)
            mask = o.subset_mask(N, H, W, boxes[c])
            for n, h, w in itertools.product(range(N), range(H), range(W)):
                inside = (n, h, w) in members
                assert o.in_subset(boxes[c], n, h, w) == inside
                assert bool(mask[n, h, w]) == inside
            assert mask.sum() == len(members) == o.subset_size(boxes[c])
            # expected s from the algorithm's data sizes
            if mode in (o.NS, o.BS, o.VDN):
                assert o.subset_size(boxes[c]) == kw["n_s"] * H * W
            elif mode == o.FS:
                assert o.subset_size(boxes[c]) == N * kw["patch_h"] * kw["patch_w"]
            else:
                assert o.subset_size(boxes[c]) == N * H * W
            # the mask equals numpy's own slicing of an index tensor
            t = np.zeros((N, H, W), dtype=bool)
            t[n0:n0 + nc, h0:h0 + hc, w0:w0 + wc] = True
            assert (t == mask).all()
