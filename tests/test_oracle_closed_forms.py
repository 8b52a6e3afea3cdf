"""The oracle's ratio / cost helpers against the numbers the paper prints."""
import pytest

from conftest import read_golden
from oracle import bns_oracle as o


def _pct(x, digits):
    return round(100.0 * x, digits)


def test_sampling_ratio_labels():
    g = read_golden("paper_closed_forms.txt")
    N, H, W = 128, 32, 32
    bs = o.sample_index(N, 1, H, W, o.BS, n_s=4, seed=1)[0]
    assert _pct(o.sampling_ratio(N, H, W, bs), 1) == float(g["bs_4_of_128_percent"])
    vdn = o.sample_index(N, 1, H, W, o.VDN, n_s=1)[0]
    assert _pct(o.sampling_ratio(N, H, W, vdn), 1) == float(g["vdn_1_of_128_percent"])
    assert _pct(o.sampling_ratio(N, H, W, vdn), 2) == float(g["ratio_1_of_128_percent"])
    vdn2 = o.sample_index(N, 1, H, W, o.VDN, n_s=2)[0]
    assert _pct(o.sampling_ratio(N, H, W, vdn2), 1) == float(g["ratio_2_of_128_percent"])
    fs32 = o.sample_index(N, 1, H, W, o.FS, patch_h=8, patch_w=4, seed=1)[0]      # 32 of 1024 points
    assert _pct(o.sampling_ratio(N, H, W, fs32), 1) == float(g["fs_1_of_32_percent"])
    fs64 = o.sample_index(N, 1, H, W, o.FS, patch_h=4, patch_w=4, seed=1)[0]
    assert _pct(o.sampling_ratio(N, H, W, fs64), 1) == float(g["ratio_1_of_64_percent"])
    d = o.sample_index(64, 1, H, W, o.NS, n_s=3)[0]
    assert _pct(o.sampling_ratio(64, H, W, d), 1) == float(g["ratio_3_of_64_percent"])


def test_adder_tree_speedup_and_visited_fraction():
    g = read_golden("paper_closed_forms.txt")
    m = int(g["adder_tree_m"])
    s = m // int(g["adder_tree_ratio_den"])
    assert m == 56 * 56 * 128
    speedup = o.adder_tree_speedup(m, s)
    assert round(100 * (speedup - 1), 1) == float(g["adder_tree_speedup_percent"])
    assert _pct(o.statistics_traffic_fraction(m, s), 1) == float(g["visited_percent"])
