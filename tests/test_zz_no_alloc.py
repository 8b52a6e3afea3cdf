"""bns_backward_builtin_workspace (the entry point that takes no workspace and allocates nothing) against
bns_backward, through the C ABI: two calls in a row on the library's built-in scratch memory, the second on
a smaller input, each compared bit for bit with bns_backward on a caller-provided workspace and with the
oracle.  Runs with the default kernel choice (single-launch kernels: exchange slots in the scratch memory)
and with the streaming kernels forced (partial sums in the scratch memory)."""
import numpy as np
import pytest
import torch

from paper_1810_10962_amd import bns
from paper_1810_10962_amd.workloads import BS, FS, Workload, make_inputs
from parity import assert_parity, oracle_reference

pytestmark = pytest.mark.gpu

CASES = [
    # (first call, second call on a smaller input)
    (Workload(name="noalloc_a", N=24, C=96, H=28, W=28, mode=BS, n_s=3, data_seed=11, sampling_seed=5, layer_id=2),
     Workload(name="noalloc_b", N=6, C=40, H=14, W=14, mode=FS, patch_h=5, patch_w=4, data_seed=12, sampling_seed=6,
              layer_id=1, epoch=3)),
    (Workload(name="noalloc_c", N=16, C=64, H=20, W=20, mode=FS, patch_h=6, patch_w=6, dtype="bf16", data_seed=13,
              sampling_seed=7),
     Workload(name="noalloc_d", N=5, C=7, H=7, W=7, mode=BS, n_s=2, dtype="bf16", data_seed=14, sampling_seed=8)),
]


def _one_call(wl):
    inp = make_inputs(wl)
    b = bns.Buffers(wl, inp)
    b.forward()
    b.backward()                                        # bns_backward on the caller's workspace
    want = b.results()
    for name in ("dx", "dgamma", "dbeta"):
        getattr(b, name).fill_(float("nan"))
    print(f"[gpu-case] bns_backward_builtin_workspace {wl.name} {wl.shape} {wl.dtype} mode={wl.mode}", flush=True)
    bns.bns_backward_builtin_workspace(b.shape, b.spec, b.seed, b.x, b.dy, b.gamma, b.save_mean, b.save_invstd,
                                       b.dx, b.dgamma, b.dbeta)
    got = b.results()
    for name in ("dx", "dgamma", "dbeta"):
        assert np.array_equal(got[name], want[name]), f"{wl.name} {name}: differs from bns_backward"
    assert_parity(got, oracle_reference(wl, inp), wl, what=wl.name, inp=inp)
    assert bns.bns_expired_waits(None, stream_of=b.x) == 0        # the count kept in the built-in scratch


@pytest.mark.parametrize("path", [0, 1], ids=["auto", "streaming"])
@pytest.mark.parametrize("case", range(len(CASES)))
def test_builtin_workspace_matches_bns_backward_twice_in_a_row(case, path):
    bns.bns_set_option("path", path)
    try:
        first, second = CASES[case]
        _one_call(first)
        _one_call(second)
    finally:
        bns.bns_set_option("path", 0)


def test_builtin_workspace_rejects_what_does_not_fit():
    # the built-in scratch holds the workspace of at most 3840 channels (N x C x H x W); nothing is launched
    shape = bns.make_shape(2, 5000, 2, 2)
    spec = bns.make_spec(BS, 1)
    assert bns.bns_workspace_bytes(shape, spec) > (4 << 20) + 256
    t = torch.zeros(2 * 5000 * 2 * 2, device="cuda")
    v = torch.zeros(5000, device="cuda")
    with pytest.raises(bns.BnsError) as e:
        bns.bns_backward_builtin_workspace(shape, spec, 1, t, t.clone(), v, v, v, t.clone(), v.clone(), v.clone())
    assert e.value.status == bns.BNS_EWORKSPACE
