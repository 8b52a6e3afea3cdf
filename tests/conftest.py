import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def read_golden(name):
    """Parse tests/golden/<name>: '#' comments, 'key = value' lines -> dict of str."""
    out = {}
    with open(os.path.join(ROOT, "tests", "golden", name)) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            k, v = line.split("=", 1)
            out[k.strip()] = v.strip()
    return out


GUARD_BYTES = 4096
FRONT_BYTES = 4096 + 16      # guard in front; it also puts every buffer at the least alignment the interface allows
WRITTEN_BUFFERS = ("workspace", "y", "dx", "save_mean", "save_invstd", "running_mean", "running_var", "dgamma", "dbeta",
                   "save_mean_parts")
READ_BUFFERS = ("x", "dy", "gamma", "beta")


@pytest.fixture(scope="session", autouse=True)
def guard_bytes_behind_written_buffers():
    """GPU tests: every buffer of bns.Buffers that a kernel writes (outputs, statistics, the workspace, sized
    exactly as bns_workspace_bytes says) lies between guard bytes of a known pattern, 16 bytes off any larger
    alignment, and results() fails if a kernel touched the guards; every input lies between NaNs, which a read
    outside it would carry into the outputs that the parity checks then reject."""
    try:
        import torch
        if not torch.cuda.is_available():
            yield
            return
        from paper_1810_10962_amd import bns
    except Exception:
        yield
        return
    plain_init, plain_results = bns.Buffers.__init__, bns.Buffers.results

    def init(self, *args, **kwargs):
        plain_init(self, *args, **kwargs)
        self._guards = {}
        for name in WRITTEN_BUFFERS:
            t = getattr(self, name, None)
            if t is None:
                continue
            nbytes = t.numel() * t.element_size()
            big = torch.full((FRONT_BYTES + nbytes + (-nbytes) % 16 + GUARD_BYTES,), 0xA5, dtype=torch.uint8,
                             device=t.device)
            view = big[FRONT_BYTES:FRONT_BYTES + nbytes].view(t.dtype).view(t.shape)
            view.copy_(t)
            setattr(self, name, view)
            self._guards[name] = (big, nbytes)
        for name in READ_BUFFERS:                        # inputs: NaN around them, so a read outside them shows
            t = getattr(self, name, None)
            if t is None:
                continue
            front = FRONT_BYTES // t.element_size()
            big = torch.full((front + t.numel() + GUARD_BYTES // 2,), float("nan"), dtype=t.dtype, device=t.device)
            view = big[front:front + t.numel()].view(t.shape)
            view.copy_(t)
            setattr(self, name, view)
        self._fwd_args = self._bwd_args = None          # marshalled pointers are stale

    def results(self):
        out = plain_results(self)
        for name, (big, nbytes) in self._guards.items():
            around = torch.cat([big[:FRONT_BYTES], big[FRONT_BYTES + nbytes:]])
            assert bool((around == 0xA5).all()), \
                f"{int((around != 0xA5).sum())} guard bytes around {name} were overwritten"
        return out

    bns.Buffers.__init__, bns.Buffers.results = init, results
    yield
    bns.Buffers.__init__, bns.Buffers.results = plain_init, plain_results
