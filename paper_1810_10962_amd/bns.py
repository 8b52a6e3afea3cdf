"""ctypes binding of libbns.so: same names as include/bns.h, argument marshalling only.

Tensors are torch tensors on the GPU (PyTorch supplies device memory and streams);
their ``data_ptr()`` and the current HIP stream are handed to the C ABI.  Every step of
the computation runs in the library's kernels.  There is no fallback: if the shared
library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
import re

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbns.so")
HEADER_PATH = os.path.join(os.path.dirname(_HERE), "include", "bns.h")

BNS_OK, BNS_EINVAL, BNS_EUNSUPPORTED, BNS_EWORKSPACE, BNS_EDEVICE = range(5)
BNS_FULL, BNS_NS, BNS_BS, BNS_FS, BNS_VDN = range(5)
BNS_F32, BNS_BF16 = 0, 1
BNS_NCHW, BNS_NHWC = 0, 1


class bns_shape(C.Structure):
    _fields_ = [("N", C.c_int32), ("C", C.c_int32), ("H", C.c_int32), ("W", C.c_int32), ("dtype", C.c_int32),
                ("layout", C.c_int32)]


class bns_spec(C.Structure):
    _fields_ = [("mode", C.c_int32), ("n_s", C.c_int32), ("patch_h", C.c_int32), ("patch_w", C.c_int32),
                ("fs_per_channel", C.c_int32), ("layer_id", C.c_uint32), ("epoch", C.c_uint32)]


class bns_box(C.Structure):
    _fields_ = [("n0", C.c_int32), ("n_cnt", C.c_int32), ("h0", C.c_int32), ("h_cnt", C.c_int32),
                ("w0", C.c_int32), ("w_cnt", C.c_int32)]


class BnsError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = _lib.bns_status_string(status).decode() if _lib is not None else str(status)
        super().__init__(f"{where}: {msg}")


_lib = None
_P = C.c_void_p
_SHP, _SPC = C.POINTER(bns_shape), C.POINTER(bns_spec)
_PROTOS = {
    "bns_status_string": (C.c_char_p, [C.c_int]),
    "bns_sample_index": (C.c_int, [_SHP, _SPC, C.c_uint64, C.POINTER(bns_box)]),
    "bns_sample_index_device": (C.c_int, [_SHP, _SPC, C.c_uint64, _P, _P]),
    "bns_workspace_bytes": (C.c_size_t, [_SHP, _SPC]),
    "bns_forward": (C.c_int, [_SHP, _SPC, C.c_uint64, _P, _P, _P, C.c_float, C.c_float,
                              _P, _P, _P, _P, _P, _P, C.c_size_t, _P]),
    "bns_backward": (C.c_int, [_SHP, _SPC, C.c_uint64, _P, _P, _P, _P, _P, _P, _P, _P, _P, C.c_size_t, _P]),
    "bns_backward_builtin_workspace": (C.c_int, [_SHP, _SPC, C.c_uint64, _P, _P, _P, _P, _P, _P, _P, _P, _P]),
    "bns_expired_waits": (C.c_int, [_P, C.c_size_t, _P, C.POINTER(C.c_int32)]),
    "bns_forward_stats": (C.c_int, [_SHP, _SPC, C.c_uint64, _P, C.c_float, C.c_float, _P, _P, _P, _P,
                                    _P, C.c_size_t, _P]),
    "bns_forward_normalize": (C.c_int, [_SHP, _P, _P, _P, _P, _P, _P, _P]),
    "bns_backward_reduce": (C.c_int, [_SHP, _P, _P, _P, _P, _P, _P, _P, C.c_size_t, _P]),
    "bns_backward_dx": (C.c_int, [_SHP, _SPC, C.c_uint64, _P, _P, _P, _P, _P, _P, _P, _P, _P]),
    "bns_sample_index_mixed": (C.c_int, [_SHP, _SPC, C.c_uint64, C.c_int32, C.POINTER(bns_box)]),
    "bns_forward_mixed": (C.c_int, [_SHP, _SPC, C.c_uint64, C.c_int32, C.c_float, _P, _P, _P, C.c_float, C.c_float,
                                    _P, _P, _P, _P, _P, _P, _P, C.c_size_t, _P]),
    "bns_backward_mixed": (C.c_int, [_SHP, _SPC, C.c_uint64, C.c_int32, C.c_float, _P, _P, _P, _P, _P, _P,
                                     _P, _P, _P, _P, C.c_size_t, _P]),
    "bns_inference": (C.c_int, [_SHP, _P, _P, _P, _P, _P, C.c_float, _P, _P]),
    "bns_moving_average_weight": (C.c_float, [C.c_uint64, C.c_float]),
    "bns_copy_reference": (C.c_int, [_P, _P, C.c_size_t, _P]),
    "bns_set_option": (C.c_int, [C.c_char_p, C.c_int32]),
    "bns_get_option": (C.c_int32, [C.c_char_p]),
}


def load(reload: bool = False):
    """Load libbns.so (built by ``__graft_entry__.build()``); raises if it is not there."""
    global _lib
    if _lib is not None and not reload:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} not found: build it with `python __graft_entry__.py` "
                          "(there is no CPU fallback)")
    # PyTorch ships a HIP runtime of its own.  The device memory and streams this binding hands to the library
    # come from it, so it has to be the one runtime in the process: loaded before libbns.so, whose dependency
    # on libamdhip64 then resolves to it.  (The other order puts two runtimes side by side; launches then fail
    # or crash.)
    import torch  # noqa: F401
    lib = C.CDLL(LIB_PATH)
    for name, (res, args) in _PROTOS.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    return lib


def declared_symbols():
    """Names of the functions that include/bns.h declares."""
    text = open(HEADER_PATH).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(bns_[a-z_0-9]+)\s*\(", text)))


def missing_symbols():
    lib = load()
    out = []
    for name in declared_symbols():
        try:
            getattr(lib, name)
        except AttributeError:
            out.append(name)
    return out + [n for n in declared_symbols() if n not in _PROTOS]


# --------------------------------------------------------------------------------------
# marshalling helpers
# --------------------------------------------------------------------------------------
def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(t):
    import torch
    return C.c_void_p(torch.cuda.current_stream(t.device).cuda_stream)


def _check(status, where):
    if status != BNS_OK:
        raise BnsError(status, where)


def make_shape(N, C_, H, W, dtype="f32", layout="nchw") -> bns_shape:
    return bns_shape(N, C_, H, W, {"f32": BNS_F32, "bf16": BNS_BF16}[dtype] if isinstance(dtype, str) else dtype,
                     {"nchw": BNS_NCHW, "nhwc": BNS_NHWC}[layout] if isinstance(layout, str) else layout)


def make_spec(mode, n_s=0, patch_h=0, patch_w=0, fs_per_channel=0, layer_id=0, epoch=0) -> bns_spec:
    return bns_spec(mode, n_s, patch_h, patch_w, fs_per_channel, layer_id, epoch)


def _boxes_to_numpy(arr, n):
    return np.ctypeslib.as_array(C.cast(arr, C.POINTER(C.c_int32)), shape=(n, 6)).copy()


# --------------------------------------------------------------------------------------
# the entry points, one Python function per C function
# --------------------------------------------------------------------------------------
def bns_status_string(status: int) -> str:
    return load().bns_status_string(status).decode()


def bns_sample_index(shape: bns_shape, spec: bns_spec, seed: int) -> np.ndarray:
    """Host index: int32 array [C, 6] = (n0, n_cnt, h0, h_cnt, w0, w_cnt)."""
    lib = load()
    n = max(int(shape.C), 0)
    arr = (bns_box * max(n, 1))()
    _check(lib.bns_sample_index(C.byref(shape), C.byref(spec), C.c_uint64(seed), arr), "bns_sample_index")
    return _boxes_to_numpy(arr, n)


def bns_sample_index_device(shape: bns_shape, spec: bns_spec, seed: int, device="cuda:0") -> np.ndarray:
    """The same index computed by the device generator; returned as a host array."""
    import torch
    lib = load()
    out = torch.empty((shape.C, 6), dtype=torch.int32, device=device)
    _check(lib.bns_sample_index_device(C.byref(shape), C.byref(spec), C.c_uint64(seed), _ptr(out), _stream(out)),
           "bns_sample_index_device")
    return out.cpu().numpy()


def bns_workspace_bytes(shape: bns_shape, spec: bns_spec) -> int:
    return int(load().bns_workspace_bytes(C.byref(shape), C.byref(spec)))


def bns_forward(shape, spec, seed, x, gamma, beta, eps, momentum, y, save_mean, save_invstd,
                running_mean, running_var, workspace):
    _check(load().bns_forward(C.byref(shape), C.byref(spec), C.c_uint64(seed), _ptr(x), _ptr(gamma), _ptr(beta),
                              C.c_float(eps), C.c_float(momentum), _ptr(y), _ptr(save_mean), _ptr(save_invstd),
                              _ptr(running_mean), _ptr(running_var), _ptr(workspace),
                              C.c_size_t(workspace.numel() * workspace.element_size()), _stream(x)), "bns_forward")


def bns_backward(shape, spec, seed, x, dy, gamma, save_mean, save_invstd, dx, dgamma, dbeta, workspace):
    _check(load().bns_backward(C.byref(shape), C.byref(spec), C.c_uint64(seed), _ptr(x), _ptr(dy), _ptr(gamma),
                               _ptr(save_mean), _ptr(save_invstd), _ptr(dx), _ptr(dgamma), _ptr(dbeta),
                               _ptr(workspace), C.c_size_t(workspace.numel() * workspace.element_size()),
                               _stream(x)), "bns_backward")


def bns_backward_builtin_workspace(shape, spec, seed, x, dy, gamma, save_mean, save_invstd, dx, dgamma, dbeta):
    _check(load().bns_backward_builtin_workspace(C.byref(shape), C.byref(spec), C.c_uint64(seed), _ptr(x), _ptr(dy),
                                                 _ptr(gamma), _ptr(save_mean), _ptr(save_invstd), _ptr(dx),
                                                 _ptr(dgamma), _ptr(dbeta), _stream(x)),
           "bns_backward_builtin_workspace")


def bns_expired_waits(workspace=None, stream_of=None) -> int:
    """Waits between blocks that ran out in the calls on `workspace` (None: the built-in scratch) since the last query."""
    import torch
    out = C.c_int32(-1)
    t = workspace if workspace is not None else stream_of
    stream = _stream(t) if t is not None else C.c_void_p(torch.cuda.current_stream().cuda_stream)
    nbytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(load().bns_expired_waits(_ptr(workspace), C.c_size_t(nbytes), stream, C.byref(out)), "bns_expired_waits")
    return int(out.value)


def bns_forward_stats(shape, spec, seed, x, eps, momentum, save_mean, save_invstd, running_mean, running_var,
                      workspace):
    _check(load().bns_forward_stats(C.byref(shape), C.byref(spec), C.c_uint64(seed), _ptr(x), C.c_float(eps),
                                    C.c_float(momentum), _ptr(save_mean), _ptr(save_invstd), _ptr(running_mean),
                                    _ptr(running_var), _ptr(workspace),
                                    C.c_size_t(workspace.numel() * workspace.element_size()), _stream(x)),
           "bns_forward_stats")


def bns_forward_normalize(shape, x, gamma, beta, save_mean, save_invstd, y):
    _check(load().bns_forward_normalize(C.byref(shape), _ptr(x), _ptr(gamma), _ptr(beta), _ptr(save_mean),
                                        _ptr(save_invstd), _ptr(y), _stream(x)), "bns_forward_normalize")


def bns_backward_reduce(shape, x, dy, save_mean, save_invstd, dgamma, dbeta, workspace):
    _check(load().bns_backward_reduce(C.byref(shape), _ptr(x), _ptr(dy), _ptr(save_mean), _ptr(save_invstd),
                                      _ptr(dgamma), _ptr(dbeta), _ptr(workspace),
                                      C.c_size_t(workspace.numel() * workspace.element_size()), _stream(x)),
           "bns_backward_reduce")


def bns_backward_dx(shape, spec, seed, x, dy, gamma, save_mean, save_invstd, dgamma, dbeta, dx):
    _check(load().bns_backward_dx(C.byref(shape), C.byref(spec), C.c_uint64(seed), _ptr(x), _ptr(dy), _ptr(gamma),
                                  _ptr(save_mean), _ptr(save_invstd), _ptr(dgamma), _ptr(dbeta), _ptr(dx),
                                  _stream(x)), "bns_backward_dx")


def bns_sample_index_mixed(shape: bns_shape, spec: bns_spec, seed: int, n_v: int) -> np.ndarray:
    """Host index of the sampled real set for "VDN + sampling": int32 array [C, 6]."""
    lib = load()
    n = max(int(shape.C), 0)
    arr = (bns_box * max(n, 1))()
    _check(lib.bns_sample_index_mixed(C.byref(shape), C.byref(spec), C.c_uint64(seed), C.c_int32(n_v), arr),
           "bns_sample_index_mixed")
    return _boxes_to_numpy(arr, n)


def bns_forward_mixed(shape, spec, seed, n_v, mix_beta, x, gamma, beta, eps, momentum, y, save_mean, save_invstd,
                      save_mean_parts, running_mean, running_var, workspace):
    _check(load().bns_forward_mixed(C.byref(shape), C.byref(spec), C.c_uint64(seed), C.c_int32(n_v),
                                    C.c_float(mix_beta), _ptr(x), _ptr(gamma), _ptr(beta), C.c_float(eps),
                                    C.c_float(momentum), _ptr(y), _ptr(save_mean), _ptr(save_invstd),
                                    _ptr(save_mean_parts), _ptr(running_mean), _ptr(running_var), _ptr(workspace),
                                    C.c_size_t(workspace.numel() * workspace.element_size()), _stream(x)),
           "bns_forward_mixed")


def bns_backward_mixed(shape, spec, seed, n_v, mix_beta, x, dy, gamma, save_mean, save_invstd, save_mean_parts,
                       dx, dgamma, dbeta, workspace):
    _check(load().bns_backward_mixed(C.byref(shape), C.byref(spec), C.c_uint64(seed), C.c_int32(n_v),
                                     C.c_float(mix_beta), _ptr(x), _ptr(dy), _ptr(gamma), _ptr(save_mean),
                                     _ptr(save_invstd), _ptr(save_mean_parts), _ptr(dx), _ptr(dgamma), _ptr(dbeta),
                                     _ptr(workspace), C.c_size_t(workspace.numel() * workspace.element_size()),
                                     _stream(x)), "bns_backward_mixed")


def bns_inference(shape, x, gamma, beta, running_mean, running_var, eps, y):
    _check(load().bns_inference(C.byref(shape), _ptr(x), _ptr(gamma), _ptr(beta), _ptr(running_mean),
                                _ptr(running_var), C.c_float(eps), _ptr(y), _stream(x)), "bns_inference")


def bns_moving_average_weight(iteration: int, alpha: float) -> float:
    return float(load().bns_moving_average_weight(C.c_uint64(iteration), C.c_float(alpha)))


def bns_copy_reference(dst, src):
    nbytes = src.numel() * src.element_size()
    _check(load().bns_copy_reference(_ptr(dst), _ptr(src), C.c_size_t(nbytes), _stream(src)), "bns_copy_reference")


def bns_set_option(name: str, value: int):
    _check(load().bns_set_option(name.encode(), C.c_int32(value)), f"bns_set_option({name})")


def bns_get_option(name: str) -> int:
    return int(load().bns_get_option(name.encode()))


# --------------------------------------------------------------------------------------
# convenience for tests, smoke and bench: device buffers for one workload
# --------------------------------------------------------------------------------------
class Buffers:
    """Device tensors for one workload: inputs uploaded, outputs and workspace allocated.

    ``inputs`` and ``results()`` are always indexed [n, c, h, w]; for an "nhwc" workload the device
    copies of x, dy, y, dx are stored N x H x W x C (a transposition of the data, nothing else).
    """

    def __init__(self, wl, inputs, device="cuda:0"):
        import torch
        tdt = torch.float32 if wl.dtype == "f32" else torch.bfloat16
        dev = torch.device(device)
        self.wl = wl
        self.nhwc = getattr(wl, "layout", "nchw") == "nhwc"
        self.shape = make_shape(wl.N, wl.C, wl.H, wl.W, wl.dtype, "nhwc" if self.nhwc else "nchw")
        self.spec = make_spec(wl.mode, wl.n_s, wl.patch_h, wl.patch_w, wl.fs_per_channel, wl.layer_id, wl.epoch)
        self.seed = wl.sampling_seed
        up = lambda a, dt=torch.float32: torch.from_numpy(np.ascontiguousarray(a)).to(dev).to(dt).contiguous()
        stored = (lambda a: np.transpose(a, (0, 2, 3, 1))) if self.nhwc else (lambda a: a)
        self.x = up(stored(inputs["x"]), tdt)
        self.dy = up(stored(inputs["dy"]), tdt)
        self.gamma = up(inputs["gamma"])
        self.beta = up(inputs["beta"])
        self.running_mean = up(inputs["running_mean"])
        self.running_var = up(inputs["running_var"])
        self.y = torch.empty_like(self.x)
        self.dx = torch.empty_like(self.x)
        f32 = dict(dtype=torch.float32, device=dev)
        self.save_mean = torch.empty(wl.C, **f32)
        self.save_invstd = torch.empty(wl.C, **f32)
        self.dgamma = torch.empty(wl.C, **f32)
        self.dbeta = torch.empty(wl.C, **f32)
        self.workspace = torch.empty(max(bns_workspace_bytes(self.shape, self.spec), 16), dtype=torch.uint8,
                                     device=dev)
        self.n_v = getattr(wl, "n_v", 0) if wl.mode != BNS_VDN else 0
        self._fwd_args = self._bwd_args = None
        self.save_mean_parts = torch.empty(2 * wl.C, **f32) if self.n_v else None

    def _stream_ptr(self):
        import torch
        return C.c_void_p(torch.cuda.current_stream(self.x.device).cuda_stream)

    def forward(self):
        if self.n_v == 0:
            # same call as bns_forward(...) below, with the argument marshalling done once per buffer set
            if self._fwd_args is None:
                ws = self.workspace
                self._fwd_args = (C.byref(self.shape), C.byref(self.spec), C.c_uint64(self.seed), _ptr(self.x),
                                  _ptr(self.gamma), _ptr(self.beta), C.c_float(self.wl.eps),
                                  C.c_float(self.wl.momentum), _ptr(self.y), _ptr(self.save_mean),
                                  _ptr(self.save_invstd), _ptr(self.running_mean), _ptr(self.running_var), _ptr(ws),
                                  C.c_size_t(ws.numel() * ws.element_size()))
            _check(_lib.bns_forward(*self._fwd_args, self._stream_ptr()), "bns_forward")
        else:
            # same call as bns_forward_mixed(...), marshalled once
            if self._fwd_args is None:
                ws = self.workspace
                self._fwd_args = (C.byref(self.shape), C.byref(self.spec), C.c_uint64(self.seed), C.c_int32(self.n_v),
                                  C.c_float(self.wl.mix_beta), _ptr(self.x), _ptr(self.gamma), _ptr(self.beta),
                                  C.c_float(self.wl.eps), C.c_float(self.wl.momentum), _ptr(self.y),
                                  _ptr(self.save_mean), _ptr(self.save_invstd), _ptr(self.save_mean_parts),
                                  _ptr(self.running_mean), _ptr(self.running_var), _ptr(ws),
                                  C.c_size_t(ws.numel() * ws.element_size()))
            _check(_lib.bns_forward_mixed(*self._fwd_args, self._stream_ptr()), "bns_forward_mixed")

    def backward(self):
        if self.n_v == 0:
            if self._bwd_args is None:
                ws = self.workspace
                self._bwd_args = (C.byref(self.shape), C.byref(self.spec), C.c_uint64(self.seed), _ptr(self.x),
                                  _ptr(self.dy), _ptr(self.gamma), _ptr(self.save_mean), _ptr(self.save_invstd),
                                  _ptr(self.dx), _ptr(self.dgamma), _ptr(self.dbeta), _ptr(ws),
                                  C.c_size_t(ws.numel() * ws.element_size()))
            _check(_lib.bns_backward(*self._bwd_args, self._stream_ptr()), "bns_backward")
        else:
            if self._bwd_args is None:
                ws = self.workspace
                self._bwd_args = (C.byref(self.shape), C.byref(self.spec), C.c_uint64(self.seed), C.c_int32(self.n_v),
                                  C.c_float(self.wl.mix_beta), _ptr(self.x), _ptr(self.dy), _ptr(self.gamma),
                                  _ptr(self.save_mean), _ptr(self.save_invstd), _ptr(self.save_mean_parts),
                                  _ptr(self.dx), _ptr(self.dgamma), _ptr(self.dbeta), _ptr(ws),
                                  C.c_size_t(ws.numel() * ws.element_size()))
            _check(_lib.bns_backward_mixed(*self._bwd_args, self._stream_ptr()), "bns_backward_mixed")

    def results(self):
        import torch
        torch.cuda.synchronize()
        host = lambda t: t.detach().float().cpu().numpy()
        logical = (lambda t: np.ascontiguousarray(np.transpose(host(t), (0, 3, 1, 2)))) if self.nhwc else host
        return dict(y=logical(self.y), dx=logical(self.dx), save_mean=host(self.save_mean),
                    save_invstd=host(self.save_invstd), running_mean=host(self.running_mean),
                    running_var=host(self.running_var), dgamma=host(self.dgamma), dbeta=host(self.dbeta),
                    boxes=(bns_sample_index_mixed(self.shape, self.spec, self.seed, self.n_v) if self.n_v
                           else bns_sample_index(self.shape, self.spec, self.seed)),
                    **({"save_mean_parts": host(self.save_mean_parts)} if self.n_v else {}))


def run_workload(wl, inputs, device="cuda:0"):
    """Upload, one forward + backward through the C ABI, download everything as numpy."""
    b = Buffers(wl, inputs, device)
    b.forward()
    b.backward()
    return b.results()
