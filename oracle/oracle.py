"""ctypes binding of the fp64 CPU oracle in oracle.c -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the bench's CPU-baseline leg import this.  It
marshals numpy arrays (logical NCHW / OIHW, converted to contiguous fp64) into
the C functions; all arithmetic is in oracle.c.  It imports nothing from the
HIP package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None

__all__ = [
    "build", "out_size", "conv2d", "bn", "bn_fold", "scale_shift", "relu", "add", "maxpool2d",
    "global_avgpool", "fc", "basic_block", "resnet18_stage", "resnet18", "pack_params",
    "set_threads", "max_threads",
]

_dp = ctypes.POINTER(ctypes.c_double)


def build(force: bool = False) -> str:
    """Compile oracle.c into liboracle.so with gcc (OpenMP, -O2, strict fp)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        try:
            _omp = ctypes.CDLL("libgomp.so.1")
            _lib._omp = _omp
        except OSError:  # pragma: no cover
            _lib._omp = None
    return _lib


def set_threads(n: int) -> None:
    lib = _load()
    if lib._omp is not None:
        lib._omp.omp_set_num_threads(int(n))


def max_threads() -> int:
    lib = _load()
    return int(lib._omp.omp_get_max_threads()) if lib._omp is not None else 1


def _d(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _p(a: np.ndarray):
    return a.ctypes.data_as(_dp)


def out_size(n: int, kernel: int, stride: int, pad: int) -> int:
    return int(_load().oracle_out_size(int(n), int(kernel), int(stride), int(pad)))


def conv2d(x, w, stride: int = 1, pad: int = 0) -> np.ndarray:
    x, w = _d(x), _d(w)
    N, C, H, W = x.shape
    K, C2, R, S = w.shape
    assert C == C2
    P, Q = out_size(H, R, stride, pad), out_size(W, S, stride, pad)
    y = np.empty((N, K, P, Q), dtype=np.float64)
    _load().oracle_conv2d(_p(x), _p(w), _p(y), N, C, H, W, K, R, S, int(stride), int(pad))
    return y


def bn(x, gamma, beta, mean, var, eps: float) -> np.ndarray:
    x = _d(x)
    N, C = x.shape[:2]
    hw = int(np.prod(x.shape[2:], dtype=np.int64))
    y = np.empty_like(x)
    g, b, m, v = _d(gamma), _d(beta), _d(mean), _d(var)
    _load().oracle_bn(_p(x), _p(g), _p(b), _p(m), _p(v), ctypes.c_double(eps), _p(y), N, C, hw)
    return y


def bn_fold(gamma, beta, mean, var, eps: float):
    g, b, m, v = _d(gamma), _d(beta), _d(mean), _d(var)
    C = g.shape[0]
    scale, shift = np.empty(C), np.empty(C)
    _load().oracle_bn_fold(_p(g), _p(b), _p(m), _p(v), ctypes.c_double(eps), _p(scale), _p(shift), C)
    return scale, shift


def scale_shift(x, scale, shift) -> np.ndarray:
    x, sc, sh = _d(x), _d(scale), _d(shift)
    N, C = x.shape[:2]
    hw = int(np.prod(x.shape[2:], dtype=np.int64))
    y = np.empty_like(x)
    _load().oracle_scale_shift(_p(x), _p(sc), _p(sh), _p(y), N, C, hw)
    return y


def relu(x) -> np.ndarray:
    x = _d(x)
    y = np.empty_like(x)
    _load().oracle_relu(_p(x), _p(y), ctypes.c_size_t(x.size))
    return y


def add(a, b) -> np.ndarray:
    a, b = _d(a), _d(b)
    assert a.shape == b.shape
    y = np.empty_like(a)
    _load().oracle_add(_p(a), _p(b), _p(y), ctypes.c_size_t(a.size))
    return y


def maxpool2d(x, kernel: int = 3, stride: int = 2, pad: int = 1) -> np.ndarray:
    x = _d(x)
    N, C, H, W = x.shape
    P, Q = out_size(H, kernel, stride, pad), out_size(W, kernel, stride, pad)
    y = np.empty((N, C, P, Q), dtype=np.float64)
    _load().oracle_maxpool2d(_p(x), _p(y), N, C, H, W, int(kernel), int(stride), int(pad))
    return y


def global_avgpool(x) -> np.ndarray:
    x = _d(x)
    N, C = x.shape[:2]
    hw = int(np.prod(x.shape[2:], dtype=np.int64))
    v = np.empty((N, C), dtype=np.float64)
    _load().oracle_global_avgpool(_p(x), _p(v), N, C, hw)
    return v


def fc(v, w, b=None) -> np.ndarray:
    v, w = _d(v), _d(w)
    N, cin = v.shape
    cout = w.shape[0]
    assert w.shape[1] == cin
    y = np.empty((N, cout), dtype=np.float64)
    bb = _d(b) if b is not None else None
    _load().oracle_fc(_p(v), _p(w), _p(bb) if bb is not None else None, _p(y), N, cin, cout)
    return y


def _ptr_array(arrs):
    keep = [_d(a) for a in arrs]
    arr = (_dp * len(keep))(*[_p(a) for a in keep])
    return arr, keep


def basic_block(x, convs, eps: float, stride: int = 1) -> np.ndarray:
    """convs: list of 2 or 3 tuples (w, gamma, beta, mean, var): conv1, conv2[, down]."""
    x = _d(x)
    N, C, H, _ = x.shape
    K = np.shape(convs[0][0])[0]
    flat = [t for cv in convs for t in cv]
    pa, keep = _ptr_array(flat)
    P = out_size(H, 3, stride, 1)
    y = np.empty((N, K, P, P), dtype=np.float64)
    _load().oracle_basic_block(_p(x), pa, int(len(convs) == 3), ctypes.c_double(eps), _p(y),
                               N, C, H, K, int(stride))
    del keep
    return y


def pack_params(params: dict):
    """dict from workloads.make_resnet18_params -> (pointer array, keep-alive list)."""
    flat = []
    for i in range(20):
        flat += [params["conv_w"][i], params["gamma"][i], params["beta"][i], params["mean"][i],
                 params["var"][i]]
    flat += [params["fc_w"], params["fc_b"]]
    return _ptr_array(flat)


_STAGE_OUT = [(64, 56, 56), (64, 56, 56), (128, 28, 28), (256, 14, 14), (512, 7, 7)]


def resnet18_stage(j: int, params: dict, eps: float, x) -> np.ndarray:
    if not 0 <= int(j) <= 5:
        raise ValueError(f"bad stage {j}")
    x = _d(x)
    N = x.shape[0]
    pa, keep = pack_params(params)
    out = np.empty((N, 1000) if j == 5 else (N,) + _STAGE_OUT[j], dtype=np.float64)
    rc = _load().oracle_resnet18_stage(int(j), pa, ctypes.c_double(eps), _p(x), _p(out), N)
    if rc != 0:
        raise ValueError(f"bad stage {j}")
    del keep
    return out


def resnet18(params: dict, eps: float, x, want_stages: bool = False):
    """logits [N,1000]; with want_stages also the list of the six stage outputs."""
    x = _d(x)
    N = x.shape[0]
    pa, keep = pack_params(params)
    logits = np.empty((N, 1000), dtype=np.float64)
    if want_stages:
        outs = [np.empty((N,) + s, dtype=np.float64) for s in _STAGE_OUT] + [logits]
        so = (_dp * 6)(*[_p(o) for o in outs])
    else:
        outs, so = None, None
    rc = _load().oracle_resnet18(pa, ctypes.c_double(eps), _p(x), _p(logits), N, so)
    if rc != 0:
        raise RuntimeError("oracle_resnet18 failed")
    del keep
    return (logits, outs) if want_stages else logits
