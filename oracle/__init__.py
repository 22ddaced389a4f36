"""CPU oracle for the SqueezeNet forward path -- TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper over ``sq_oracle.c`` (plain nested loops, double
accumulation; see that file's header for the passages of the paper it follows
and the readings it takes).  Only ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import this package.  It imports nothing
from the GPU package and the GPU package imports nothing from here.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sq_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

TAP_NAMES = ("conv1", "pool1", "fire2", "fire3", "fire4", "pool4", "fire5", "fire6",
             "fire7", "fire8", "pool8", "fire9", "conv10", "means", "probs")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, no fast-math, OpenMP over planes)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
    return _lib


_F = ctypes.POINTER(ctypes.c_float)


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _p(a):
    return None if a is None else a.ctypes.data_as(_F)


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise ValueError(f"oracle {what} rejected its arguments (code {rc})")


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_num_threads(t: int) -> None:
    _load().oracle_set_num_threads(int(t))


def conv2d(x, w, b=None, stride: int = 1, pad: int = 0, relu: bool = False) -> np.ndarray:
    x, w = _f32(x), _f32(w)
    b = None if b is None else _f32(b)
    N, Cin, H, W = x.shape
    Cout, Cin2, K, K2 = w.shape
    if Cin2 != Cin or K2 != K:
        raise ValueError("kernel shape does not match the input")
    if b is not None and b.shape != (Cout,):
        raise ValueError("bias shape")
    if H + 2 * pad < K or W + 2 * pad < K or stride < 1 or pad < 0:
        raise ValueError("window does not fit")
    Ho = (H + 2 * pad - K) // stride + 1
    Wo = (W + 2 * pad - K) // stride + 1
    out = np.empty((N, Cout, Ho, Wo), dtype=np.float32)
    rc = _load().oracle_conv2d(_p(x), _p(w), _p(b), _p(out), N, Cin, H, W, Cout, K,
                               int(stride), int(pad), int(bool(relu)))
    _check(rc, "conv2d")
    return out


def maxpool(x, k: int = 3, stride: int = 2) -> np.ndarray:
    x = _f32(x)
    N, C, H, W = x.shape
    if H < k or W < k or stride < 1:
        raise ValueError("window does not fit")
    Ho, Wo = (H - k) // stride + 1, (W - k) // stride + 1
    out = np.empty((N, C, Ho, Wo), dtype=np.float32)
    _check(_load().oracle_maxpool(_p(x), _p(out), N, C, H, W, int(k), int(stride)), "maxpool")
    return out


def avgpool_global(x) -> np.ndarray:
    x = _f32(x)
    N, C, H, W = x.shape
    out = np.empty((N, C), dtype=np.float32)
    _check(_load().oracle_avgpool_global(_p(x), _p(out), N, C, H, W), "avgpool_global")
    return out


def softmax(x) -> np.ndarray:
    x = _f32(x)
    N, C = x.shape
    out = np.empty((N, C), dtype=np.float32)
    _check(_load().oracle_softmax(_p(x), _p(out), N, C), "softmax")
    return out


def fire(x, w_sq, b_sq, w_e1, b_e1, w_e3, b_e3) -> np.ndarray:
    x = _f32(x)
    w_sq, w_e1, w_e3 = _f32(w_sq), _f32(w_e1), _f32(w_e3)
    b_sq = None if b_sq is None else _f32(b_sq)
    b_e1 = None if b_e1 is None else _f32(b_e1)
    b_e3 = None if b_e3 is None else _f32(b_e3)
    N, Cin, H, W = x.shape
    Csq, Ce1, Ce3 = w_sq.shape[0], w_e1.shape[0], w_e3.shape[0]
    if w_sq.shape != (Csq, Cin, 1, 1) or w_e1.shape != (Ce1, Csq, 1, 1) \
            or w_e3.shape != (Ce3, Csq, 3, 3):
        raise ValueError("fire kernel shapes")
    out = np.empty((N, Ce1 + Ce3, H, W), dtype=np.float32)
    rc = _load().oracle_fire(_p(x), _p(w_sq), _p(b_sq), _p(w_e1), _p(b_e1), _p(w_e3),
                             _p(b_e3), _p(out), N, Cin, H, W, Csq, Ce1, Ce3)
    _check(rc, "fire")
    return out


_TAP_SHAPES = ((96, 111), (96, 55), (128, 55), (128, 55), (256, 55), (256, 27), (256, 27),
               (384, 27), (384, 27), (512, 27), (512, 13), (512, 13), (1000, 13))


def squeezenet(x, params, want_taps: bool = False):
    """x: [N,3,224,224]; params: 52 arrays (weight, bias per convolution in network
    order).  Returns probs [N,1000], or (probs, {stage name: array}) with want_taps."""
    x = _f32(x)
    N = x.shape[0]
    if x.shape[1:] != (3, 224, 224) or len(params) != 52:
        raise ValueError("squeezenet expects [N,3,224,224] and 52 parameter arrays")
    ps = [_f32(p) for p in params]
    arr = (_F * 52)(*[_p(p) for p in ps])
    probs = np.empty((N, 1000), dtype=np.float32)
    taps = {}
    tap_arr = None
    if want_taps:
        for name, (c, h) in zip(TAP_NAMES, _TAP_SHAPES):
            taps[name] = np.empty((N, c, h, h), dtype=np.float32)
        taps["means"] = np.empty((N, 1000), dtype=np.float32)
        taps["probs"] = np.empty((N, 1000), dtype=np.float32)
        ptrs = [_p(taps[n]) for n in TAP_NAMES] + [None]
        tap_arr = (_F * 16)(*ptrs)
    rc = _load().oracle_squeezenet(_p(x), arr, _p(probs), N, tap_arr)
    _check(rc, "squeezenet")
    return (probs, taps) if want_taps else probs
