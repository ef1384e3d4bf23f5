"""ctypes front end of oracle/conv_ref.c (test infrastructure only).

The C file is the oracle; this module only compiles it with gcc, marshals
numpy arrays in and out, and states the comparison rule. It imports nothing
from the GPU package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "conv_ref.c")
_LIB = os.path.join(_HERE, "libconv_ref.so")
_lib = None

_f32p = ctypes.POINTER(ctypes.c_float)
_f64p = ctypes.POINTER(ctypes.c_double)
_i32p = ctypes.POINTER(ctypes.c_int)
_u64p = ctypes.POINTER(ctypes.c_uint64)


def build(force: bool = False) -> str:
    """Compile the oracle with gcc -O2 (no fast-math, no FMA contraction across the fp64 sums)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lpthread", "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        ints9 = [ctypes.c_int] * 9
        lib.conv_ref.argtypes = [_f32p, _f32p, _f64p, _f64p] + ints9 + [ctypes.c_int]
        lib.conv_ref.restype = ctypes.c_int
        lib.conv_ref_points.argtypes = [_f32p, _f32p, _i32p, ctypes.c_long, _f64p, _f64p] + ints9
        lib.conv_ref_points.restype = ctypes.c_int
        lib.conv_ref_counted.argtypes = [_f32p, _f32p, _f64p, _u64p, _u64p, _u64p] + ints9
        lib.conv_ref_counted.restype = ctypes.c_int
        _lib = lib
    return _lib


def _prep(x, w, pad_h, pad_w):
    x = np.ascontiguousarray(x, dtype=np.float32)
    w = np.ascontiguousarray(w, dtype=np.float32)
    if x.ndim != 4 or w.ndim != 4 or x.shape[1] != w.shape[1]:
        raise ValueError("expected x[N,C,H,W] and w[K,C,R,S] with equal C")
    N, C, H, W = x.shape
    K, _, R, S = w.shape
    P, Q = H + 2 * pad_h - R + 1, W + 2 * pad_w - S + 1
    return x, w, (N, C, H, W, K, R, S, pad_h, pad_w), P, Q


def _check(rc):
    if rc != 0:
        raise ValueError({-1: "null pointer", -2: "bad dimension", -3: "empty output"}.get(rc, f"error {rc}"))


def conv_ref(x, w, pad_h: int, pad_w: int, nthreads: int = 0):
    """Full layer: returns (y, yabs) as float64 arrays [N,K,P,Q]; yabs = sum |x*w| per output."""
    x, w, dims, P, Q = _prep(x, w, pad_h, pad_w)
    if P <= 0 or Q <= 0:
        _check(-3)
    if nthreads <= 0:
        nthreads = os.cpu_count() or 1
    y = np.empty((dims[0], dims[4], P, Q), dtype=np.float64)
    ya = np.empty_like(y)
    rc = _load().conv_ref(x.ctypes.data_as(_f32p), w.ctypes.data_as(_f32p), y.ctypes.data_as(_f64p),
                          ya.ctypes.data_as(_f64p), *dims, nthreads)
    _check(rc)
    return y, ya


def conv_ref_points(x, w, pad_h: int, pad_w: int, coords):
    """Selected outputs: coords is an int array [npts,4] of (n,k,p,q); returns (y, yabs) of length npts."""
    x, w, dims, P, Q = _prep(x, w, pad_h, pad_w)
    coords = np.ascontiguousarray(coords, dtype=np.int32).reshape(-1, 4)
    y = np.empty(coords.shape[0], dtype=np.float64)
    ya = np.empty_like(y)
    rc = _load().conv_ref_points(x.ctypes.data_as(_f32p), w.ctypes.data_as(_f32p), coords.ctypes.data_as(_i32p),
                                 coords.shape[0], y.ctypes.data_as(_f64p), ya.ctypes.data_as(_f64p), *dims)
    _check(rc)
    return y, ya


def conv_ref_counted(x, w, pad_h: int, pad_w: int):
    """Single-threaded run that also counts multiply-adds: returns (y, x_touch, w_touch, macs)."""
    x, w, dims, P, Q = _prep(x, w, pad_h, pad_w)
    y = np.empty((dims[0], dims[4], P, Q), dtype=np.float64)
    xt = np.zeros(x.shape, dtype=np.uint64)
    wt = np.zeros(w.shape, dtype=np.uint64)
    macs = ctypes.c_uint64(0)
    rc = _load().conv_ref_counted(x.ctypes.data_as(_f32p), w.ctypes.data_as(_f32p), y.ctypes.data_as(_f64p),
                                  xt.ctypes.data_as(_u64p), wt.ctypes.data_as(_u64p), ctypes.byref(macs), *dims)
    _check(rc)
    return y, xt, wt, int(macs.value)


def conv_bias_relu_ref(x, w, bias, pad_h: int, pad_w: int, relu: bool, nthreads: int = 0):
    """The layer with its epilogue (Section 2.1: the weighted sums are usually passed through a non-linear
    function such as ReLU): conv_ref, plus bias[k] on every output of channel k (None: no bias), then
    max(., 0) if relu. Returns (y, yabs) in fp64 with yabs = sum |x*w| + |bias[k]|, the magnitude the
    tolerance rule scales with."""
    y, ya = conv_ref(x, w, pad_h, pad_w, nthreads=nthreads)
    if bias is not None:
        b = np.asarray(bias, dtype=np.float64).reshape(1, -1, 1, 1)
        if b.shape[1] != y.shape[1]:
            raise ValueError("bias needs one value per filter")
        y = y + b
        ya = ya + np.abs(b)
    if relu:
        y = np.maximum(y, 0.0)
    return y, ya


def within_tolerance(y_test, y_ref, yabs_ref, rel: float = 1e-5, abs_: float = 1e-6):
    """The acceptance rule: |y_test - y_ref| <= rel * sum|x*w| + abs_, elementwise.

    Returns (ok, worst) where worst is the largest (|diff| - abs_) / (rel * yabs) seen
    (values <= 1 pass; outputs with yabs == 0 are judged on the absolute term alone).
    """
    d = np.abs(np.asarray(y_test, dtype=np.float64) - y_ref)
    bound = rel * yabs_ref + abs_
    ok = bool(np.all(d <= bound))
    with np.errstate(divide="ignore", invalid="ignore"):
        ratio = np.where(yabs_ref > 0, (d - abs_) / (rel * yabs_ref), np.where(d <= abs_, 0.0, np.inf))
    return ok, float(ratio.max()) if ratio.size else 0.0
