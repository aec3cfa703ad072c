"""ctypes front end of the fp64 CPU oracle (oracle/conv_oracle.c).

TEST INFRASTRUCTURE ONLY.  Nothing in the product package imports this; only tests, the smoke check
and the benchmark's cpu_baseline leg do.  It imports nothing from the HIP path.

Functions and what pins each of them (tests/test_oracle_*.py, all CPU):
  conv2d / conv2d_points  brute force on tiny inputs against a differently structured routine, a
                          hand-computed example, 1x1 conv == matrix product (shapes of Table 1),
                          delta filters, linearity, all-ones input, float64 library conv.
  dims                    the worked example of Section 4.1 (M=256, N=128, K=1152).
  round_bf16              all 65536 bfloat16 patterns round-trip; 10^6 float32 values against a
                          library cast; hand-written tie cases.
  maxpool2d, relu         textbook definitions; brute force and library comparison.
  conv_layer              conv2d, then + residual, then relu: composition of the above, nothing else.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "conv_oracle.c")
_LIB = os.path.join(_HERE, "liboracle_conv.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP, no intrinsics, no BLAS)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-std=c99", "-shared", "-fPIC", "-Wall",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        dp, ip = ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int32)
        i, i64 = ctypes.c_int, ctypes.c_int64
        lib.oracle_out_dim.argtypes = [i, i, i, i]
        lib.oracle_out_dim.restype = i
        lib.oracle_conv2d_f64.argtypes = [dp, dp, dp] + [i] * 9
        lib.oracle_conv2d_f64.restype = None
        lib.oracle_conv2d_f64_points.argtypes = [dp, dp, ip, dp, i64] + [i] * 9
        lib.oracle_conv2d_f64_points.restype = None
        lib.oracle_maxpool2d_f64.argtypes = [dp, dp] + [i] * 7
        lib.oracle_maxpool2d_f64.restype = None
        lib.oracle_round_bf16.argtypes = [dp, dp, i64]
        lib.oracle_round_bf16.restype = None
        lib.oracle_num_threads.argtypes = []
        lib.oracle_num_threads.restype = i
        _lib = lib
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def num_threads() -> int:
    """Threads the OpenMP loops actually use."""
    return int(_load().oracle_num_threads())


def out_dim(size: int, filt: int, stride: int, pad: int) -> int:
    return int(_load().oracle_out_dim(size, filt, stride, pad))


def dims(N, C, H, W, K, R, S, stride, pad):
    """Derived sizes of one layer: P, Q and the im2col product M x Ngemm x Kgemm (Section 4.1)."""
    P, Q = out_dim(H, R, stride, pad), out_dim(W, S, stride, pad)
    M, Ng, Kg = N * P * Q, K, C * R * S
    return dict(P=P, Q=Q, M=M, Ngemm=Ng, Kgemm=Kg, flops=2 * M * Ng * Kg)


def conv2d(x, w, stride: int = 1, pad: int = 0) -> np.ndarray:
    """x NCHW, w KCRS -> y NKPQ, float64, direct from the definition."""
    x, w = _f64(x), _f64(w)
    N, C, H, W = x.shape
    K, C2, R, S = w.shape
    if C2 != C:
        raise ValueError("channel mismatch")
    P, Q = out_dim(H, R, stride, pad), out_dim(W, S, stride, pad)
    if P <= 0 or Q <= 0:
        raise ValueError("empty output")
    y = np.empty((N, K, P, Q), dtype=np.float64)
    _load().oracle_conv2d_f64(_p(x), _p(w), _p(y), N, C, H, W, K, R, S, stride, pad)
    return y


def conv2d_points(x, w, idx, stride: int = 1, pad: int = 0) -> np.ndarray:
    """Selected outputs only; idx is an (npts,4) array of (n,k,p,q)."""
    x, w = _f64(x), _f64(w)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    N, C, H, W = x.shape
    K, _, R, S = w.shape
    out = np.empty(idx.shape[0], dtype=np.float64)
    _load().oracle_conv2d_f64_points(_p(x), _p(w), idx.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                                     _p(out), idx.shape[0], N, C, H, W, K, R, S, stride, pad)
    return out


def maxpool2d(x, win: int = 3, stride: int = 2, pad: int = 1) -> np.ndarray:
    x = _f64(x)
    N, C, H, W = x.shape
    P, Q = out_dim(H, win, stride, pad), out_dim(W, win, stride, pad)
    y = np.empty((N, C, P, Q), dtype=np.float64)
    _load().oracle_maxpool2d_f64(_p(x), _p(y), N, C, H, W, win, stride, pad)
    return y


def relu(x) -> np.ndarray:
    return np.maximum(_f64(x), 0.0)


def round_bf16(x) -> np.ndarray:
    """Nearest bfloat16, ties to even, as float64."""
    x = _f64(x)
    y = np.empty_like(x)
    _load().oracle_round_bf16(_p(x), _p(y), x.size)
    return y


def conv_layer(x, w, stride, pad, residual=None, apply_relu=False) -> np.ndarray:
    """One step of a conv stack, unrounded: conv, then + residual, then ReLU, all float64."""
    y = conv2d(x, w, stride, pad)
    if residual is not None:
        y = y + _f64(residual)
    if apply_relu:
        y = relu(y)
    return y
