"""ctypes loader for the FP64 direct-summation oracle in ``conv1d_oracle.c``.

TEST INFRASTRUCTURE ONLY: the product path never imports this module.

The arithmetic lives in the C file (plain nested loops following Eq. 2 and
Algorithms 1, 3 and 4 of the paper, read as the adjoint triple of one bilinear
map); this file only compiles it with gcc, marshals numpy float64 arrays and
returns numpy float64 arrays.  Every function returns ``(value, abs_sum)`` when
``with_abs`` is true: ``abs_sum`` is the same sum over ``|product|`` and is the
denominator of the parity metric.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "conv1d_oracle.c")
_LIB = os.path.join(_HERE, "libconv1d_oracle.so")
_lib = None

_D = ctypes.POINTER(ctypes.c_double)
_I64 = ctypes.POINTER(ctypes.c_int64)
_L = ctypes.c_long


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O2 -fopenmp); returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        dims = [_L] * 7
        lib.conv1d_oracle_threads.restype = ctypes.c_int
        lib.conv1d_oracle_out_width.restype = _L
        lib.conv1d_oracle_out_width.argtypes = [_L] * 4
        for name in ("conv1d_oracle_fwd", "conv1d_oracle_bwd_data", "conv1d_oracle_bwd_weight"):
            fn = getattr(lib, name)
            fn.restype = None
            fn.argtypes = [_D, _D, _D, _D] + dims
        for name in ("conv1d_oracle_fwd_at", "conv1d_oracle_bwd_data_at",
                     "conv1d_oracle_bwd_weight_at"):
            fn = getattr(lib, name)
            fn.restype = None
            fn.argtypes = [_D, _D, _I64, _L, _D, _D] + dims
        lib.conv1d_oracle_round_bf16.restype = ctypes.c_double
        lib.conv1d_oracle_round_bf16.argtypes = [ctypes.c_double]
        lib.conv1d_oracle_epilogue.restype = None
        lib.conv1d_oracle_epilogue.argtypes = [_D, _D, _D, _L, _L, _L, ctypes.c_int, ctypes.c_int]
        _lib = lib
    return _lib


def threads() -> int:
    """Number of OpenMP threads the oracle will use."""
    return int(_load().conv1d_oracle_threads())


def out_width(W: int, S: int, d: int, P: int) -> int:
    """Q = W + 2P - (S-1)d  (stride 1; Section 2, Fig. 1)."""
    return int(_load().conv1d_oracle_out_width(W, S, d, P))


def _f64(a, shape):
    a = np.ascontiguousarray(a, dtype=np.float64)
    if a.shape != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {a.shape}")
    return a


def _p(a):
    return a.ctypes.data_as(_D) if a is not None else ctypes.cast(None, _D)


def _dims(x_shape, w_shape, d, P):
    N, C, W = x_shape
    K, C2, S = w_shape
    if C2 != C:
        raise ValueError("channel mismatch")
    Q = W + 2 * P - (S - 1) * d
    if min(N, C, K, W, S) < 1 or d < 1 or P < 0 or Q < 1:
        raise ValueError("invalid convolution geometry")
    return N, C, K, W, S, Q


def fwd(x, w, d: int, P: int, with_abs: bool = False):
    """Y[n,k,q] = sum_c sum_s X[n,c,q+s*d-P] * Wt[k,c,s]   (Eq. 2 / Algorithm 1)."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    w = np.ascontiguousarray(w, dtype=np.float64)
    N, C, K, W, S, Q = _dims(x.shape, w.shape, d, P)
    y = np.empty((N, K, Q), dtype=np.float64)
    ya = np.empty_like(y) if with_abs else None
    _load().conv1d_oracle_fwd(_p(x), _p(w), _p(y), _p(ya), N, C, K, W, S, d, P)
    return (y, ya) if with_abs else y


def bwd_data(dy, w, W: int, d: int, P: int, with_abs: bool = False):
    """dX[n,c,i] = sum_k sum_s Wt[k,c,s] * dY[n,k,i+P-s*d]   (Section 3.2)."""
    dy = np.ascontiguousarray(dy, dtype=np.float64)
    w = np.ascontiguousarray(w, dtype=np.float64)
    K, C, S = w.shape
    N = dy.shape[0]
    _, _, _, _, _, Q = _dims((N, C, W), w.shape, d, P)
    dy = _f64(dy, (N, K, Q))
    dx = np.empty((N, C, W), dtype=np.float64)
    da = np.empty_like(dx) if with_abs else None
    _load().conv1d_oracle_bwd_data(_p(dy), _p(w), _p(dx), _p(da), N, C, K, W, S, d, P)
    return (dx, da) if with_abs else dx


def bwd_weight(x, dy, S: int, d: int, P: int, with_abs: bool = False):
    """dW[k,c,s] = sum_n sum_q X[n,c,q+s*d-P] * dY[n,k,q]   (Section 3.3 / Algorithm 4)."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    dy = np.ascontiguousarray(dy, dtype=np.float64)
    N, C, W = x.shape
    K = dy.shape[1]
    _, _, _, _, _, Q = _dims(x.shape, (K, C, S), d, P)
    dy = _f64(dy, (N, K, Q))
    dw = np.empty((K, C, S), dtype=np.float64)
    da = np.empty_like(dw) if with_abs else None
    _load().conv1d_oracle_bwd_weight(_p(x), _p(dy), _p(dw), _p(da), N, C, K, W, S, d, P)
    return (dw, da) if with_abs else dw


def _idx(idx, bounds):
    idx = np.ascontiguousarray(idx, dtype=np.int64)
    if idx.ndim != 2 or idx.shape[1] != 3:
        raise ValueError("idx must be (count, 3)")
    if idx.size and ((idx < 0).any() or (idx >= np.asarray(bounds, dtype=np.int64)).any()):
        raise ValueError("sample coordinate out of range")
    return idx


def fwd_at(x, w, idx, d: int, P: int):
    """fwd at sampled (n,k,q) triples; returns (values, abs_sums)."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    w = np.ascontiguousarray(w, dtype=np.float64)
    N, C, K, W, S, Q = _dims(x.shape, w.shape, d, P)
    idx = _idx(idx, (N, K, Q))
    out = np.empty(len(idx), dtype=np.float64)
    oa = np.empty_like(out)
    _load().conv1d_oracle_fwd_at(_p(x), _p(w), idx.ctypes.data_as(_I64), len(idx), _p(out), _p(oa),
                                 N, C, K, W, S, d, P)
    return out, oa


def bwd_data_at(dy, w, idx, W: int, d: int, P: int):
    """bwd_data at sampled (n,c,i) triples; returns (values, abs_sums)."""
    dy = np.ascontiguousarray(dy, dtype=np.float64)
    w = np.ascontiguousarray(w, dtype=np.float64)
    K, C, S = w.shape
    N = dy.shape[0]
    _, _, _, _, _, Q = _dims((N, C, W), w.shape, d, P)
    dy = _f64(dy, (N, K, Q))
    idx = _idx(idx, (N, C, W))
    out = np.empty(len(idx), dtype=np.float64)
    oa = np.empty_like(out)
    _load().conv1d_oracle_bwd_data_at(_p(dy), _p(w), idx.ctypes.data_as(_I64), len(idx), _p(out),
                                      _p(oa), N, C, K, W, S, d, P)
    return out, oa


def bwd_weight_at(x, dy, idx, S: int, d: int, P: int):
    """bwd_weight at sampled (k,c,s) triples; returns (values, abs_sums)."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    dy = np.ascontiguousarray(dy, dtype=np.float64)
    N, C, W = x.shape
    K = dy.shape[1]
    _, _, _, _, _, Q = _dims(x.shape, (K, C, S), d, P)
    dy = _f64(dy, (N, K, Q))
    idx = _idx(idx, (K, C, S))
    out = np.empty(len(idx), dtype=np.float64)
    oa = np.empty_like(out)
    _load().conv1d_oracle_bwd_weight_at(_p(x), _p(dy), idx.ctypes.data_as(_I64), len(idx), _p(out),
                                        _p(oa), N, C, K, W, S, d, P)
    return out, oa


def round_bf16(v: float) -> float:
    """Nearest bfloat16 to a double, ties to even (the storage rounding of Section 4.4's BF16 layers)."""
    return float(_load().conv1d_oracle_round_bf16(float(v)))


def epilogue(y, bias=None, relu: bool = False, out_bf16: bool = False, yabs=None):
    """In place on y[N,K,width] (float64): + bias[k] (Section 3: the bias the framework adds), max(., 0) and bfloat16
    storage (Section 4.4: the BF16 ReLU that follows the layer).  yabs, when given, gains |bias[k]|."""
    if y.dtype != np.float64 or not y.flags.c_contiguous or y.ndim != 3:
        raise ValueError("y must be a contiguous float64 array [N, K, width]")
    N, K, width = y.shape
    b = None if bias is None else _f64(bias, (K,))
    if yabs is not None and (yabs.dtype != np.float64 or yabs.shape != y.shape or not yabs.flags.c_contiguous):
        raise ValueError("yabs must match y")
    _load().conv1d_oracle_epilogue(_p(y), _p(yabs), _p(b), N, K, width, int(bool(relu)), int(bool(out_bf16)))
    return y


def fwd_ex(x, w, d: int, P: int, bias=None, relu: bool = False, out_bf16: bool = False, with_abs: bool = False):
    """The forward pass followed by the epilogue: round_bf16?(relu?(fwd(x, w) + bias?))."""
    y, ya = fwd(x, w, d, P, with_abs=True)
    epilogue(y, bias, relu, out_bf16, ya)
    return (y, ya) if with_abs else y


def bwd_data_ex(dy, w, W: int, d: int, P: int, out_bf16: bool = False, with_abs: bool = False):
    """The backward-data pass with its result stored as bfloat16 (Section 4.4: gradients stay in BF16)."""
    dx, da = bwd_data(dy, w, W, d, P, with_abs=True)
    epilogue(dx, None, False, out_bf16, da)
    return (dx, da) if with_abs else dx
