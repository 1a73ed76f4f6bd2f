"""ORACLE — test infrastructure only.

Slow, plain CPU reference for the operator the paper accelerates (Section
"Techniques": the 3x3 2-D convolution operator, replaced by a Winograd path).
Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It shares no code with the HIP library
and never imports it.

  conv2d_direct      fp64 direct cross-correlation (C, OpenMP) — the definition.
  conv2d_direct_at   the same sum for selected output elements only.
  conv2d_general     fp64 direct cross-correlation, R x R filter, stride, padding (C, OpenMP).
  winograd_ref       fp64 numpy Winograd algorithm, step by step (stage checks).

Every function is pinned by ``tests/test_oracle_pins.py`` (hand cases, exact
rational identities, closed forms, invariants, a library routine).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "conv2d_direct.c")
_SRC_GENERAL = os.path.join(_HERE, "conv2d_general.c")
_LIB = os.path.join(_HERE, "liboracle_conv2d.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (no GPU toolchain involved)."""
    newest = max(os.path.getmtime(_SRC), os.path.getmtime(_SRC_GENERAL))
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < newest:
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99",
               "-o", _LIB, _SRC, _SRC_GENERAL]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int64)
        lib.oracle_conv2d_f64.restype = ctypes.c_int
        lib.oracle_conv2d_f64.argtypes = [dp, dp, dp, dp] + [ctypes.c_int] * 5
        lib.oracle_conv2d_f64_at.restype = ctypes.c_int
        lib.oracle_conv2d_f64_at.argtypes = [dp, dp, dp, ip, ctypes.c_int64, dp] + [ctypes.c_int] * 5
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_conv2d_general_f64.restype = ctypes.c_int
        lib.oracle_conv2d_general_f64.argtypes = [dp, dp, dp, dp] + [ctypes.c_int] * 8
        _lib = lib
    return _lib


def _f64(a, shape=None):
    a = np.ascontiguousarray(np.asarray(a), dtype=np.float64)  # fp16/fp32 promote exactly
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError(f"expected shape {shape}, got {a.shape}")
    return a


def _ptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def conv2d_direct(x, w, bias=None) -> np.ndarray:
    """y[N,K,H,W] (fp64) from x[N,C,H,W], w[K,C,3,3], bias[K] or None.

    Inputs of any float dtype are promoted exactly to fp64 first, so input
    quantisation is not part of the error budget.
    """
    x = _f64(x)
    N, C, H, W = x.shape
    w = _f64(w)
    K = w.shape[0]
    if w.shape != (K, C, 3, 3):
        raise ValueError(f"w must be [K,{C},3,3], got {w.shape}")
    b = None if bias is None else _f64(bias, (K,))
    y = np.empty((N, K, H, W), dtype=np.float64)
    rc = _load().oracle_conv2d_f64(_ptr(x), _ptr(w), None if b is None else _ptr(b), _ptr(y),
                                   N, C, H, W, K)
    if rc != 0:
        raise RuntimeError("oracle_conv2d_f64 rejected its arguments")
    return y


def conv2d_general(x, w, bias=None, stride: int = 1, pad: int = None) -> np.ndarray:
    """y[N,K,Ho,Wo] (fp64) from x[N,C,H,W], w[K,C,R,R], bias[K] or None; pad defaults to (R-1)//2."""
    x = _f64(x)
    N, C, H, W = x.shape
    w = _f64(w)
    K, R = w.shape[0], w.shape[2]
    if w.shape != (K, C, R, R):
        raise ValueError(f"w must be [K,{C},R,R], got {w.shape}")
    if pad is None:
        pad = (R - 1) // 2
    b = None if bias is None else _f64(bias, (K,))
    Ho, Wo = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - R) // stride + 1
    y = np.empty((N, K, Ho, Wo), dtype=np.float64)
    rc = _load().oracle_conv2d_general_f64(_ptr(x), _ptr(w), None if b is None else _ptr(b), _ptr(y),
                                           N, C, H, W, K, R, stride, pad)
    if rc != 0:
        raise RuntimeError("oracle_conv2d_general_f64 rejected its arguments")
    return y


def conv2d_direct_at(x, w, bias, flat_idx) -> np.ndarray:
    """The elements y.ravel()[flat_idx] of conv2d_direct, computed one by one."""
    x = _f64(x)
    N, C, H, W = x.shape
    w = _f64(w)
    K = w.shape[0]
    if w.shape != (K, C, 3, 3):
        raise ValueError(f"w must be [K,{C},3,3], got {w.shape}")
    b = None if bias is None else _f64(bias, (K,))
    idx = np.ascontiguousarray(np.asarray(flat_idx), dtype=np.int64)
    out = np.empty(idx.shape, dtype=np.float64)
    rc = _load().oracle_conv2d_f64_at(
        _ptr(x), _ptr(w), None if b is None else _ptr(b),
        idx.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), idx.size, _ptr(out),
        N, C, H, W, K)
    if rc != 0:
        raise RuntimeError("oracle_conv2d_f64_at rejected its arguments")
    return out


def rel_l2(y, y_ref) -> float:
    """||y - y_ref||_2 / ||y_ref||_2 over the whole tensor, in fp64."""
    y = np.asarray(y, dtype=np.float64).ravel()
    r = np.asarray(y_ref, dtype=np.float64).ravel()
    den = float(np.linalg.norm(r))
    if den == 0.0:
        raise ValueError("reference is all zero; compare exactly instead")
    return float(np.linalg.norm(y - r)) / den
