"""CPU oracle for the convolution hot path.  TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It shares no code with the HIP library
and never imports it.

Contents
  conv_direct.c   float64 convolution straight from the definition (C, OpenMP)
  cook_toom.py    exact-rational Winograd/Cook-Toom matrices for F(n, k)
  winograd.py     float64 Winograd convolution taken step by step (Section 3.3.1)
  memory_plan.py  checker for the memory pool of a chain of operators (Section 3.2)
  cost_model.py   the analytic scheme-selection cost (Section 3.2) and the
                  Strassen stop rule (Section 3.3.2)

Pins (tests/test_oracle_*.py): brute-force Python loops on tiny shapes, closed
forms (all-ones, unit impulse), k = 1 against a float64 matrix product, the
float64 library convolution of PyTorch on CPU, exact rational verification of
the transform identity, and the step-by-step Winograd against the definition.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "conv_direct.c")
_LIB = os.path.join(_HERE, "liboracle_conv.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile conv_direct.c with gcc (-O2, OpenMP) into oracle/liboracle_conv.so."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i64 = ctypes.c_int64
        vp = ctypes.c_void_p
        lib.oracle_conv2d_f64.restype = ctypes.c_int
        lib.oracle_conv2d_f64.argtypes = [vp, vp, vp, vp] + [i64] * 13
        lib.oracle_conv2d_f64_points.restype = ctypes.c_int
        lib.oracle_conv2d_f64_points.argtypes = [vp, vp, vp, vp, i64, vp] + [i64] * 13
        lib.oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _pair(v):
    if isinstance(v, (tuple, list)):
        return int(v[0]), int(v[1])
    return int(v), int(v)


def out_size(h, k, stride, pad, dil):
    return (h + 2 * pad - dil * (k - 1) - 1) // stride + 1


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def conv2d(x: np.ndarray, w: np.ndarray, b: Optional[np.ndarray], stride=1, pad=0, dil=1) -> np.ndarray:
    """float64 convolution of float32 tensors x[N,C,H,W], w[K,C,kh,kw], b[K] or None."""
    lib = _load()
    x = np.ascontiguousarray(x, dtype=np.float32)
    w = np.ascontiguousarray(w, dtype=np.float32)
    bb = None if b is None else np.ascontiguousarray(b, dtype=np.float32)
    N, C, H, W = x.shape
    K, C2, kh, kw = w.shape
    assert C == C2, "channel mismatch"
    sh, sw = _pair(stride)
    ph, pw = _pair(pad)
    dh, dw = _pair(dil)
    Ho, Wo = out_size(H, kh, sh, ph, dh), out_size(W, kw, sw, pw, dw)
    y = np.empty((N, K, Ho, Wo), dtype=np.float64)
    rc = lib.oracle_conv2d_f64(x.ctypes.data, w.ctypes.data, None if bb is None else bb.ctypes.data,
                               y.ctypes.data, N, C, H, W, K, kh, kw, sh, sw, ph, pw, dh, dw)
    if rc != 0:
        raise ValueError(f"oracle_conv2d_f64 rejected the shape (rc={rc})")
    return y


def conv2d_points(x, w, b, coords: np.ndarray, stride=1, pad=0, dil=1) -> np.ndarray:
    """The same definition at sampled output coordinates (rows of n,k,oy,ox)."""
    lib = _load()
    x = np.ascontiguousarray(x, dtype=np.float32)
    w = np.ascontiguousarray(w, dtype=np.float32)
    bb = None if b is None else np.ascontiguousarray(b, dtype=np.float32)
    coords = np.ascontiguousarray(coords, dtype=np.int64)
    assert coords.ndim == 2 and coords.shape[1] == 4
    N, C, H, W = x.shape
    K, _, kh, kw = w.shape
    sh, sw = _pair(stride)
    ph, pw = _pair(pad)
    dh, dw = _pair(dil)
    out = np.empty((coords.shape[0],), dtype=np.float64)
    rc = lib.oracle_conv2d_f64_points(x.ctypes.data, w.ctypes.data, None if bb is None else bb.ctypes.data,
                                      coords.ctypes.data, coords.shape[0], out.ctypes.data,
                                      N, C, H, W, K, kh, kw, sh, sw, ph, pw, dh, dw)
    if rc != 0:
        raise ValueError(f"oracle_conv2d_f64_points rejected the shape (rc={rc})")
    return out


def error_ratio(y: np.ndarray, ref: np.ndarray) -> float:
    """max|y - ref| / max|ref| over the whole tensor: the parity metric."""
    ref = np.asarray(ref, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    denom = float(np.max(np.abs(ref))) if ref.size else 0.0
    if ref.size == 0:
        return 0.0
    if denom == 0.0:
        return float(np.max(np.abs(y - ref)))
    return float(np.max(np.abs(y - ref))) / denom
