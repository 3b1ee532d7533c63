"""ctypes loader for the C direct-convolution oracle (test infrastructure only)."""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "direct_conv.c")
_LIB = os.path.join(_HERE, "liboracle_direct.so")
_lib = None


def build_direct(force: bool = False) -> str:
    """Compile direct_conv.c with gcc (baseline x86-64 so the object runs on any host)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O3", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build_direct()
        lib = ctypes.CDLL(_LIB)
        lib.oracle_direct_conv2d.argtypes = [ctypes.c_void_p] * 3 + [ctypes.c_int] * 7
        lib.oracle_direct_conv2d.restype = None
        lib.oracle_requant_shift_clamp.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int]
        lib.oracle_requant_shift_clamp.restype = None
        lib.oracle_maxpool2x2.argtypes = [ctypes.c_void_p, ctypes.c_void_p] + [ctypes.c_int] * 3
        lib.oracle_maxpool2x2.restype = None
        _lib = lib
    return _lib


def num_threads() -> int:
    """Threads the OpenMP loops will use (OMP_NUM_THREADS, else the visible cores)."""
    env = os.environ.get("OMP_NUM_THREADS")
    if env:
        try:
            return max(1, int(env.split(",")[0]))
        except ValueError:
            pass
    try:
        return len(os.sched_getaffinity(0))
    except AttributeError:
        return os.cpu_count() or 1


def direct_conv2d(x: np.ndarray, w: np.ndarray, pad: int) -> np.ndarray:
    """y[n,k,oy,ox] = sum_{c,i,j} xpad[n,c,oy+i-pad,ox+j-pad] * w[k,c,i,j], int32, stride 1."""
    assert x.dtype == np.int8 and w.dtype == np.int8 and x.ndim == 4 and w.ndim == 4
    N, C, H, W = x.shape
    K, C2, r, r2 = w.shape
    assert C == C2 and r == r2
    Ho, Wo = H + 2 * pad - r + 1, W + 2 * pad - r + 1
    assert Ho > 0 and Wo > 0
    x = np.ascontiguousarray(x)
    w = np.ascontiguousarray(w)
    y = np.empty((N, K, Ho, Wo), dtype=np.int32)
    _load().oracle_direct_conv2d(x.ctypes.data, w.ctypes.data, y.ctypes.data, N, C, K, H, W, r, pad)
    return y


def requant_shift_clamp(y: np.ndarray, shift: int) -> np.ndarray:
    """clamp(floor(y / 2^shift), -128, 127) as int8."""
    assert y.dtype == np.int32
    y = np.ascontiguousarray(y)
    a = np.empty(y.shape, dtype=np.int8)
    _load().oracle_requant_shift_clamp(y.ctypes.data, a.ctypes.data, y.size, shift)
    return a


def maxpool2x2(a: np.ndarray) -> np.ndarray:
    """2x2 stride-2 max-pool over the last two axes of an int8 array (even H, W)."""
    assert a.dtype == np.int8 and a.shape[-1] % 2 == 0 and a.shape[-2] % 2 == 0
    a = np.ascontiguousarray(a)
    H, W = a.shape[-2:]
    planes = a.size // (H * W)
    b = np.empty(a.shape[:-2] + (H // 2, W // 2), dtype=np.int8)
    _load().oracle_maxpool2x2(a.ctypes.data, b.ctypes.data, planes, H, W)
    return b
