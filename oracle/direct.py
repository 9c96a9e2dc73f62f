"""TEST INFRASTRUCTURE ONLY: ctypes front for oracle/conv2d_direct.c.

conv2d by its definition (Fig. 5 step 1 / Fig. 1b / Table 2 access [n, i+k];
int8 operands, int32 accumulation, Sec. 5.1).  The shared object is compiled with
gcc on first use if it has not been built yet (building the checker is not using it).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "conv2d_direct.c")
_SO = os.path.join(_HERE, "liboracle_conv.so")
_lib = None


def build(force: bool = False) -> str:
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O3", "-fopenmp", "-shared", "-fPIC",
                               "-o", _SO, _SRC])
    return _SO


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.oracle_conv2d_int8.restype = ctypes.c_int
        lib.oracle_conv2d_int8.argtypes = [ctypes.c_int] * 9 + [ctypes.c_void_p] * 3
        lib.oracle_conv2d_int8_dilated.restype = ctypes.c_int
        lib.oracle_conv2d_int8_dilated.argtypes = [ctypes.c_int] * 10 + [ctypes.c_void_p] * 3
        lib.oracle_threads.restype = ctypes.c_int
        lib.oracle_set_threads.argtypes = [ctypes.c_int]
        _lib = lib
    return _lib


def threads() -> int:
    return _load().oracle_threads()


def set_threads(t: int) -> None:
    _load().oracle_set_threads(int(t))


def out_hw(H, W, R, S, stride, pad):
    return (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1


def conv2d_int8(x: np.ndarray, w: np.ndarray, stride: int, pad: int) -> np.ndarray:
    """x: [N,C,H,W] int8, w: [K,C,R,S] int8 -> [N,K,P,Q] int32."""
    assert x.dtype == np.int8 and w.dtype == np.int8
    N, C, H, W = x.shape
    K, C2, R, S = w.shape
    assert C == C2
    x = np.ascontiguousarray(x)
    w = np.ascontiguousarray(w)
    P, Q = out_hw(H, W, R, S, stride, pad)
    if P <= 0 or Q <= 0:
        raise ValueError("kernel larger than padded input")
    out = np.empty((N, K, P, Q), dtype=np.int32)
    rc = _load().oracle_conv2d_int8(N, C, H, W, K, R, S, stride, pad,
                                    x.ctypes.data, w.ctypes.data, out.ctypes.data)
    if rc != 0:
        raise ValueError("oracle_conv2d_int8: invalid arguments")
    return out


def out_hw_dilated(H, W, R, S, stride, pad, dilation):
    return ((H + 2 * pad - dilation * (R - 1) - 1) // stride + 1,
            (W + 2 * pad - dilation * (S - 1) - 1) // stride + 1)


def conv2d_int8_dilated(x: np.ndarray, w: np.ndarray, stride: int, pad: int, dilation: int) -> np.ndarray:
    """Dilated convolution (Sec. 6.1): x [N,C,H,W] int8, w [K,C,R,S] int8 -> [N,K,P,Q] int32,
    kernel tap (r, s) reading the padded input at (p*stride + r*dilation, q*stride + s*dilation)."""
    assert x.dtype == np.int8 and w.dtype == np.int8
    N, C, H, W = x.shape
    K, C2, R, S = w.shape
    assert C == C2
    x = np.ascontiguousarray(x)
    w = np.ascontiguousarray(w)
    P, Q = out_hw_dilated(H, W, R, S, stride, pad, dilation)
    if P <= 0 or Q <= 0:
        raise ValueError("spread kernel larger than padded input")
    out = np.empty((N, K, P, Q), dtype=np.int32)
    rc = _load().oracle_conv2d_int8_dilated(N, C, H, W, K, R, S, stride, pad, dilation,
                                            x.ctypes.data, w.ctypes.data, out.ctypes.data)
    if rc != 0:
        raise ValueError("oracle_conv2d_int8_dilated: invalid arguments")
    return out
