"""TEST INFRASTRUCTURE ONLY: loader for the C convolution oracle (conv_ref.c).

The arithmetic lives in conv_ref.c (paper Sec. 2.2 / Sec. 4.2: inner product of a kernel
tensor with a sliding input window).  This module only compiles that file with the host C
compiler and marshals numpy arrays into it.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "conv_ref.c")
_LIB = os.path.join(_HERE, "libconvref.so")
_lib = None


def build(force=False):
    """Compile conv_ref.c with gcc (never hipcc).  Rebuilds when the source is newer."""
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-o", _LIB, _SRC]
    subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i = ctypes.c_int
        lib.conv_ref_f64.restype = i
        lib.conv_ref_f64.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p] + [i] * 9
        lib.conv_ref_points_f64.restype = i
        lib.conv_ref_points_f64.argtypes = ([ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                             ctypes.c_int64, ctypes.c_void_p] + [i] * 9)
        _lib = lib
    return _lib


def out_extent(H, W, R, S, stride, pad):
    """Output height and width: floor((extent + 2 pad - kernel)/stride) + 1."""
    return (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1


def conv_ref(x, w, stride=1, pad=0, return_threads=False):
    """y[n,k,p,q] = sum_{c,r,s} xpad[n,c,p*stride+r-pad,q*stride+s-pad] * w[k,c,r,s]  (fp64 result)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    w = np.ascontiguousarray(w, dtype=np.float32)
    N, C, H, W = x.shape
    K, C2, R, S = w.shape
    if C2 != C:
        raise ValueError("channel mismatch")
    P, Q = out_extent(H, W, R, S, stride, pad)
    if P < 1 or Q < 1:
        raise ValueError("empty output")
    y = np.empty((N, K, P, Q), dtype=np.float64)
    rc = _load().conv_ref_f64(x.ctypes.data, w.ctypes.data, y.ctypes.data,
                              N, C, H, W, K, R, S, stride, pad)
    if rc < 0:
        raise ValueError("conv_ref_f64 rejected the arguments")
    return (y, rc) if return_threads else y


def conv_ref_points(x, w, idx, stride=1, pad=0):
    """The same definition at chosen outputs only; idx is an (M,4) array of (n,k,p,q)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    w = np.ascontiguousarray(w, dtype=np.float32)
    idx = np.ascontiguousarray(idx, dtype=np.int32).reshape(-1, 4)
    N, C, H, W = x.shape
    K, C2, R, S = w.shape
    if C2 != C:
        raise ValueError("channel mismatch")
    out = np.empty(idx.shape[0], dtype=np.float64)
    rc = _load().conv_ref_points_f64(x.ctypes.data, w.ctypes.data, idx.ctypes.data, idx.shape[0],
                                     out.ctypes.data, N, C, H, W, K, R, S, stride, pad)
    if rc < 0:
        raise ValueError("conv_ref_points_f64 rejected the arguments")
    return out


def conv_ref_hwc(x_hwc, w, stride=1, pad=0):
    """The same definition for tensors stored channels-innermost (the HWC layout of Table 1,
    Sec. 6.2): x_hwc[n,h,w,c], result y[n,p,q,k]; w stays [k,c,r,s].  Only the index order
    differs, so the tensors are permuted around conv_ref."""
    x = np.ascontiguousarray(np.transpose(np.asarray(x_hwc), (0, 3, 1, 2)))
    y = conv_ref(x, w, stride, pad)
    return np.ascontiguousarray(np.transpose(y, (0, 2, 3, 1)))


def conv_ref_cwh(x_cwh, w, stride=1, pad=0):
    """The same definition for images stored with the W axis before the H axis (the CWH layout of Table 1,
    Sec. 6.2): x_cwh[n,c,w,h], result y[n,k,q,p]; w stays [k,c,r,s].  Only the index order differs, so the
    tensors are permuted around conv_ref."""
    x = np.ascontiguousarray(np.transpose(np.asarray(x_cwh), (0, 1, 3, 2)))
    y = conv_ref(x, w, stride, pad)
    return np.ascontiguousarray(np.transpose(y, (0, 1, 3, 2)))
