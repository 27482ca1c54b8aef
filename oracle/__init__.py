"""ctypes front end of the CPU oracle (``conv_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
CPU-baseline leg of the benchmark, never by the product package.  It shares no
code with the HIP path.

All tensors are numpy float64 arrays in the logical layouts of Section II of
the paper: ``I[N,C,H,W]``, ``W[K,C,R,S]``, ``O[N,K,P,Q]``.  The functions are
the naive loop nests of Algorithms 1, 6 and 8 with zero padding added (see the
header of ``conv_oracle.c`` for the readings taken).  Wherever a function takes
``pad`` it is one value for both axes or a pair ``(pad_h, pad_w)``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "conv_oracle.c")
_LIB = os.path.join(_HERE, "libconv_oracle.so")
_lib = None


class _Shape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int)
                for n in ("N", "C", "K", "H", "W", "R", "S", "stride", "pad_h", "pad_w")]


def _pads(pad):
    """``pad`` is one value for both axes, or a pair (pad_h, pad_w)."""
    if isinstance(pad, (tuple, list)):
        ph, pw = pad
        return int(ph), int(pw)
    return int(pad), int(pad)


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2 -fopenmp); returns the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-std=c99", "-shared", "-fPIC", "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        sp = ctypes.POINTER(_Shape)
        for name in ("oracle_conv_fwd", "oracle_conv_bwd_data", "oracle_conv_upd"):
            fn = getattr(lib, name)
            fn.argtypes = [sp, dp, dp, dp]
            fn.restype = None
        lib.oracle_conv_upd_entries.argtypes = [sp, dp, dp, ctypes.c_int,
                                                ctypes.POINTER(ctypes.c_int), dp]
        lib.oracle_conv_upd_entries.restype = None
        lib.oracle_out_h.argtypes = [sp]
        lib.oracle_out_w.argtypes = [sp]
        lib.oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _f64(a, shape):
    a = np.ascontiguousarray(a, dtype=np.float64)
    if tuple(a.shape) != tuple(shape):
        raise ValueError("expected shape %r, got %r" % (tuple(shape), tuple(a.shape)))
    return a


def _ptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def out_hw(H, W, R, S, stride, pad):
    """Output extent P = floor((H + 2 pad_h - R)/stride) + 1, Q likewise with pad_w."""
    g = _Shape(1, 1, 1, H, W, R, S, stride, *_pads(pad))
    lib = _load()
    return lib.oracle_out_h(ctypes.byref(g)), lib.oracle_out_w(ctypes.byref(g))


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def fwd(I, Wt, stride=1, pad=0):
    """Algorithm 1.  I[N,C,H,W], Wt[K,C,R,S] -> O[N,K,P,Q]."""
    N, C, H, W = I.shape
    K, C2, R, S = Wt.shape
    if C2 != C:
        raise ValueError("channel mismatch")
    g = _Shape(N, C, K, H, W, R, S, stride, *_pads(pad))
    P, Q = out_hw(H, W, R, S, stride, pad)
    I = _f64(I, (N, C, H, W))
    Wt = _f64(Wt, (K, C, R, S))
    O = np.empty((N, K, P, Q), dtype=np.float64)
    _load().oracle_conv_fwd(ctypes.byref(g), _ptr(I), _ptr(Wt), _ptr(O))
    return O


def fwd_fused(I, Wt, stride=1, pad=0, bias=None, residual=None, relu=False, scale=None):
    """Algorithm 4 (Section II-G) with L() = per-channel scale (a normalisation layer applied
    with given statistics), bias add, residual add, ReLU, applied to each output element
    once its reduction is complete:
        O = L(scale[k] * conv(I, Wt) + bias[k] + residual[n,k,oj,oi]),  L = max(., 0) if relu.
    Written out with numpy on top of ``fwd``; all in float64."""
    O = fwd(I, Wt, stride, pad)
    if scale is not None:
        g = np.asarray(scale, dtype=np.float64)
        for k in range(O.shape[1]):
            O[:, k, :, :] *= g[k]
    if bias is not None:
        b = np.asarray(bias, dtype=np.float64)
        for k in range(O.shape[1]):
            O[:, k, :, :] += b[k]
    if residual is not None:
        O = O + np.asarray(residual, dtype=np.float64)
    if relu:
        O = np.where(O > 0.0, O, 0.0)
    return O


def bwd_data(dO, Wt, H, W, stride=1, pad=0):
    """Algorithm 6.  dO[N,K,P,Q], Wt[K,C,R,S] -> dI[N,C,H,W]."""
    N, K, P, Q = dO.shape
    K2, C, R, S = Wt.shape
    if K2 != K:
        raise ValueError("channel mismatch")
    if (P, Q) != out_hw(H, W, R, S, stride, pad):
        raise ValueError("dO spatial extent does not match the geometry")
    g = _Shape(N, C, K, H, W, R, S, stride, *_pads(pad))
    dO = _f64(dO, (N, K, P, Q))
    Wt = _f64(Wt, (K, C, R, S))
    dI = np.empty((N, C, H, W), dtype=np.float64)
    _load().oracle_conv_bwd_data(ctypes.byref(g), _ptr(dO), _ptr(Wt), _ptr(dI))
    return dI


def upd(I, dO, R, S, stride=1, pad=0):
    """Algorithm 8.  I[N,C,H,W], dO[N,K,P,Q] -> dW[K,C,R,S]."""
    N, C, H, W = I.shape
    N2, K, P, Q = dO.shape
    if N2 != N or (P, Q) != out_hw(H, W, R, S, stride, pad):
        raise ValueError("dO does not match the geometry")
    g = _Shape(N, C, K, H, W, R, S, stride, *_pads(pad))
    I = _f64(I, (N, C, H, W))
    dO = _f64(dO, (N, K, P, Q))
    dW = np.empty((K, C, R, S), dtype=np.float64)
    _load().oracle_conv_upd(ctypes.byref(g), _ptr(I), _ptr(dO), _ptr(dW))
    return dW


def upd_entries(I, dO, R, S, stride, pad, entries):
    """Algorithm 8 for selected dW[k,c,r,s] only; ``entries`` is an (E,4) int array."""
    N, C, H, W = I.shape
    N2, K, P, Q = dO.shape
    if N2 != N or (P, Q) != out_hw(H, W, R, S, stride, pad):
        raise ValueError("dO does not match the geometry")
    e = np.ascontiguousarray(entries, dtype=np.int32).reshape(-1, 4)
    if e.size and (e.min() < 0 or (e.max(axis=0) >= np.array([K, C, R, S])).any()):
        raise ValueError("entry index out of range")
    g = _Shape(N, C, K, H, W, R, S, stride, *_pads(pad))
    I = _f64(I, (N, C, H, W))
    dO = _f64(dO, (N, K, P, Q))
    out = np.empty((e.shape[0],), dtype=np.float64)
    _load().oracle_conv_upd_entries(ctypes.byref(g), _ptr(I), _ptr(dO), e.shape[0],
                                    e.ctypes.data_as(ctypes.POINTER(ctypes.c_int)), _ptr(out))
    return out
