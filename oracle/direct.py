"""fp64 direct-sum oracle for fprop / bprop / accGrad (paper Sec. 2.1, Eqs. 1-3).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The GPU library never imports or calls this
module, and this module never imports the GPU package.

The arithmetic lives in ``direct_conv.c`` (plain nested loops in double
precision, no Fourier transform anywhere); this file only compiles that C file
with gcc when the shared object is absent and marshals numpy arrays to it.

Pins (tests that tie the oracle to something other than itself; all CPU-only):
hand-computed small cases, delta kernels (orientation and crop offset), k=1 and
k=n degenerate cases, all-ones closed forms, linearity, the adjoint identity,
per-map-pair agreement with scipy.signal correlate2d/convolve2d, whole-layer
agreement with torch conv2d and its autograd in fp64, and an independent
pure-Python loop nest on tiny shapes.  The numerical outputs on the random
benchmark layers themselves are not printed anywhere in the paper: parity there
rests on these pins.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "direct_conv.c")
_LIB = os.path.join(_HERE, "liboracle_direct.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile direct_conv.c into liboracle_direct.so (gcc, OpenMP, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O3", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off",
               "-fno-fast-math", "-std=c11", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        dp = ctypes.POINTER(ctypes.c_double)
        lp = ctypes.POINTER(ctypes.c_long)
        for name in ("oracle_fprop", "oracle_bprop", "oracle_accgrad"):
            fn = getattr(lib, name)
            fn.restype = None
            fn.argtypes = [dp, dp, dp] + [ctypes.c_int] * 7 + [lp, ctypes.c_long]
        lib.oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads() -> int:
    """Number of OpenMP threads the oracle will use."""
    return int(_load().oracle_num_threads())


def _f64(a):
    return np.ascontiguousarray(np.asarray(a), dtype=np.float64)


def _dp(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _units(units):
    if units is None:
        return None, None, 0
    u = np.ascontiguousarray(np.asarray(units), dtype=np.int64)
    return u, u.ctypes.data_as(ctypes.POINTER(ctypes.c_long)), int(u.size)


def _pair(v):
    """An int (square) or a (height, width) pair."""
    if isinstance(v, (tuple, list)):
        h, w = v
        return int(h), int(w)
    return int(v), int(v)


def _dims(x_shape, w_shape):
    S, f, nh, nw = x_shape
    fo, f2, kh, kw = w_shape
    if f != f2 or kh > nh or kw > nw or min(S, f, fo, nh, nw, kh, kw) < 1:
        raise ValueError(f"inconsistent shapes x{tuple(x_shape)} w{tuple(w_shape)}")
    return S, f, fo, nh, nw, kh, kw


def _rot180(w):
    """Kernels with both spatial indices reversed: the true convolution with w is the
    cross-correlation with this (the other reading of the paper's "*")."""
    return np.ascontiguousarray(np.asarray(w)[..., ::-1, ::-1])


def fprop(x, w, units=None, true_conv=False):
    """Eq. (1): y[s,j] = sum_i x[s,i] (star) w[j,i], valid window, shape [S,fo,noh,now].

    ``units`` (optional) lists output maps s*fo+j; the result is then
    [len(units), noh, now] in list order.  ``true_conv``: read (star) as the true
    convolution (kernel index reversed) instead of the cross-correlation.
    """
    if true_conv:
        w = _rot180(w)
    x, w = _f64(x), _f64(w)
    S, f, fo, nh, nw, kh, kw = _dims(x.shape, w.shape)
    noh, now = nh - kh + 1, nw - kw + 1
    u, up, nu = _units(units)
    out = np.empty((nu, noh, now) if u is not None else (S, fo, noh, now), dtype=np.float64)
    _load().oracle_fprop(_dp(x), _dp(w), _dp(out), S, f, fo, nh, nw, kh, kw, up, nu)
    return out


def bprop(g, w, n, units=None, true_conv=False):
    """Eq. (2): dx[s,i] = sum_j g[s,j] (star) w[j,i] rotated, full window, shape [S,f,nh,nw].

    ``n`` is the input size: an int for square maps or (nh, nw).  ``units`` lists input maps s*f+i.
    """
    if true_conv:
        w = _rot180(w)
    g, w = _f64(g), _f64(w)
    fo, f, kh, kw = w.shape
    nh, nw = _pair(n)
    S = g.shape[0]
    noh, now = nh - kh + 1, nw - kw + 1
    if g.shape != (S, fo, noh, now):
        raise ValueError(f"g{g.shape} does not match w{w.shape} and n={n}")
    u, up, nu = _units(units)
    out = np.empty((nu, nh, nw) if u is not None else (S, f, nh, nw), dtype=np.float64)
    _load().oracle_bprop(_dp(g), _dp(w), _dp(out), S, f, fo, nh, nw, kh, kw, up, nu)
    return out


def accgrad(g, x, k, units=None, true_conv=False):
    """Eq. (3): dw[j,i] = sum_s g[s,j] (star) x[s,i], kh x kw window, shape [fo,f,kh,kw].

    ``k`` is the kernel size: an int for square kernels or (kh, kw).  ``units`` lists kernels j*f+i.
    ``true_conv``: the gradient with respect to the kernels of a true convolution, i.e. the same
    sums stored with both kernel indices reversed.
    """
    if true_conv:
        return _rot180(accgrad(g, x, k, units))
    g, x = _f64(g), _f64(x)
    S, f, nh, nw = x.shape
    kh, kw = _pair(k)
    fo = g.shape[1]
    noh, now = nh - kh + 1, nw - kw + 1
    if g.shape != (S, fo, noh, now):
        raise ValueError(f"g{g.shape} does not match x{x.shape} and k={k}")
    u, up, nu = _units(units)
    out = np.empty((nu, kh, kw) if u is not None else (fo, f, kh, kw), dtype=np.float64)
    _load().oracle_accgrad(_dp(g), _dp(x), _dp(out), S, f, fo, nh, nw, kh, kw, up, nu)
    return out
