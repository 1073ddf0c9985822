"""TEST INFRASTRUCTURE ONLY: ctypes front for the fp64 direct-convolution oracle.

The arithmetic lives in ``conv_oracle.c`` (Algorithm 1 and the gradient equation
of Section 2 of arXiv 1804.04806, written out as plain loops).  This module only
compiles that file with gcc, marshals numpy arrays, and offers the "run it on
slices" helpers that express the paper's micro-batching semantics (Section 2:
Forward and BackwardData divide directly; BackwardFilter repeats sequentially
with output scale 1).
"""
import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "conv_oracle.c")
_LIB = os.path.join(_HERE, "libconv_oracle.so")


def build(force=False):
    """Compile conv_oracle.c with gcc (-O2, OpenMP). Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99",
                               "-o", _LIB, _SRC])
    return _LIB


class _CLayer(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int64) for n in
                ("N", "C", "H", "W", "K", "R", "S", "sh", "sw", "ph", "pw")]


@dataclass(frozen=True)
class Layer:
    """Layer shape: X (N,C,H,W), filter (K,C,R,S), stride (sh,sw), zero padding (ph,pw)."""
    N: int
    C: int
    H: int
    W: int
    K: int
    R: int
    S: int
    sh: int = 1
    sw: int = 1
    ph: int = 0
    pw: int = 0

    @property
    def P(self):
        return (self.H + 2 * self.ph - self.R) // self.sh + 1

    @property
    def Q(self):
        return (self.W + 2 * self.pw - self.S) // self.sw + 1

    def with_batch(self, n):
        return Layer(n, self.C, self.H, self.W, self.K, self.R, self.S,
                     self.sh, self.sw, self.ph, self.pw)

    def _c(self):
        return _CLayer(self.N, self.C, self.H, self.W, self.K, self.R, self.S,
                       self.sh, self.sw, self.ph, self.pw)

    @property
    def x_shape(self):
        return (self.N, self.C, self.H, self.W)

    @property
    def w_shape(self):
        return (self.K, self.C, self.R, self.S)

    @property
    def y_shape(self):
        return (self.N, self.K, self.P, self.Q)


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int64)
        lp = ctypes.POINTER(_CLayer)
        lib.oc_threads.restype = ctypes.c_int
        lib.oc_conv_fwd.argtypes = [lp, dp, dp, dp]
        lib.oc_conv_bwd_data.argtypes = [lp, dp, dp, dp]
        lib.oc_conv_bwd_filter.argtypes = [lp, dp, dp, ctypes.c_double, dp]
        lib.oc_conv_fwd_at.argtypes = [lp, dp, dp, ip, ctypes.c_int64, dp]
        lib.oc_conv_bwd_data_at.argtypes = [lp, dp, dp, ip, ctypes.c_int64, dp]
        lib.oc_conv_bwd_filter_at.argtypes = [lp, dp, dp, ip, ctypes.c_int64, dp]
        for f in (lib.oc_conv_fwd, lib.oc_conv_bwd_data, lib.oc_conv_bwd_filter,
                  lib.oc_conv_fwd_at, lib.oc_conv_bwd_data_at, lib.oc_conv_bwd_filter_at):
            f.restype = None
        _lib = lib
    return _lib


def threads():
    """Number of host threads the C oracle runs on."""
    return int(_load().oc_threads())


def _d(a, shape):
    a = np.ascontiguousarray(a, dtype=np.float64)
    if a.shape != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {a.shape}")
    return a


def _p(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _i(idx):
    idx = np.ascontiguousarray(idx, dtype=np.int64)
    return idx, idx.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))


def conv_fwd(L, x, w):
    """Y = conv(X, W): Algorithm 1 with zero padding and stride."""
    x, w = _d(x, L.x_shape), _d(w, L.w_shape)
    y = np.empty(L.y_shape, dtype=np.float64)
    if y.size:
        _load().oc_conv_fwd(ctypes.byref(L._c()), _p(x), _p(w), _p(y))
    return y


def conv_bwd_data(L, dy, w):
    """dX: adjoint of Forward with respect to X."""
    dy, w = _d(dy, L.y_shape), _d(w, L.w_shape)
    dx = np.empty(L.x_shape, dtype=np.float64)
    if dx.size:
        _load().oc_conv_bwd_data(ctypes.byref(L._c()), _p(dy), _p(w), _p(dx))
    return dx


def conv_bwd_filter(L, x, dy, beta=0.0, dw=None):
    """dW = beta * dW + sum over samples (Section 2 gradient equation, no 1/N)."""
    x, dy = _d(x, L.x_shape), _d(dy, L.y_shape)
    if dw is None:
        out = np.zeros(L.w_shape, dtype=np.float64)
    else:
        out = np.array(_d(dw, L.w_shape), copy=True)
    _load().oc_conv_bwd_filter(ctypes.byref(L._c()), _p(x), _p(dy), float(beta), _p(out))
    return out


def conv_fwd_at(L, x, w, idx):
    """Forward at the flat output indices ``idx`` (each a full exact reduction)."""
    x, w = _d(x, L.x_shape), _d(w, L.w_shape)
    idx, ip = _i(idx)
    out = np.empty(idx.size, dtype=np.float64)
    _load().oc_conv_fwd_at(ctypes.byref(L._c()), _p(x), _p(w), ip, idx.size, _p(out))
    return out


def conv_bwd_data_at(L, dy, w, idx):
    dy, w = _d(dy, L.y_shape), _d(w, L.w_shape)
    idx, ip = _i(idx)
    out = np.empty(idx.size, dtype=np.float64)
    _load().oc_conv_bwd_data_at(ctypes.byref(L._c()), _p(dy), _p(w), ip, idx.size, _p(out))
    return out


def conv_bwd_filter_at(L, x, dy, idx):
    x, dy = _d(x, L.x_shape), _d(dy, L.y_shape)
    idx, ip = _i(idx)
    out = np.empty(idx.size, dtype=np.float64)
    _load().oc_conv_bwd_filter_at(ctypes.byref(L._c()), _p(x), _p(dy), ip, idx.size, _p(out))
    return out


# ---- micro-batching semantics (Section 2 / Section 3 of the paper) -----------------

def _offsets(L, parts):
    if sum(parts) != L.N or any(b <= 0 for b in parts):
        raise ValueError("micro-batch sizes must be positive and sum to N")
    o = 0
    for b in parts:
        yield o, b
        o += b


def micro_fwd(L, x, w, parts):
    """Forward run one micro-batch at a time on disjoint sample slices."""
    x = _d(x, L.x_shape)
    return np.concatenate([conv_fwd(L.with_batch(b), x[o:o + b], w) for o, b in _offsets(L, parts)])


def micro_bwd_data(L, dy, w, parts):
    dy = _d(dy, L.y_shape)
    return np.concatenate([conv_bwd_data(L.with_batch(b), dy[o:o + b], w) for o, b in _offsets(L, parts)])


def micro_bwd_filter(L, x, dy, parts, beta=0.0, dw=None):
    """BackwardFilter repeated sequentially: caller's beta first, output scale 1 afterwards."""
    x, dy = _d(x, L.x_shape), _d(dy, L.y_shape)
    acc = dw
    for i, (o, b) in enumerate(_offsets(L, parts)):
        acc = conv_bwd_filter(L.with_batch(b), x[o:o + b], dy[o:o + b],
                              beta=(beta if i == 0 else 1.0), dw=acc)
    return acc
