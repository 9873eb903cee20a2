"""Python face of the fp64 CPU oracle (oracle/conv_oracle.c).

TEST INFRASTRUCTURE, NOT PRODUCT CODE: only tests/, the smoke check and the cpu_baseline leg of
bench.py may import this module.  It shares nothing with the GPU library and never imports it.

The arithmetic lives in conv_oracle.c (seven nested fp64 loops following the tensor roles of
Fig. 2 and the stride / dilation / padding descriptor of Sec. IV-A of the MIOpen paper, with the
bias + activation fusion of Sec. V and the conv + bias + batch-norm + activation row of Table I).
This file only builds that C file with gcc, loads it with ctypes and marshals numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "conv_oracle.c")
_LIB = os.path.join(_HERE, "libconv_oracle.so")

ACT_IDENTITY, ACT_RELU, ACT_LEAKY_RELU, ACT_TANH, ACT_LOGISTIC = 0, 1, 2, 3, 4

_lib = None


def build(force: bool = False) -> str:
    """Compile conv_oracle.c into libconv_oracle.so next to it (gcc, OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-o", tmp, _SRC, "-lm"]
        )
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int)
        ints = [ctypes.c_int] * 7 + [ctypes.c_int] * 6 + [ctypes.c_int, ctypes.c_int, ctypes.c_double]
        lib.conv_oracle_fwd.restype = ctypes.c_int
        lib.conv_oracle_fwd.argtypes = [dp, dp, dp, dp, ctypes.c_double, dp] + ints
        lib.conv_oracle_fwd_points.restype = ctypes.c_int
        lib.conv_oracle_fwd_points.argtypes = [dp, dp, dp, dp, ctypes.c_double, ip, ctypes.c_long, dp] + ints
        lib.conv_oracle_out_extent.restype = ctypes.c_int
        lib.conv_oracle_out_extent.argtypes = [ctypes.c_int] * 5
        lib.conv_oracle_threads.restype = ctypes.c_int
        lib.conv_oracle_threads.argtypes = []
        _lib = lib
    return _lib


def threads() -> int:
    """Number of OpenMP threads the oracle will use."""
    return int(_load().conv_oracle_threads())


def out_extent(size: int, filt: int, pad: int, stride: int, dil: int) -> int:
    return int(_load().conv_oracle_out_extent(size, filt, pad, stride, dil))


def _pair(v):
    if isinstance(v, (tuple, list)):
        a, b = v
        return int(a), int(b)
    return int(v), int(v)


def _f64(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float64)


def _ptr(a):
    dp = ctypes.POINTER(ctypes.c_double)
    return ctypes.cast(None, dp) if a is None else a.ctypes.data_as(dp)


def _bn_pack(bn, K):
    """bn = (gamma, beta, mean, var) each of K values -> one 4*K fp64 array, or None."""
    if bn is None:
        return None
    g, b, m, v = (np.asarray(t, dtype=np.float64).reshape(-1) for t in bn)
    assert g.size == b.size == m.size == v.size == K
    return np.ascontiguousarray(np.concatenate([g, b, m, v]))


def _dims(x, w, groups):
    N, C, H, W = x.shape
    K, Cg, R, S = w.shape
    if C % groups or K % groups or Cg != C // groups:
        raise ValueError("channel / group mismatch: x %s w %s groups %d" % (x.shape, w.shape, groups))
    return N, C, H, W, K, R, S


def conv_fwd(x, w, bias=None, *, pad=0, stride=1, dil=1, groups=1, act=ACT_IDENTITY, alpha=0.0,
             bn=None, eps=1e-5):
    """y = act(bn(conv(x, w) + bias)) in fp64.  x[N,C,H,W], w[K,C/groups,R,S], bias[K] or None."""
    x, w, bias = _f64(x), _f64(w), _f64(bias)
    N, C, H, W, K, R, S = _dims(x, w, groups)
    ph, pw = _pair(pad)
    sh, sw = _pair(stride)
    dh, dw = _pair(dil)
    Ho, Wo = out_extent(H, R, ph, sh, dh), out_extent(W, S, pw, sw, dw)
    if Ho < 1 or Wo < 1:
        raise ValueError("empty output")
    if bias is not None and bias.size != K:
        raise ValueError("bias must have K values")
    bnp = _bn_pack(bn, K)
    y = np.empty((N, K, Ho, Wo), dtype=np.float64)
    rc = _load().conv_oracle_fwd(_ptr(x), _ptr(w), _ptr(bias), _ptr(bnp), float(eps), _ptr(y),
                                 N, C, H, W, K, R, S, ph, pw, sh, sw, dh, dw, groups,
                                 int(act), float(alpha))
    if rc != 0:
        raise ValueError("conv_oracle_fwd rejected the parameters (rc=%d)" % rc)
    return y


def conv_fwd_points(x, w, bias, idx, *, pad=0, stride=1, dil=1, groups=1, act=ACT_IDENTITY,
                    alpha=0.0, bn=None, eps=1e-5):
    """Same definition, only at the outputs listed in idx (an int array of (n,k,p,q) rows)."""
    x, w, bias = _f64(x), _f64(w), _f64(bias)
    N, C, H, W, K, R, S = _dims(x, w, groups)
    ph, pw = _pair(pad)
    sh, sw = _pair(stride)
    dh, dw = _pair(dil)
    idx = np.ascontiguousarray(idx, dtype=np.int32).reshape(-1, 4)
    bnp = _bn_pack(bn, K)
    out = np.empty(idx.shape[0], dtype=np.float64)
    rc = _load().conv_oracle_fwd_points(
        _ptr(x), _ptr(w), _ptr(bias), _ptr(bnp), float(eps),
        idx.ctypes.data_as(ctypes.POINTER(ctypes.c_int)), idx.shape[0], _ptr(out),
        N, C, H, W, K, R, S, ph, pw, sh, sw, dh, dw, groups, int(act), float(alpha))
    if rc != 0:
        raise ValueError("conv_oracle_fwd_points rejected the parameters (rc=%d)" % rc)
    return out
