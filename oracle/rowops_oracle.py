"""ctypes binding of rowops_oracle.c (plain C, fp64) -- test infrastructure only.

RMSNorm forward, LayerNorm forward and backward, rotary forward: the row-wise neighbours of
attention in the paper's kernel-suite table.  The arithmetic lives in rowops_oracle.c; this
file only marshals numpy arrays (activations as bf16 bit patterns in uint16, parameters and
tables in float32, results in float64).
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rowops_oracle.c")
_LIB = os.path.join(_HERE, "liboracle_rowops.so")
_lib = None


def build(force=False):
    """Compile rowops_oracle.c with gcc (OpenMP) into liboracle_rowops.so next to it."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        u16p, f32p, f64p = (ctypes.POINTER(t) for t in (ctypes.c_uint16, ctypes.c_float,
                                                        ctypes.c_double))
        L, F = ctypes.c_long, ctypes.c_float
        lib.oracle_rmsnorm_fwd.argtypes = [u16p, f32p, L, L, F, f64p]
        lib.oracle_layernorm_fwd.argtypes = [u16p, f32p, f32p, L, L, F, f64p, f64p, f64p]
        lib.oracle_layernorm_bwd.argtypes = [u16p, u16p, f32p, L, L, F, f64p, f64p, f64p]
        lib.oracle_rotary_fwd.argtypes = [u16p, f32p, f32p, L, L, L, f64p]
        for f in (lib.oracle_rmsnorm_fwd, lib.oracle_layernorm_fwd, lib.oracle_layernorm_bwd,
                  lib.oracle_rotary_fwd):
            f.restype = ctypes.c_int
        _lib = lib
    return _lib


def _u16(x, ndim):
    x = np.ascontiguousarray(x)
    if x.dtype != np.uint16 or x.ndim != ndim:
        raise TypeError("activations are bf16 bit patterns in uint16 arrays of %d dims" % ndim)
    return x


def _f32(x, shape):
    x = np.ascontiguousarray(x, dtype=np.float32)
    if x.shape != shape:
        raise ValueError("expected a float32 array of shape %r" % (shape,))
    return x


def _p(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct))


def _ok(rc, what):
    if rc != 0:
        raise RuntimeError("%s failed (rc=%d)" % (what, rc))


def rmsnorm_fwd(x, w, eps):
    """y [rows, cols] f64 = x * w / sqrt(mean(x^2, axis=1) + eps)."""
    x = _u16(x, 2); rows, cols = x.shape; w = _f32(w, (cols,))
    y = np.empty((rows, cols), np.float64)
    _ok(_load().oracle_rmsnorm_fwd(_p(x, ctypes.c_uint16), _p(w, ctypes.c_float), rows, cols,
                                   ctypes.c_float(np.float32(eps)), _p(y, ctypes.c_double)),
        "oracle_rmsnorm_fwd")
    return y


def layernorm_fwd(x, w, b, eps):
    """y [rows, cols], mean [rows], rstd [rows] (f64); biased variance."""
    x = _u16(x, 2); rows, cols = x.shape; w = _f32(w, (cols,)); b = _f32(b, (cols,))
    y = np.empty((rows, cols), np.float64)
    mean, rstd = np.empty(rows, np.float64), np.empty(rows, np.float64)
    _ok(_load().oracle_layernorm_fwd(_p(x, ctypes.c_uint16), _p(w, ctypes.c_float),
                                     _p(b, ctypes.c_float), rows, cols,
                                     ctypes.c_float(np.float32(eps)), _p(y, ctypes.c_double),
                                     _p(mean, ctypes.c_double), _p(rstd, ctypes.c_double)),
        "oracle_layernorm_fwd")
    return y, mean, rstd


def layernorm_bwd(dy, x, w, eps):
    """dx [rows, cols], dw [cols], db [cols] (f64) for upstream gradient dy on y."""
    x = _u16(x, 2); rows, cols = x.shape; dy = _u16(dy, 2); w = _f32(w, (cols,))
    if dy.shape != x.shape:
        raise ValueError("dy and x must have one shape")
    dx = np.empty((rows, cols), np.float64)
    dw, db = np.empty(cols, np.float64), np.empty(cols, np.float64)
    _ok(_load().oracle_layernorm_bwd(_p(dy, ctypes.c_uint16), _p(x, ctypes.c_uint16),
                                     _p(w, ctypes.c_float), rows, cols,
                                     ctypes.c_float(np.float32(eps)), _p(dx, ctypes.c_double),
                                     _p(dw, ctypes.c_double), _p(db, ctypes.c_double)),
        "oracle_layernorm_bwd")
    return dx, dw, db


def rotary_fwd(x, cos, sin):
    """y [B,H,S,D] f64: rotate-half pairing (d, d + D/2) by the angles of cos/sin [S, D/2]."""
    x = _u16(x, 4); B, H, S, D = x.shape
    cos = _f32(cos, (S, D // 2)); sin = _f32(sin, (S, D // 2))
    y = np.empty((B, H, S, D), np.float64)
    _ok(_load().oracle_rotary_fwd(_p(x, ctypes.c_uint16), _p(cos, ctypes.c_float),
                                  _p(sin, ctypes.c_float), B * H, S, D, _p(y, ctypes.c_double)),
        "oracle_rotary_fwd")
    return y
