"""ctypes binding of attn_oracle.c (plain C, fp64) -- test infrastructure only.

The arithmetic lives in attn_oracle.c; this file only marshals numpy arrays.  Inputs are
bf16 bit patterns held in numpy uint16 arrays of shape [B,H,S,D] (C-contiguous); outputs
are float64.  See attn_oracle.c for the definition that is implemented (textbook scaled
dot-product attention in the natural-log, max-stabilised form; the paper's kernel-suite
section names the operator, its debugging table fixes the log base).
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "attn_oracle.c")
_LIB = os.path.join(_HERE, "liboracle_attn.so")
_lib = None


def build(force=False):
    """Compile attn_oracle.c with gcc (OpenMP) into liboracle_attn.so next to it."""
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
        u16p = ctypes.POINTER(ctypes.c_uint16)
        f64p = ctypes.POINTER(ctypes.c_double)
        i = ctypes.c_int
        lib.oracle_attn_fwd_rect.argtypes = [u16p, u16p, u16p, i, i, i, i, i, i, ctypes.c_float, i,
                                             i, f64p, f64p, f64p]
        lib.oracle_attn_fwd_rect.restype = i
        lib.oracle_attn_bwd_rect.argtypes = [u16p, u16p, u16p, u16p, i, i, i, i, i, i,
                                             ctypes.c_float, i, i, f64p, f64p, f64p, f64p]
        lib.oracle_attn_bwd_rect.restype = i
        lib.oracle_f16_to_f64.argtypes = [ctypes.c_uint16]
        lib.oracle_f16_to_f64.restype = ctypes.c_double
        lib.oracle_num_threads.argtypes = []
        lib.oracle_num_threads.restype = i
        _lib = lib
    return _lib


def num_threads():
    """OpenMP threads the oracle will use (omp_get_max_threads)."""
    return int(_load().oracle_num_threads())


def _u16(x, shape=None):
    x = np.ascontiguousarray(x)
    if x.dtype != np.uint16:
        raise TypeError("oracle inputs are bf16 bit patterns in uint16 arrays")
    if x.ndim != 4 or (shape is not None and x.shape != shape):
        raise ValueError("oracle inputs must all be [B,H,S,D] of one shape")
    return x


def _kv(x, qshape):
    """K or V: [B,Hkv,Sk,D] with Hkv dividing the query head count (Hkv = H: multi-head);
    Sk may differ from the query length (rectangular attention)."""
    x = _u16(x)
    B, H, S, D = qshape
    if x.shape[0] != B or x.shape[3] != D or x.shape[1] < 1 or H % x.shape[1]:
        raise ValueError("K/V must be [B,Hkv,Sk,D] with Hkv dividing H")
    return x


def _p(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct)) if a is not None else None


_DTYPES = {"bf16": 0, "f16": 1}


def f16_to_f64(h):
    """The oracle's own widening of one IEEE fp16 bit pattern (exposed so it can be pinned)."""
    return float(_load().oracle_f16_to_f64(int(h)))


def attn_fwd(Q, K, V, scale, causal, want_probs=False, dtype="bf16"):
    """O [B,H,Sq,D] f64, LSE [B,H,Sq] f64 (natural log) [, P [B,H,Sq,Sk] f64].
    K, V: [B,Hkv,Sk,D]; query head h reads K/V head h // (H // Hkv).  With causal=True and
    Sk > Sq the mask is aligned bottom-right: row i sees keys 0 .. i + Sk - Sq.  `dtype` says
    how the uint16 inputs are to be read: "bf16" or "f16" (IEEE half)."""
    Q = _u16(Q); K = _kv(K, Q.shape); V = _u16(V, K.shape)
    B, H, S, D = Q.shape
    Hkv, Sk = K.shape[1], K.shape[2]
    O = np.empty((B, H, S, D), np.float64)
    LSE = np.empty((B, H, S), np.float64)
    P = np.empty((B, H, S, Sk), np.float64) if want_probs else None
    rc = _load().oracle_attn_fwd_rect(_p(Q, ctypes.c_uint16), _p(K, ctypes.c_uint16),
                                     _p(V, ctypes.c_uint16), B, H, Hkv, S, Sk, D,
                                     ctypes.c_float(np.float32(scale)), int(bool(causal)),
                                     _DTYPES[dtype], _p(O, ctypes.c_double), _p(LSE, ctypes.c_double),
                                     _p(P, ctypes.c_double))
    if rc != 0:
        raise RuntimeError("oracle_attn_fwd failed (rc=%d)" % rc)
    return (O, LSE, P) if want_probs else (O, LSE)


def attn_probs(Q, K, V, scale, causal):
    """The full probability matrix P [B,H,Sq,Sk] (zeros outside the mask); small shapes only."""
    return attn_fwd(Q, K, V, scale, causal, want_probs=True)[2]


def attn_bwd(Q, K, V, dO, scale, causal, want_dscores=False, dtype="bf16"):
    """dQ [B,H,Sq,D], dK, dV [B,Hkv,Sk,D] f64 [, dS [B,H,Sq,Sk] f64] for upstream gradient dO on O."""
    Q = _u16(Q); K = _kv(K, Q.shape); V = _u16(V, K.shape); dO = _u16(dO, Q.shape)
    B, H, S, D = Q.shape
    Hkv, Sk = K.shape[1], K.shape[2]
    dQ = np.empty((B, H, S, D), np.float64)
    dK = np.empty((B, Hkv, Sk, D), np.float64)
    dV = np.empty_like(dK)
    dS = np.empty((B, H, S, Sk), np.float64) if want_dscores else None
    rc = _load().oracle_attn_bwd_rect(_p(Q, ctypes.c_uint16), _p(K, ctypes.c_uint16),
                                     _p(V, ctypes.c_uint16), _p(dO, ctypes.c_uint16),
                                     B, H, Hkv, S, Sk, D, ctypes.c_float(np.float32(scale)),
                                     int(bool(causal)), _DTYPES[dtype], _p(dQ, ctypes.c_double),
                                     _p(dK, ctypes.c_double), _p(dV, ctypes.c_double),
                                     _p(dS, ctypes.c_double))
    if rc != 0:
        raise RuntimeError("oracle_attn_bwd failed (rc=%d)" % rc)
    return (dQ, dK, dV, dS) if want_dscores else (dQ, dK, dV)


def attn_dscores(Q, K, V, dO, scale, causal):
    """dS [B,H,Sq,Sk] = P * (dP - delta) (zeros outside the mask); small shapes only."""
    return attn_bwd(Q, K, V, dO, scale, causal, want_dscores=True)[3]
