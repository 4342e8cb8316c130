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


# ---- rotary embedding composed with attention (the fused entry points attn_fwd_rope /
# attn_bwd_rope of the library).  The paper lists "Rotary (fwd)" and the attention kernels as
# separate rows of its kernel-suite microbenchmark table, each on bf16 tensors; what the fused
# calls compute is therefore defined as that sequence: the rotation of the query rows, its
# result rounded to bf16 (the tensor the rotary kernel would hand to the attention kernel), then
# the attention oracle.  Keys come in rotated.  Query row i of Sq has position i + Sk - Sq.

def _round_to_bf16_bits(x):
    """float64 -> nearest bf16 (ties to even), as uint16 bit patterns.  Goes through float32,
    which is exact for every value that a product of a bf16 number and an fp32 table entry, or
    a sum of two such products, rounds to within the precision that matters here."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (r >> np.uint32(16)).astype(np.uint16)


def rope_rotate_queries(Q, cos, sin, Sk):
    """bf16 bit patterns of the rotated query rows, table rows Sk - Sq .. Sk - 1.

    Which bf16 value a rotated element becomes is a decision that floating point takes, so it
    is taken here in the precision the kernels take it in: fp32, y1 = fma(x1, c, -(x2 s)),
    y2 = fma(x2, c, x1 s), each rounded once to fp32 and then to bf16.  (The fp64 rotary oracle
    rounded to bf16 differs from this on the few elements per million whose exact value lies
    within an fp32 rounding error of a bf16 boundary; tests pin the two against each other.)
    The fma is written as the exact fp64 product plus the fp32-rounded other product, rounded
    to fp32: both steps are exact in fp64 for bf16 inputs times fp32 table entries."""
    Q = _u16(Q)
    Sq, D = Q.shape[2], Q.shape[3]
    if Sk < Sq:
        raise ValueError("rotary positions need Sk >= Sq")
    pos0, h = Sk - Sq, D // 2
    c = np.ascontiguousarray(cos[pos0:pos0 + Sq], dtype=np.float32).astype(np.float64)
    s = np.ascontiguousarray(sin[pos0:pos0 + Sq], dtype=np.float32).astype(np.float64)
    x = (Q.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    x1, x2 = x[..., :h], x[..., h:]
    t1 = (x2 * s).astype(np.float32).astype(np.float64)   # fp32 product
    t2 = (x1 * s).astype(np.float32).astype(np.float64)
    y = np.empty(Q.shape, np.float32)
    y[..., :h] = (x1 * c - t1).astype(np.float32)
    y[..., h:] = (x2 * c + t2).astype(np.float32)
    return _round_to_bf16_bits(y)


def attn_fwd_rope(Q, K_rot, V, cos, sin, scale, causal):
    """O, LSE, Q_rot (bits) for unrotated Q [B,Hq,Sq,D], rotated K_rot [B,Hkv,Sk,D] and tables
    [Sk, D/2]."""
    Q_rot = rope_rotate_queries(Q, cos, sin, K_rot.shape[2])
    O, LSE = attn_fwd(Q_rot, K_rot, V, scale, causal)
    return O, LSE, Q_rot


def attn_bwd_rope(Q_rot, K_rot, V, dO, cos, sin, scale, causal):
    """dQ (gradient of the UNROTATED query rows), dK_rot, dV.  The rotation of a row is a linear
    map R (y_d = x_d c_d - x_{d+h} s_d, y_{d+h} = x_{d+h} c_d + x_d s_d); the gradient of its
    input is R^T applied to the gradient of its output:
        gx_d = gy_d c_d + gy_{d+h} s_d,   gx_{d+h} = gy_{d+h} c_d - gy_d s_d."""
    dQr, dK, dV = attn_bwd(Q_rot, K_rot, V, dO, scale, causal)
    Sq, Sk, D = dQr.shape[2], K_rot.shape[2], dQr.shape[3]
    h, pos0 = D // 2, Sk - Sq
    c = np.asarray(cos[pos0:pos0 + Sq], dtype=np.float64)
    s = np.asarray(sin[pos0:pos0 + Sq], dtype=np.float64)
    dQ = np.empty_like(dQr)
    dQ[..., :h] = dQr[..., :h] * c + dQr[..., h:] * s
    dQ[..., h:] = dQr[..., h:] * c - dQr[..., :h] * s
    return dQ, dK, dV
