"""Thin ctypes binding of the row-wise entry points of include/rowops.h (RMSNorm forward,
LayerNorm forward and backward, rotary forward): argument marshalling only, every step runs
in the HIP kernels of libmi355attn.so."""
import ctypes

from .binding import ATTN_OK, AttnError, _stream_ptr, lib

EXPORTS = ("rowops_rmsnorm_fwd", "rowops_layernorm_fwd", "rowops_layernorm_bwd_workspace_bytes",
           "rowops_layernorm_bwd", "rowops_rotary_fwd")
_bound = False


def _lib():
    global _bound
    L = lib()
    if not _bound:
        vp, i32, i64, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float
        L.rowops_rmsnorm_fwd.argtypes = [vp, vp, vp, i64, i32, i64, i64, f32, vp]
        L.rowops_layernorm_fwd.argtypes = [vp, vp, vp, vp, vp, vp, i64, i32, i64, i64, f32, vp]
        L.rowops_layernorm_bwd_workspace_bytes.argtypes = [i64, i32]
        L.rowops_layernorm_bwd_workspace_bytes.restype = ctypes.c_size_t
        L.rowops_layernorm_bwd.argtypes = [vp] * 8 + [vp, ctypes.c_size_t, i64, i32, i64, i64, i64, vp]
        L.rowops_rotary_fwd.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32] + [i64] * 6 + [vp]
        for n in ("rowops_rmsnorm_fwd", "rowops_layernorm_fwd", "rowops_layernorm_bwd",
                  "rowops_rotary_fwd"):
            getattr(L, n).restype = ctypes.c_int
        _bound = True
    return L


def _rows(t, name):
    import torch
    if t.dtype != torch.bfloat16 or not t.is_cuda or t.dim() != 2 or t.stride(1) != 1:
        raise ValueError("%s must be a bf16 [rows, cols] GPU tensor with contiguous rows" % name)
    return t


def _f32(t, shape, name):
    import torch
    if t.dtype != torch.float32 or not t.is_cuda or not t.is_contiguous() or tuple(t.shape) != shape:
        raise ValueError("%s must be a contiguous fp32 GPU tensor of shape %r" % (name, shape))
    return t


def _check(rc, where):
    if rc != ATTN_OK:
        raise AttnError(rc, where)


def rmsnorm_fwd(x, w, eps, y=None, stream=None):
    import torch
    _rows(x, "x"); rows, cols = x.shape; _f32(w, (cols,), "w")
    y = torch.empty_like(x) if y is None else _rows(y, "y")
    _check(_lib().rowops_rmsnorm_fwd(x.data_ptr(), w.data_ptr(), y.data_ptr(), rows, cols,
                                     x.stride(0), y.stride(0), float(eps),
                                     _stream_ptr(torch, stream)), "rowops_rmsnorm_fwd")
    return y


def layernorm_fwd(x, w, b, eps, y=None, mean=None, rstd=None, stream=None):
    import torch
    _rows(x, "x"); rows, cols = x.shape; _f32(w, (cols,), "w"); _f32(b, (cols,), "b")
    y = torch.empty_like(x) if y is None else _rows(y, "y")
    mean = torch.empty(rows, dtype=torch.float32, device=x.device) if mean is None else mean
    rstd = torch.empty(rows, dtype=torch.float32, device=x.device) if rstd is None else rstd
    _f32(mean, (rows,), "mean"); _f32(rstd, (rows,), "rstd")
    _check(_lib().rowops_layernorm_fwd(x.data_ptr(), w.data_ptr(), b.data_ptr(), y.data_ptr(),
                                       mean.data_ptr(), rstd.data_ptr(), rows, cols, x.stride(0),
                                       y.stride(0), float(eps), _stream_ptr(torch, stream)),
           "rowops_layernorm_fwd")
    return y, mean, rstd


def layernorm_bwd_workspace_bytes(rows, cols):
    return int(_lib().rowops_layernorm_bwd_workspace_bytes(rows, cols))


def layernorm_bwd(dy, x, w, mean, rstd, dx=None, dw=None, db=None, workspace=None, stream=None):
    import torch
    _rows(x, "x"); _rows(dy, "dy"); rows, cols = x.shape
    if dy.shape != x.shape:
        raise ValueError("dy and x must have one shape")
    _f32(w, (cols,), "w"); _f32(mean, (rows,), "mean"); _f32(rstd, (rows,), "rstd")
    dx = torch.empty_like(x) if dx is None else _rows(dx, "dx")
    dw = torch.empty(cols, dtype=torch.float32, device=x.device) if dw is None else dw
    db = torch.empty(cols, dtype=torch.float32, device=x.device) if db is None else db
    _f32(dw, (cols,), "dw"); _f32(db, (cols,), "db")
    need = layernorm_bwd_workspace_bytes(rows, cols)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    _check(_lib().rowops_layernorm_bwd(dy.data_ptr(), x.data_ptr(), w.data_ptr(), mean.data_ptr(),
                                       rstd.data_ptr(), dx.data_ptr(), dw.data_ptr(), db.data_ptr(),
                                       workspace.data_ptr(),
                                       workspace.numel() * workspace.element_size(), rows, cols,
                                       dy.stride(0), x.stride(0), dx.stride(0),
                                       _stream_ptr(torch, stream)), "rowops_layernorm_bwd")
    return dx, dw, db


def rotary_fwd(x, cos, sin, y=None, stream=None):
    import torch
    if x.dtype != torch.bfloat16 or not x.is_cuda or x.dim() != 4 or x.stride(3) != 1:
        raise ValueError("x must be a bf16 [B,H,S,D] GPU tensor with a contiguous D axis")
    B, H, S, D = x.shape
    _f32(cos, (S, D // 2), "cos"); _f32(sin, (S, D // 2), "sin")
    if y is None:
        y = torch.empty_strided(x.shape, x.stride(), dtype=x.dtype, device=x.device)
    elif y.shape != x.shape or y.dtype != x.dtype or y.stride(3) != 1:
        raise ValueError("y must match x in shape and type")
    _check(_lib().rowops_rotary_fwd(x.data_ptr(), cos.data_ptr(), sin.data_ptr(), y.data_ptr(),
                                    B, H, S, D, *x.stride()[:3], *y.stride()[:3],
                                    _stream_ptr(torch, stream)), "rowops_rotary_fwd")
    return y
