"""ctypes binding of libmi355attn.so -- argument marshalling only.

Every step of the attention path runs inside the HIP library; this file passes device
pointers of torch tensors (PyTorch is used for device memory and streams only) through the
C ABI declared in include/attn.h.  There is no CPU or PyTorch fallback: if the library has
not been built, loading fails with an error.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmi355attn.so")

ATTN_OK = 0
ATTN_ERR_NULL = -1
ATTN_ERR_SHAPE = -2
ATTN_ERR_STRIDE = -3
ATTN_ERR_ALIGN = -4
ATTN_ERR_WORKSPACE = -5
ATTN_ERR_SCALE = -6
ATTN_ERR_LAUNCH = -7

EXPORTS = ("attn_params_contiguous", "attn_fwd", "attn_bwd_workspace_bytes", "attn_bwd",
           "attn_bwd_stages", "attn_gqa_params_contiguous", "attn_fwd_gqa",
           "attn_bwd_gqa_workspace_bytes", "attn_bwd_gqa", "attn_bwd_gqa_stages",
           "attn_rect_params_contiguous", "attn_fwd_rect_workspace_bytes", "attn_fwd_rect",
           "attn_bwd_rect_workspace_bytes", "attn_bwd_rect", "attn_fwd_rect_f16",
           "attn_bwd_rect_f16", "attn_bwd_rect_noalloc", "attn_fwd_rope_workspace_bytes", "attn_fwd_rope",
           "attn_bwd_rope", "attn_probe_mfma_bf16",
           "attn_probe_atomic_f32", "attn_probe_stream",
           "attn_status_string", "attn_version")
NOALLOC_SCRATCH_BYTES = 8 << 20
STAGE_DELTA, STAGE_DKDV, STAGE_DQ = 1, 2, 4
STAGE_ALL = 7


class AttnParams(ctypes.Structure):
    """Mirror of attn_params_t."""
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("S", ctypes.c_int32),
                ("D", ctypes.c_int32), ("stride_b", ctypes.c_int64),
                ("stride_h", ctypes.c_int64), ("stride_s", ctypes.c_int64),
                ("scale", ctypes.c_float), ("causal", ctypes.c_int32)]


class AttnGqaParams(ctypes.Structure):
    """Mirror of attn_gqa_params_t."""
    _fields_ = [("B", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32),
                ("S", ctypes.c_int32), ("D", ctypes.c_int32),
                ("q_stride_b", ctypes.c_int64), ("q_stride_h", ctypes.c_int64),
                ("q_stride_s", ctypes.c_int64), ("kv_stride_b", ctypes.c_int64),
                ("kv_stride_h", ctypes.c_int64), ("kv_stride_s", ctypes.c_int64),
                ("scale", ctypes.c_float), ("causal", ctypes.c_int32)]


class AttnRectParams(ctypes.Structure):
    """Mirror of attn_rect_params_t."""
    _fields_ = [("B", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32),
                ("Sq", ctypes.c_int32), ("Sk", ctypes.c_int32), ("D", ctypes.c_int32),
                ("q_stride_b", ctypes.c_int64), ("q_stride_h", ctypes.c_int64),
                ("q_stride_s", ctypes.c_int64), ("kv_stride_b", ctypes.c_int64),
                ("kv_stride_h", ctypes.c_int64), ("kv_stride_s", ctypes.c_int64),
                ("scale", ctypes.c_float), ("causal", ctypes.c_int32)]


class AttnError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s: %s (status %d)" % (where, status_string(status), status))


_lib = None


def lib():
    """Load the HIP library (built in-tree by build.py); raise if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                "libmi355attn.so is not built (%s missing): run "
                "`python -c 'import __graft_entry__ as g; g.build()'` first; "
                "there is no fallback path" % LIB_PATH)
        # torch ships its own copy of the HIP runtime.  If this library were loaded first it
        # would bring in the system copy, and kernels registered with one runtime cannot be
        # launched on the streams of the other (the launch fails).  Importing torch first
        # makes its copy the one both use; the tensors and streams come from torch anyway.
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        vp, pp = ctypes.c_void_p, ctypes.POINTER(AttnParams)
        L.attn_params_contiguous.argtypes = [pp] + [ctypes.c_int32] * 4 + [ctypes.c_float,
                                                                           ctypes.c_int32]
        L.attn_params_contiguous.restype = None
        L.attn_fwd.argtypes = [vp, vp, vp, vp, vp, pp, vp]
        L.attn_fwd.restype = ctypes.c_int
        L.attn_bwd_workspace_bytes.argtypes = [pp]
        L.attn_bwd_workspace_bytes.restype = ctypes.c_size_t
        L.attn_bwd.argtypes = [vp] * 9 + [vp, ctypes.c_size_t, pp, vp]
        L.attn_bwd.restype = ctypes.c_int
        L.attn_bwd_stages.argtypes = [vp] * 9 + [vp, ctypes.c_size_t, pp, vp, ctypes.c_uint32]
        L.attn_bwd_stages.restype = ctypes.c_int
        gp = ctypes.POINTER(AttnGqaParams)
        L.attn_gqa_params_contiguous.argtypes = [gp] + [ctypes.c_int32] * 5 + [ctypes.c_float,
                                                                               ctypes.c_int32]
        L.attn_gqa_params_contiguous.restype = None
        L.attn_fwd_gqa.argtypes = [vp, vp, vp, vp, vp, gp, vp]
        L.attn_fwd_gqa.restype = ctypes.c_int
        L.attn_bwd_gqa_workspace_bytes.argtypes = [gp]
        L.attn_bwd_gqa_workspace_bytes.restype = ctypes.c_size_t
        L.attn_bwd_gqa.argtypes = [vp] * 9 + [vp, ctypes.c_size_t, gp, vp]
        L.attn_bwd_gqa.restype = ctypes.c_int
        L.attn_bwd_gqa_stages.argtypes = [vp] * 9 + [vp, ctypes.c_size_t, gp, vp, ctypes.c_uint32]
        L.attn_bwd_gqa_stages.restype = ctypes.c_int
        rp = ctypes.POINTER(AttnRectParams)
        L.attn_rect_params_contiguous.argtypes = [rp] + [ctypes.c_int32] * 6 + [ctypes.c_float,
                                                                               ctypes.c_int32]
        L.attn_rect_params_contiguous.restype = None
        L.attn_fwd_rect_workspace_bytes.argtypes = [rp]
        L.attn_fwd_rect_workspace_bytes.restype = ctypes.c_size_t
        L.attn_fwd_rect.argtypes = [vp, vp, vp, vp, vp, vp, ctypes.c_size_t, rp, vp]
        L.attn_fwd_rect.restype = ctypes.c_int
        L.attn_bwd_rect_workspace_bytes.argtypes = [rp]
        L.attn_bwd_rect_workspace_bytes.restype = ctypes.c_size_t
        L.attn_bwd_rect.argtypes = [vp] * 9 + [vp, ctypes.c_size_t, rp, vp]
        L.attn_bwd_rect.restype = ctypes.c_int
        L.attn_fwd_rect_f16.argtypes = L.attn_fwd_rect.argtypes
        L.attn_fwd_rect_f16.restype = ctypes.c_int
        L.attn_bwd_rect_f16.argtypes = L.attn_bwd_rect.argtypes
        L.attn_bwd_rect_f16.restype = ctypes.c_int
        L.attn_fwd_rope_workspace_bytes.argtypes = [rp]
        L.attn_fwd_rope_workspace_bytes.restype = ctypes.c_size_t
        L.attn_fwd_rope.argtypes = [vp] * 8 + [vp, ctypes.c_size_t, rp, vp]
        L.attn_fwd_rope.restype = ctypes.c_int
        L.attn_bwd_rope.argtypes = [vp] * 11 + [vp, ctypes.c_size_t, rp, vp]
        L.attn_bwd_rope.restype = ctypes.c_int
        L.attn_bwd_rect_noalloc.argtypes = [vp] * 9 + [rp, vp]
        L.attn_bwd_rect_noalloc.restype = ctypes.c_int
        L.attn_probe_mfma_bf16.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, vp, ctypes.c_size_t,
                                           ctypes.POINTER(ctypes.c_double), vp]
        L.attn_probe_mfma_bf16.restype = ctypes.c_int
        L.attn_probe_atomic_f32.argtypes = [ctypes.c_int] * 4 + [vp, ctypes.c_size_t,
                                            ctypes.POINTER(ctypes.c_double), vp]
        L.attn_probe_atomic_f32.restype = ctypes.c_int
        L.attn_probe_stream.argtypes = [vp, ctypes.c_size_t, ctypes.c_int, ctypes.c_int, vp, vp]
        L.attn_probe_stream.restype = ctypes.c_int
        L.attn_status_string.argtypes = [ctypes.c_int]
        L.attn_status_string.restype = ctypes.c_char_p
        L.attn_version.argtypes = []
        L.attn_version.restype = ctypes.c_int
        _lib = L
    return _lib


def status_string(status):
    return lib().attn_status_string(int(status)).decode()


def attn_version():
    return int(lib().attn_version())


def attn_probe_mfma_bf16(workgroups, iters, sink, random_operands=False, stream=None):
    """Enqueue the MFMA-only measurement kernel; returns the floating-point operations one
    launch executes.  `sink`: fp32 CUDA tensor of at least workgroups * 512 elements."""
    import torch
    assert sink.is_cuda and sink.dtype == torch.float32 and sink.is_contiguous()
    st = torch.cuda.current_stream().cuda_stream if stream is None else stream
    flop = ctypes.c_double(0.0)
    rc = lib().attn_probe_mfma_bf16(int(workgroups), int(iters), int(bool(random_operands)),
                                    sink.data_ptr(), sink.numel(),
                                    ctypes.byref(flop), ctypes.c_void_p(st))
    if rc != 0:
        raise AttnError(rc, "attn_probe_mfma_bf16")
    return flop.value


def attn_probe_atomic_f32(BH, S, key_block, causal, acc, stream=None):
    """Enqueue the atomic-add measurement kernel on the zeroed fp32 tensor `acc` (at least
    BH * S * 128 elements); returns the bytes one launch adds."""
    import torch
    assert acc.is_cuda and acc.dtype == torch.float32 and acc.is_contiguous()
    st = torch.cuda.current_stream().cuda_stream if stream is None else stream
    nbytes = ctypes.c_double(0.0)
    rc = lib().attn_probe_atomic_f32(int(BH), int(S), int(key_block), int(bool(causal)),
                                     acc.data_ptr(), acc.numel(), ctypes.byref(nbytes),
                                     ctypes.c_void_p(st))
    if rc != 0:
        raise AttnError(rc, "attn_probe_atomic_f32")
    return nbytes.value


def attn_probe_stream(src, workgroups, checksum, direct=False, nontemporal=False, stream=None):
    """Enqueue the read-streaming measurement kernel over the CUDA tensor `src` (all of its
    bytes); `checksum`: int32 CUDA tensor of `workgroups` elements, receives the XOR of the
    32-bit words each work-group read.  Returns the bytes one launch reads."""
    import torch
    assert src.is_cuda and src.is_contiguous() and checksum.is_cuda and checksum.is_contiguous()
    assert checksum.dtype == torch.int32 and checksum.numel() >= workgroups
    st = torch.cuda.current_stream().cuda_stream if stream is None else stream
    nbytes = src.numel() * src.element_size()
    rc = lib().attn_probe_stream(src.data_ptr(), nbytes, int(workgroups),
                                 int(bool(direct)) | (int(bool(nontemporal)) << 1),
                                 checksum.data_ptr(), ctypes.c_void_p(st))
    if rc != 0:
        raise AttnError(rc, "attn_probe_stream")
    return nbytes


def make_params(B, H, S, D, scale, causal, strides=None):
    """attn_params_t for a [B,H,S,D] tensor; strides=(sb, sh, ss) in elements or None for
    contiguous."""
    p = AttnParams()
    lib().attn_params_contiguous(ctypes.byref(p), B, H, S, D, float(scale), int(bool(causal)))
    if strides is not None:
        p.stride_b, p.stride_h, p.stride_s = (int(s) for s in strides)
    return p


def _strides3(t):
    """(stride_b, stride_h, stride_s) of a [B,H,S,D] tensor in elements.  The stride of an axis
    of length 1 is never used to address anything and may hold any value (numpy and torch both
    leave it arbitrary): it is replaced by the one a dense tensor would have, which always
    passes the library's stride checks."""
    B, H, S, D = t.shape
    ss = t.stride(2) if S > 1 else D
    sh = t.stride(1) if H > 1 else S * ss
    sb = t.stride(0) if B > 1 else H * sh
    return sb, sh, ss


def _params_for(t, scale, causal):
    if t.dim() != 4 or t.stride(3) != 1:
        raise ValueError("expected a [B,H,S,D] tensor with a contiguous D axis")
    B, H, S, D = t.shape
    return make_params(B, H, S, D, scale, causal, _strides3(t))


def _same_layout(ref, *ts):
    # (the stride of an axis of length 1 is never used and may be anything)
    def strides(t):
        return tuple(st for n, st in zip(t.shape, t.stride()) if n > 1)
    for t in ts:
        if t.shape != ref.shape or strides(t) != strides(ref) or t.dtype != ref.dtype \
                or t.device != ref.device:
            raise ValueError("all bf16 tensors must share shape, strides, dtype and device")


def _stream_ptr(torch, stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _on_stream(torch, stream):
    """Context in which tensors this binding allocates itself belong to the stream the kernels
    are enqueued on: torch's caching allocator ties a block to the stream that was current when
    it was allocated, and would otherwise hand a dropped workspace to other work of the
    current stream while kernels on `stream` still use it."""
    import contextlib
    return contextlib.nullcontext() if stream is None else torch.cuda.stream(stream)



def _elem_types(torch):
    return (torch.bfloat16, torch.float16)


def _check_lse(torch, LSE, shape):
    if LSE.dtype != torch.float32 or not LSE.is_contiguous() or tuple(LSE.shape) != tuple(shape):
        raise ValueError("LSE must be a contiguous fp32 [B,Hq,Sq] tensor")


def _forward(where, entry, params, ws_bytes_fn, Q, K, V, O, LSE, workspace, split, stream,
             dtypes):
    """Shared marshalling of the three forward entry points: checks, output allocation and the
    call `entry(Q, K, V, O, LSE, [workspace, bytes,] params, stream)`."""
    import torch
    if Q.dtype not in dtypes or not Q.is_cuda:
        raise ValueError("Q,K,V must be %s tensors on the GPU" % " or ".join(str(d) for d in dtypes))
    _same_layout(K, V)
    if K.dtype != Q.dtype or K.device != Q.device:
        raise ValueError("all tensors must share dtype and device")
    B, H, S, D = Q.shape
    with _on_stream(torch, stream):
        if O is None:
            O = torch.empty_strided(Q.shape, Q.stride(), dtype=Q.dtype, device=Q.device)
        else:
            _same_layout(Q, O)
        if LSE is None:
            LSE = torch.empty((B, H, S), dtype=torch.float32, device=Q.device)
        else:
            _check_lse(torch, LSE, (B, H, S))
        args = [Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), LSE.data_ptr()]
        if ws_bytes_fn is not None:  # the rectangular form takes an optional workspace
            ws_ptr, ws_bytes = None, 0
            if split:
                need = int(ws_bytes_fn(ctypes.byref(params)))
                if workspace is None and need:
                    workspace = torch.empty(need, dtype=torch.uint8, device=Q.device)
                if workspace is not None:
                    ws_ptr, ws_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
            args += [ws_ptr, ws_bytes]
    rc = entry(*args, ctypes.byref(params), _stream_ptr(torch, stream))
    if rc != ATTN_OK:
        raise AttnError(rc, where)
    return O, LSE


def _backward(where, entry, params, ws_bytes_fn, Q, K, V, O, dO, LSE, dQ, dK, dV, workspace,
              stream, dtypes, extra=()):
    """Shared marshalling of the backward entry points."""
    import torch
    if Q.dtype not in dtypes or not Q.is_cuda:
        raise ValueError("tensors must be %s on the GPU" % " or ".join(str(d) for d in dtypes))
    _same_layout(Q, O, dO)
    _same_layout(K, V)
    if K.dtype != Q.dtype or K.device != Q.device:
        raise ValueError("all tensors must share dtype and device")
    B, H, S, D = Q.shape
    _check_lse(torch, LSE, (B, H, S))
    with _on_stream(torch, stream):
        outs = []
        for t, like in ((dQ, Q), (dK, K), (dV, K)):
            if t is None:
                t = torch.empty_strided(like.shape, like.stride(), dtype=like.dtype, device=like.device)
            else:
                _same_layout(like, t)
            outs.append(t)
        dQ, dK, dV = outs
        if workspace is None:
            workspace = torch.empty(int(ws_bytes_fn(ctypes.byref(params))), dtype=torch.uint8,
                                    device=Q.device)
    rc = entry(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), dO.data_ptr(),
               LSE.data_ptr(), dQ.data_ptr(), dK.data_ptr(), dV.data_ptr(), workspace.data_ptr(),
               workspace.numel() * workspace.element_size(), ctypes.byref(params),
               _stream_ptr(torch, stream), *extra)
    if rc != ATTN_OK:
        raise AttnError(rc, where)
    return dQ, dK, dV


def attn_fwd(Q, K, V, scale, causal, O=None, LSE=None, stream=None):
    """O, LSE = attention forward.  Q,K,V: bf16 device tensors [B,H,S,D] with equal strides.
    Enqueues on `stream` (default: torch's current stream); does not synchronise."""
    import torch
    _same_layout(Q, K, V)
    return _forward("attn_fwd", lib().attn_fwd, _params_for(Q, scale, causal), None, Q, K, V, O,
                    LSE, None, False, stream, (torch.bfloat16,))


def attn_bwd_workspace_bytes(B, H, S, D):
    p = make_params(B, H, S, D, 1.0, False)
    return int(lib().attn_bwd_workspace_bytes(ctypes.byref(p)))


def attn_bwd(Q, K, V, O, dO, LSE, scale, causal, dQ=None, dK=None, dV=None, workspace=None,
             stream=None, stages=None):
    """dQ, dK, dV = attention backward for upstream gradient dO (all bf16, same strides).
    `stages` (profiling aid) restricts the call to a subset of its kernels through
    attn_bwd_stages; None calls attn_bwd."""
    import torch
    _same_layout(Q, K, V)
    entry, extra = (lib().attn_bwd, ()) if stages is None else (lib().attn_bwd_stages, (int(stages),))
    return _backward("attn_bwd", entry, _params_for(Q, scale, causal),
                     lib().attn_bwd_workspace_bytes, Q, K, V, O, dO, LSE, dQ, dK, dV, workspace,
                     stream, (torch.bfloat16,), extra)


# ---- grouped-query heads: Q, O, dO, dQ are [B,Hq,S,D]; K, V, dK, dV are [B,Hkv,S,D] ----------

def make_gqa_params(B, Hq, Hkv, S, D, scale, causal, q_strides=None, kv_strides=None):
    """attn_gqa_params_t; strides=(sb, sh, ss) in elements or None for contiguous."""
    p = AttnGqaParams()
    lib().attn_gqa_params_contiguous(ctypes.byref(p), B, Hq, Hkv, S, D, float(scale),
                                     int(bool(causal)))
    if q_strides is not None:
        p.q_stride_b, p.q_stride_h, p.q_stride_s = (int(s) for s in q_strides)
    if kv_strides is not None:
        p.kv_stride_b, p.kv_stride_h, p.kv_stride_s = (int(s) for s in kv_strides)
    return p


def _gqa_params_for(q, k, scale, causal):
    for t in (q, k):
        if t.dim() != 4 or t.stride(3) != 1:
            raise ValueError("expected [B,H,S,D] tensors with a contiguous D axis")
    B, Hq, S, D = q.shape
    if k.shape[0] != B or k.shape[2] != S or k.shape[3] != D:
        raise ValueError("K/V must be [B,Hkv,S,D] matching Q in B, S and D")
    return make_gqa_params(B, Hq, k.shape[1], S, D, scale, causal, _strides3(q), _strides3(k))


def attn_fwd_gqa(Q, K, V, scale, causal, O=None, LSE=None, stream=None):
    """O [B,Hq,S,D], LSE [B,Hq,S] = grouped-query attention forward; K, V: [B,Hkv,S,D]."""
    import torch
    return _forward("attn_fwd_gqa", lib().attn_fwd_gqa, _gqa_params_for(Q, K, scale, causal), None,
                    Q, K, V, O, LSE, None, False, stream, (torch.bfloat16,))


def attn_bwd_gqa_workspace_bytes(B, Hq, Hkv, S, D):
    p = make_gqa_params(B, Hq, Hkv, S, D, 1.0, False)
    return int(lib().attn_bwd_gqa_workspace_bytes(ctypes.byref(p)))


def attn_bwd_gqa(Q, K, V, O, dO, LSE, scale, causal, dQ=None, dK=None, dV=None, workspace=None,
                 stream=None, stages=None):
    """dQ [B,Hq,S,D], dK, dV [B,Hkv,S,D] = grouped-query attention backward."""
    import torch
    entry, extra = ((lib().attn_bwd_gqa, ()) if stages is None
                    else (lib().attn_bwd_gqa_stages, (int(stages),)))
    return _backward("attn_bwd_gqa", entry, _gqa_params_for(Q, K, scale, causal),
                     lib().attn_bwd_gqa_workspace_bytes, Q, K, V, O, dO, LSE, dQ, dK, dV,
                     workspace, stream, (torch.bfloat16,), extra)


# ---- rectangular: Q, O, dO, dQ are [B,Hq,Sq,D]; K, V, dK, dV are [B,Hkv,Sk,D]; a causal mask
# is aligned bottom-right (query row i sees keys 0 .. i + Sk - Sq) ------------------------------

def make_rect_params(B, Hq, Hkv, Sq, Sk, D, scale, causal, q_strides=None, kv_strides=None):
    """attn_rect_params_t; strides=(sb, sh, ss) in elements or None for contiguous."""
    p = AttnRectParams()
    lib().attn_rect_params_contiguous(ctypes.byref(p), B, Hq, Hkv, Sq, Sk, D, float(scale),
                                      int(bool(causal)))
    if q_strides is not None:
        p.q_stride_b, p.q_stride_h, p.q_stride_s = (int(s) for s in q_strides)
    if kv_strides is not None:
        p.kv_stride_b, p.kv_stride_h, p.kv_stride_s = (int(s) for s in kv_strides)
    return p


def _rect_params_for(q, k, scale, causal):
    for t in (q, k):
        if t.dim() != 4 or t.stride(3) != 1:
            raise ValueError("expected [B,H,S,D] tensors with a contiguous D axis")
    B, Hq, Sq, D = q.shape
    if k.shape[0] != B or k.shape[3] != D:
        raise ValueError("K/V must be [B,Hkv,Sk,D] matching Q in B and D")
    return make_rect_params(B, Hq, k.shape[1], Sq, k.shape[2], D, scale, causal,
                            _strides3(q), _strides3(k))


def attn_fwd_rect_workspace_bytes(B, Hq, Hkv, Sq, Sk, D, causal=False):
    """Bytes attn_fwd_rect needs to split this problem over the keys (0: it would not split).
    The plan may use fewer splits under a causal mask, never more."""
    p = make_rect_params(B, Hq, Hkv, Sq, Sk, D, 1.0, causal)
    return int(lib().attn_fwd_rect_workspace_bytes(ctypes.byref(p)))


def attn_fwd_rect(Q, K, V, scale, causal, O=None, LSE=None, workspace=None, split=True,
                  stream=None):
    """O [B,Hq,Sq,D], LSE [B,Hq,Sq]; K, V: [B,Hkv,Sk,D].  `split=False` passes no workspace,
    which keeps the forward in one kernel; otherwise a workspace is allocated when the
    library's plan asks for one.  bf16 or fp16 tensors (all of one type)."""
    import torch
    entry = lib().attn_fwd_rect_f16 if Q.dtype == torch.float16 else lib().attn_fwd_rect
    return _forward("attn_fwd_rect", entry, _rect_params_for(Q, K, scale, causal),
                    lib().attn_fwd_rect_workspace_bytes, Q, K, V, O, LSE, workspace, split, stream,
                    _elem_types(torch))


def attn_bwd_rect_workspace_bytes(B, Hq, Hkv, Sq, Sk, D):
    p = make_rect_params(B, Hq, Hkv, Sq, Sk, D, 1.0, False)
    return int(lib().attn_bwd_rect_workspace_bytes(ctypes.byref(p)))


def attn_bwd_rect(Q, K, V, O, dO, LSE, scale, causal, dQ=None, dK=None, dV=None, workspace=None,
                  stream=None):
    """dQ [B,Hq,Sq,D], dK, dV [B,Hkv,Sk,D] = rectangular attention backward (bf16 or fp16)."""
    import torch
    entry = lib().attn_bwd_rect_f16 if Q.dtype == torch.float16 else lib().attn_bwd_rect
    return _backward("attn_bwd_rect", entry, _rect_params_for(Q, K, scale, causal),
                     lib().attn_bwd_rect_workspace_bytes, Q, K, V, O, dO, LSE, dQ, dK, dV,
                     workspace, stream, _elem_types(torch))


def attn_bwd_rect_noalloc(Q, K, V, O, dO, LSE, scale, causal, dQ, dK, dV, stream=None):
    """attn_bwd_rect through the entry point that uses the library's static scratch: the
    caller passes every output, nothing is allocated here or in the library."""
    import torch
    if Q.dtype != torch.bfloat16 or not Q.is_cuda:
        raise ValueError("tensors must be bf16 on the GPU")
    _same_layout(Q, O, dO, dQ)
    _same_layout(K, V, dK, dV)
    B, H, S, D = Q.shape
    _check_lse(torch, LSE, (B, H, S))
    p = _rect_params_for(Q, K, scale, causal)
    rc = lib().attn_bwd_rect_noalloc(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(),
                                     dO.data_ptr(), LSE.data_ptr(), dQ.data_ptr(), dK.data_ptr(),
                                     dV.data_ptr(), ctypes.byref(p), _stream_ptr(torch, stream))
    if rc != ATTN_OK:
        raise AttnError(rc, "attn_bwd_rect_noalloc")
    return dQ, dK, dV


# ---- rotary embedding fused into the calls: Q unrotated in, K rotated in (see include/attn.h) ---

def _check_tables(torch, cos, sin, Sk, D):
    for t in (cos, sin):
        if t.dtype != torch.float32 or not t.is_cuda or not t.is_contiguous() \
                or tuple(t.shape) != (Sk, D // 2):
            raise ValueError("cos/sin tables must be contiguous fp32 [Sk, D/2] tensors on the GPU")


def attn_fwd_rope(Q, K_rot, V, cos, sin, scale, causal, O=None, LSE=None, Q_rot=None,
                  want_q_rot=True, split=True, stream=None):
    """O, LSE, Q_rot = attention forward with the rotary embedding of the query rows fused into
    their load.  Q: unrotated [B,Hq,Sq,D]; K_rot: rotated [B,Hkv,Sk,D]; cos, sin: fp32 [Sk,D/2].
    Q_rot (the rotated query rows the backward needs) is returned unless want_q_rot=False."""
    import torch
    if Q.dtype != torch.bfloat16 or not Q.is_cuda:
        raise ValueError("Q,K,V must be bf16 tensors on the GPU")
    _same_layout(K_rot, V)
    B, H, S, D = Q.shape
    _check_tables(torch, cos, sin, K_rot.shape[2], D)
    p = _rect_params_for(Q, K_rot, scale, causal)
    with _on_stream(torch, stream):
        if O is None:
            O = torch.empty_strided(Q.shape, Q.stride(), dtype=Q.dtype, device=Q.device)
        else:
            _same_layout(Q, O)
        if LSE is None:
            LSE = torch.empty((B, H, S), dtype=torch.float32, device=Q.device)
        else:
            _check_lse(torch, LSE, (B, H, S))
        if Q_rot is None and want_q_rot:
            Q_rot = torch.empty_strided(Q.shape, Q.stride(), dtype=Q.dtype, device=Q.device)
        elif Q_rot is not None:
            _same_layout(Q, Q_rot)
        ws = None
        if split:
            need = int(lib().attn_fwd_rope_workspace_bytes(ctypes.byref(p)))
            if need:
                ws = torch.empty(need, dtype=torch.uint8, device=Q.device)
    rc = lib().attn_fwd_rope(Q.data_ptr(), K_rot.data_ptr(), V.data_ptr(), cos.data_ptr(),
                             sin.data_ptr(), O.data_ptr(), LSE.data_ptr(),
                             Q_rot.data_ptr() if Q_rot is not None else None,
                             ws.data_ptr() if ws is not None else None,
                             ws.numel() if ws is not None else 0, ctypes.byref(p),
                             _stream_ptr(torch, stream))
    if rc != ATTN_OK:
        raise AttnError(rc, "attn_fwd_rope")
    return O, LSE, Q_rot


def attn_bwd_rope(Q_rot, K_rot, V, O, dO, LSE, cos, sin, scale, causal, dQ=None, dK_rot=None,
                  dV=None, workspace=None, stream=None):
    """dQ (gradient of the UNROTATED query rows), dK_rot (gradient of the rotated K), dV."""
    import torch
    _check_tables(torch, cos, sin, K_rot.shape[2], Q_rot.shape[3])
    p = _rect_params_for(Q_rot, K_rot, scale, causal)

    def entry(*args):  # the tables sit between LSE and dQ in the C signature
        return lib().attn_bwd_rope(*args[:6], cos.data_ptr(), sin.data_ptr(), *args[6:])
    return _backward("attn_bwd_rope", entry, p, lib().attn_bwd_rect_workspace_bytes, Q_rot, K_rot,
                     V, O, dO, LSE, dQ, dK_rot, dV, workspace, stream, (torch.bfloat16,))
