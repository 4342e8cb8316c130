"""torch.autograd wrapper around the fused attention entry points, so that the operator can
stand where a framework's scaled-dot-product attention stands in a training step (the paper
trains its ViT and miniGPT examples through its fused attention this way).

Marshalling only: the forward calls attn_fwd_rect and keeps (Q, K, V, O, LSE) for the
backward, which calls attn_bwd_rect.  No arithmetic happens here, and there is no fallback:
tensors the kernels cannot take (wrong device or type) raise.
"""
import torch

from . import binding


def _like(ref, t):
    """t with the shape, strides and type of ref (copied only if it differs)."""
    if t.dtype == ref.dtype and t.stride() == ref.stride():
        return t
    out = torch.empty_strided(ref.shape, ref.stride(), dtype=ref.dtype, device=ref.device)
    out.copy_(t)
    return out


def _dense(t):
    """Layouts the library takes: unit stride along D, other strides multiples of 8 elements,
    16-byte aligned base.  Anything else is copied to a contiguous tensor."""
    ok = t.stride(3) == 1 and all(s % 8 == 0 for s in t.stride()[:3]) and t.data_ptr() % 16 == 0
    return t if ok else t.contiguous()


class _FusedAttention(torch.autograd.Function):
    @staticmethod
    def forward(ctx, q, k, v, scale, causal):
        q, k = _dense(q), _dense(k)
        v = _like(k, _dense(v))
        O, LSE = binding.attn_fwd_rect(q, k, v, scale, causal)
        ctx.save_for_backward(q, k, v, O, LSE)
        ctx.scale, ctx.causal = scale, causal
        return O

    @staticmethod
    def backward(ctx, dO):
        q, k, v, O, LSE = ctx.saved_tensors
        dQ, dK, dV = binding.attn_bwd_rect(q, k, v, O, _like(O, dO), LSE, ctx.scale, ctx.causal)
        return dQ, dK, dV, None, None


def fused_attention(q, k, v, causal=False, scale=None):
    """softmax(scale * q k^T [+ causal mask]) v with gradients.  q: [B, Hq, Sq, D]; k, v:
    [B, Hkv, Sk, D] with Hkv dividing Hq; bf16 or fp16 tensors on the GPU; D a multiple of 8 up
    to 128.  scale defaults to D ** -0.5.  With causal=True query row i sees keys
    0 .. i + Sk - Sq (needs Sk >= Sq)."""
    if scale is None:
        scale = float(q.shape[-1]) ** -0.5
    return _FusedAttention.apply(q, k, v, float(scale), bool(causal))
