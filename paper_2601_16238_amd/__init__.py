"""MI355X-native fused scaled-dot-product attention (forward + backward) behind a C ABI.

`attn_fwd` / `attn_bwd` marshal torch device tensors into libmi355attn.so (hand-written
HIP kernels for gfx950).  `workloads` holds the seeded synthetic inputs.
"""
from . import workloads  # noqa: F401
from . import rowops  # noqa: F401
from .autograd import fused_attention  # noqa: F401
from .binding import (AttnError, AttnGqaParams, AttnParams, AttnRectParams,  # noqa: F401
                      attn_bwd, attn_bwd_gqa, attn_bwd_gqa_workspace_bytes, attn_bwd_rect,
                      attn_bwd_rect_noalloc, attn_bwd_rope, attn_fwd_rope,
                      attn_bwd_rect_workspace_bytes, attn_bwd_workspace_bytes, attn_fwd,
                      attn_fwd_gqa, attn_fwd_rect, attn_fwd_rect_workspace_bytes,
                      attn_probe_atomic_f32, attn_probe_mfma_bf16, attn_probe_stream, attn_version,
                      lib, make_gqa_params, make_params, make_rect_params, status_string)
