"""CPU fp64 oracles (fused attention; its row-wise neighbours) -- test infrastructure only.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this
package.  It shares nothing with the HIP library and is never a fallback for it.
"""
from .attn_oracle import (attn_fwd, attn_bwd, attn_probs, attn_dscores, build,  # noqa: F401
                          attn_fwd_rope, attn_bwd_rope, rope_rotate_queries,
                          f16_to_f64, num_threads)
from . import rowops_oracle as rowops  # noqa: F401,E402
