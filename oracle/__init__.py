"""CPU fp64 oracle for fused attention -- test infrastructure only.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this
package.  It shares nothing with the HIP library and is never a fallback for it.
"""
from .attn_oracle import (attn_fwd, attn_bwd, attn_probs, attn_dscores, build,  # noqa: F401
                          f16_to_f64, num_threads)
