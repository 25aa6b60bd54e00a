"""CPU fp64 oracle for the DiT attention hot path -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this
package; the GPU library never does.  See dit_oracle.c for what is computed and why.
"""
from .dit_oracle import (  # noqa: F401
    build,
    cross_attn,
    cross_attn_decoupled,
    self_attn_packed,
    num_threads,
    qk_rmsnorm,
    self_attn_normed,
    as_f64,
    e4m3_round,
    e4m3_quantise_rows,
    self_attn_fp8_scores,
    linear,
    rope3d,
    self_attn,
    token_positions,
)
