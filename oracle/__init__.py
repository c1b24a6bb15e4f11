"""CPU oracle for SageBwd (INT8 attention forward + backward).

TEST INFRASTRUCTURE ONLY.  This package is the slow, plain reference that the
HIP library is checked against.  It shares no code with the GPU path and must
never be imported by the product package; only tests/, the smoke check and the
benchmark's cpu_baseline leg may use it.
"""
from .sage_oracle import (  # noqa: F401
    BLOCK,
    round_to_bf16,
    qk_norm,
    key_mean,
    block_mean,
    pad_rows,
    padded_len,
    quantize_blocks,
    prepass_head,
    delta_rows,
    forward_head,
    backward_head,
    forward,
    backward,
)
