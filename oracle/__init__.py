"""CPU oracle for the PulseCol attention hot path.

TEST INFRASTRUCTURE ONLY.  This package is the slow, plain definition of what
the GPU library must compute.  It shares no code with the HIP path and must
never be imported by the product package; only the test-suite, the smoke
check and the benchmark's ``cpu_baseline`` leg may use it.
"""

from .pulsecol_oracle import (  # noqa: F401
    attention_logits,
    block_columns,
    block_scores,
    block_sparse_attention,
    column_scores,
    dense_attention,
    num_keep,
    refresh_schedule,
    refresh_schedule_power,
    refresh_schedule_random,
    row_softmax,
    select_blocks,
    select_columns,
    sparse_attention_chunked,
    sparse_attention_gathered,
    sparse_attention_masked,
    topk_columns,
)
