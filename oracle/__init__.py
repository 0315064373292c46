"""CPU fp64 oracle of the VideoScan streaming attention path (TEST INFRASTRUCTURE).

Only tests, the smoke check and the CPU-baseline leg of the benchmark import this
package.  It shares no code with the GPU library and never imports it.
"""
from .vs_oracle import (  # noqa: F401
    attention,
    bank_apply,
    bank_victim,
    compact_append,
    decode,
    decoder_layer,
    gated_unit,
    linear,
    rmsnorm,
    frame_prefill,
    frame_qkv,
    frames_prefill,
    mean_pool,
    num_threads,
    query_prefill,
    OracleError,
)
