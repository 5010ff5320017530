"""TEST INFRASTRUCTURE: fp64 CPU oracle for block-causal attention and the block cache.

Only tests/, the smoke check and the benchmark's cpu_baseline leg import this
package. It shares no code with the HIP library and never calls it.
"""
from .oracle import (  # noqa: F401
    BlockCacheOracle,
    attention,
    attention_rows,
    build,
    bf16_bits_to_f64,
    bf16_bits_through_e4m3,
    e4m3_bits_to_f64,
    quantize_e4m3,
    merge,
    threads,
)
