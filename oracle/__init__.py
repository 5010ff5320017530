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
    merge,
    threads,
)
