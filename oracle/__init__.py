"""CPU oracle for the dq8 codec -- test infrastructure, not the product.

Only tests, the smoke check and the benchmark's cpu_baseline leg import this
package.  It shares nothing with the HIP library.
"""
from .dq8_oracle import (  # noqa: F401
    DYNAMIC_TREE,
    LINEAR,
    MANTISSA,
    STATIC_TREE,
    absmax,
    absmax_segments,
    build,
    codebook,
    decode,
    decode_accumulate_avg,
    decode_accumulate_avg_segments,
    decode_avg_encode,
    decode_segments,
    encode,
    encode_segments,
    error_stats,
    set_threads,
)
