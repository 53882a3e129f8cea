"""Seeded synthetic inputs for the cyclic/hybrid decode-attention share.

This package only draws random numbers and encodes them into the storage
formats the batch is defined on (bf16 bits, fp8 e4m3 bytes + scales, a paged
pool with a shuffled slot order).  It holds none of the method's arithmetic:
no placement rule, no work-list rule, no attention.  Both the CPU oracle's
tests and the HIP path's tests feed from it.
"""
from .generate import (  # noqa: F401
    CONFIGS,
    BASE_SEED,
    make_requests,
    make_q,
    make_kv_pool,
    f32_to_bf16_bits,
    make_prefill_queue,
    make_prefill_q,
)
