"""CPU oracle for the cyclic/hybrid decode-attention share (test infrastructure).

A plain, slow, fp64 statement of what the path computes, written from the paper
(Section 3.1: cyclic KVCache placement, hybrid attention, load-aware DP-rank
routing) and from the textbook definition of softmax attention.  It exists only
to check the HIP library: tests, the smoke check and the benchmark's CPU
baseline leg may call it; the product never does, and nothing here imports the
product.

All four parts are pinned by tests that do not go through this code's own
formulas a second time (worked examples from the paper's figures, closed forms,
brute force, invariants, library routines); no function here is "parity
unpinned".
"""
from .formats import bf16_bits_to_f64, e4m3_bytes_to_f64, E4M3_TABLE  # noqa: F401
from .placement import build_placement, build_placement_hybrid_heads  # noqa: F401
from .prefill import (  # noqa: F401
    build_prefill_worklist, choose_prefill_chunk, prefill_attention_items, prefill_attention_pairs, prefill_attention_row,
    PREFILL_ITEM_FIELDS, PREFILL_PAIR_FIELDS,
)
from .recovery import plan_ffn_reload, plan_kv_reload, replace_failed_gpu  # noqa: F401
from .scheduler import adaptive_chunked_prefill, route_request, token_cost  # noqa: F401
from .worklist import build_worklist, build_worklist_units, build_launch_records, choose_chunk_tokens, ITEM_FIELDS, PAIR_FIELDS  # noqa: F401
from .attention import (  # noqa: F401
    attend,
    gather_pair_kv,
    decode_attention_pairs,
    decode_attention_items,
    merge_lse,
    unsharded_attention,
)
