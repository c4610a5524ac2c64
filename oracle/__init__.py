"""CPU oracle (fp64) for context-parallel ring attention.

TEST INFRASTRUCTURE ONLY: imported by the tests, the smoke check and the
benchmark's CPU-baseline leg. The product path never imports this package and
this package never imports the product.
"""
from .cp_oracle import (  # noqa: F401
    KVCache,
    attn,
    build,
    chunk_bounds,
    decode_owner,
    merge,
    num_threads,
    ring_passkv,
    ring_passq,
    ring_passq_decode,
    roofline_latencies,
    select_order,
    set_num_threads,
    shard_decode_batch,
    shard_partial_prefill,
    shard_positions,
    unsharded_causal,
)
