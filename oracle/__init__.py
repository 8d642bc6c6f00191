"""CPU oracle for the AttentionPack decode hot path.

TEST INFRASTRUCTURE ONLY.  Nothing in the product package may import this
module; it is used by tests/, by __graft_entry__.smoke() and by the
cpu_baseline leg of bench.py.  It shares no code with the HIP kernels.
"""
from .attnpack_oracle import (  # noqa: F401
    promote,
    bases,
    randomized_bases,
    basis_quality,
    decompress,
    compact,
    decode_attn,
    decode_attn_absorbed,
    decode_attn_batched,
    attention_probs,
    raw_attn,
    decode_attn_segments,
    merge_segments,
    select_ranks,
    quantize_i8,
    dequantize_i8,
    quantize_i4,
    unpack_i4,
    dequantize_i4,
    compression_ratio,
    decompression_flops,
    cache_bytes,
    importance_update,
)
