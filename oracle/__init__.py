"""CPU oracle for the DuoAttention deployment hot path (test infrastructure only).

Everything in this package is a plain, slow, float64 re-statement of what the
paper defines: full (causal) attention for retrieval heads and Lambda-masked
(sink + recent) attention for streaming heads, the two-cache bookkeeping, the
log-sum-exp merge identity, and the fp8 KV codec the benchmark configuration
adds.  It is NOT part of the product: only tests, the smoke check and the
benchmark's cpu_baseline leg may import it, and it imports nothing from the
GPU package.
"""
from .duo_oracle import (  # noqa: F401
    R_INCLUDES_SELF,
    visible_mask,
    visible_count,
    visible_mask_deployed,
    prefill_chunk_deployed,
    attention_rows,
    prefill_chunk,
    decode_step,
    merge_partials,
    CacheModel,
    retained_positions,
)
from .fp8_codec import (  # noqa: F401
    E4M3_MAX,
    e4m3_decode_table,
    e4m3_encode_f32,
    quantize_rows,
    dequantize_rows,
)
from .int4_codec import (  # noqa: F401
    quantize_rows_int4,
    quantize_rows_int8,
    dequantize_rows_int8,
    dequantize_rows_int4,
    pack_int4,
    unpack_int4,
)
from .gate_mixed import (  # noqa: F401
    visible_mask_block,
    gate_mixed_attention,
    gate_mixed_rows,
)
