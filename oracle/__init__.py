"""CPU fp64 oracle of the chunked-prefill decoder layer, and a plain statement of the request scheduler.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path (the HIP library and its
Python binding) may import, call or link this package; it exists so that tests,
the smoke check and the benchmark's CPU-baseline leg have an independent,
obviously-correct statement of what the layer computes.
"""
from .decoder_layer import (  # noqa: F401
    LayerParams, rmsnorm, rope_angles, mrope_angles, rope, silu, causal_gqa_attention,
    layer_forward, layer_forward_rows, ChunkedPrefill, prefill_batch, first_token_logits, rel_fro,
)
from .brute_force import attention_loops  # noqa: F401
from .scheduler import TrackedRequest, encoder_batches, schedule_round  # noqa: F401
