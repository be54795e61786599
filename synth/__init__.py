"""Seeded synthetic inputs for the chunked-prefill decoder-layer path.

This package only draws random numbers, rounds them to bf16 and describes
workload shapes.  It contains none of the layer's arithmetic, and it imports
neither the CPU oracle nor the HIP binding, so both sides can be fed from it.
"""
from .workloads import (  # noqa: F401
    LayerShape, TINY, L7B, L72B, LayerWeights, Workload, BatchRequest,
    bf16_round, bf16_bits, bits_to_f32, layer_weights, prompt_rows,
    chunk_schedule, workload, WORKLOAD_NAMES, dirichlet_chunk_lengths,
)
