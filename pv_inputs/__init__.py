"""Seeded synthetic inputs shared by the GPU path's callers and the CPU oracle's callers.

Holds only random-number drawing, the workload shape tables and the preparation of 4-bit
weights (the stand-in for a quantised checkpoint: codes and scales are inputs of both sides);
none of the decoder's or the acceptance rule's arithmetic lives here.
"""
from .configs import CONFIGS, ModelShape, TENSOR_KINDS, tensor_shape, tensor_id  # noqa: F401
from .synth import (  # noqa: F401
    build, quantile_table, fill_tensor, iter_tensors, uniform_tokens, unit_draws,
    perturb_drafts, bf16_round_f32, bf16_bits_to_f32, iter_row_chunks,
    quantize_q4, iter_row_chunks_q4, Q4_KINDS, Q4_GROUP,
)
