"""Seeded synthetic inputs shared by the GPU path's callers and the CPU oracle's callers.

Holds only random-number drawing and the workload shape tables; none of the
decoder's or the acceptance rule's arithmetic lives here.
"""
from .configs import CONFIGS, ModelShape, TENSOR_KINDS, tensor_shape, tensor_id  # noqa: F401
from .synth import (  # noqa: F401
    build, quantile_table, fill_tensor, iter_tensors, uniform_tokens, unit_draws,
    perturb_drafts, bf16_round_f32, bf16_bits_to_f32, iter_row_chunks,
)
