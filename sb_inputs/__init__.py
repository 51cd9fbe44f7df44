"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests.

This package produces *data only*: model-shape descriptions, random-init weights,
prompts and forced exit / draft schedules.  It contains none of the decoder's or
the speculation algorithm's arithmetic, and imports neither the oracle nor the
HIP library.
"""
from .configs import ModelShape, Workload, CONFIGS, tiny_shape
from .weights import make_weights, round_to_bf16, bf16_to_f32, tensor_specs, easy_token_weights
from .schedules import (make_prompt, forced_exit_schedule, accept_schedule,
                        injection_schedule)

__all__ = [
    "ModelShape", "Workload", "CONFIGS", "tiny_shape", "make_weights",
    "round_to_bf16", "bf16_to_f32", "tensor_specs", "easy_token_weights", "make_prompt",
    "forced_exit_schedule", "accept_schedule", "injection_schedule",
]
