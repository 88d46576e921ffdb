"""Seeded synthetic workloads for the pipelined decoder.

This package only *describes* workloads (model shapes, decode parameters) and
draws their random weights and context token ids.  It holds none of the
method's arithmetic: no attention, no schedule, no visibility rule.  The CPU
oracle and the HIP path are both fed from here and share nothing else.
"""

from .configs import WorkloadConfig, EncDecConfig, CONFIGS, ENCDEC_CONFIGS, get_config, max_positions
from .generate import (make_weights, make_context, make_forced_tokens, bf16_round, bf16_bits,
                       bits_to_f32, tie_lm_head, make_encdec_weights, encdec_to_bf16)

__all__ = [
    "WorkloadConfig", "CONFIGS", "ENCDEC_CONFIGS", "get_config", "max_positions",
    "make_weights", "make_context", "make_forced_tokens", "bf16_round", "bf16_bits", "bits_to_f32",
    "tie_lm_head", "EncDecConfig", "make_encdec_weights", "encdec_to_bf16",
]
