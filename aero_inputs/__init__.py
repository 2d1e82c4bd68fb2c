"""Seeded synthetic workloads for the group-based RL update (GRPO with AERO curation).

This module only draws random inputs: group structure, binary rewards, response
lengths, sampled-token ids, logits / hidden states / LM-head weights and the noise
that turns current log-probs into behaviour-policy log-probs.  It contains none of
the method's arithmetic (no softmax, no advantage, no loss), so both the float64
checker and the GPU library can be fed from it without sharing any computation.

The workloads stand in for the on-policy math / code batches the paper trains on
(binary verifiable rewards, more than a third of the queries with all-equal
rewards, kept group sizes between 2 and 16, responses of at most a few thousand
tokens with padding removed, bf16 activations, clip range 0.2).  Every draw comes
from ``numpy.random.default_rng`` keyed by ``(seed, stream, block)`` so that any
block of rows can be regenerated on its own and in parallel.
"""
from .bf16 import f32_to_bf16_bits, f32_to_f16_bits, f32_to_f8e4m3_bits
from .workloads import (
    ADV_PARAM_DEFAULTS,
    LogitsWorkload,
    FusedWorkload,
    make_config,
    make_step_groups,
    RolloutSimulator,
    draw_old_logprob,
    normal_rows,
)

__all__ = [
    "ADV_PARAM_DEFAULTS",
    "LogitsWorkload",
    "FusedWorkload",
    "make_config",
    "make_step_groups",
    "RolloutSimulator",
    "draw_old_logprob",
    "normal_rows",
    "f32_to_bf16_bits",
    "f32_to_f16_bits",
    "f32_to_f8e4m3_bits",
]
