"""Seeded synthetic inputs for batched incremental-prefill attention over a paged KV cache.

This module only draws random numbers, rounds them to bf16 bit patterns and lays out
block tables.  It contains none of the method's arithmetic (no attention, no KV append, no
quantisation) so that both the CPU oracle's tests and the GPU path can consume exactly the
same inputs without sharing any code of the method itself.

The shapes stand in for multi-round agent / iterative-RAG traces (history length l_hist and
incremental length l_incr per prefill task, one token per decode step; paper Section 3,
"System Overview", and Table 1 for the length statistics of the real traces).  Only length
distributions are synthesised; no item of any dataset is reproduced.
"""
from .batches import (Batch, make_batch, make_config, config_lengths, CONFIG_SHAPES, impose_key_ramp,
                      f32_to_bf16_bits, bf16_bits_to_f64, BASE_SEED, NAN_BF16)
from .trace import SessionTrace, make_trace_schedule, draw_tick_tensors

__all__ = ["Batch", "make_batch", "make_config", "config_lengths", "CONFIG_SHAPES",
           "f32_to_bf16_bits", "bf16_bits_to_f64", "BASE_SEED", "NAN_BF16",
           "SessionTrace", "make_trace_schedule", "draw_tick_tensors"]
