"""Seeded synthetic inputs for the history-drafted speculative decoding path.

This module only *generates inputs* (weights, RoPE table, prompts, mutated
histories, length mixes).  It holds none of the method's arithmetic: no suffix
matching, no model forward, no acceptance rule, no random-number generator the
method itself draws from.  The CPU oracle and the HIP path each consume these
arrays; neither generates its own.
"""
from .gen import (  # noqa: F401
    ModelShape,
    CONFIG_SHAPES,
    bf16_bits,
    bf16_to_f32,
    make_weights,
    rope_table,
    make_prompts,
    mutate,
    history_with_context,
    lengths_uniform,
    lengths_lognormal,
    config_seed,
)
