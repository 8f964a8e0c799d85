"""Seeded synthetic inputs for the HSD verification hot path.

This package only *draws* inputs (weights, visual-prefix embeddings, prompt
tokens, draft lengths, corruption positions).  It contains none of the
method's arithmetic: no decoder forward, no acceptance rule.  Both the CPU
oracle's tests and the HIP path's tests/bench draw their inputs from here so
that the two sides see bit-identical data.
"""
from .generators import (  # noqa: F401
    ModelDesc, MODEL_T, MODEL_M, tiny_model, make_weights, make_prefix,
    round_to_bf16, corrupt_draft, corrupt_draft_forced, CONFIGS, WorkloadConfig,
    draw_sequences, SEED_BASE,
)
