"""Seeded synthetic workloads for the draft-verify step.

Shapes, context lengths, chunk sizes and draft statistics follow the regime the
paper describes (Sec. 3: contexts of about 1K tokens and more, fixed prefill
chunks of 128/256 tokens; Sec. 4.3 / Sec. 5.1: drafts of mostly 2-8 tokens
capped at 32, copied from the context as a retrieval drafter would).  The
paper's datasets and trained weights are not used: token ids, weights and
drafts are random with the same shapes.

This module holds input generation only -- none of the method's arithmetic --
so both the CPU oracle's tests and the GPU library's tests draw the same
inputs from it.
"""
from .configs import CONFIGS, WorkloadConfig, scaled
from .generate import (
    streams, make_weights, make_context, copy_span_drafts, geometric_copy_drafts,
    inject_mismatch, gumbel_drafts, make_uniforms, rag_mix, to_bf16_values,
)

__all__ = [
    "CONFIGS", "WorkloadConfig", "scaled", "streams", "make_weights", "make_context",
    "copy_span_drafts", "geometric_copy_drafts", "inject_mismatch", "gumbel_drafts",
    "make_uniforms", "rag_mix", "to_bf16_values",
]
