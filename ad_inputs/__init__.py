"""Seeded synthetic inputs (weights, sources, guides, drafts) for Aggressive Decoding.

This module serves both the CPU oracle and the HIP path. It holds no arithmetic of
the method itself: only random draws, shapes and the edit recipes that turn a given
greedy output into a guide or a positional draft.
"""
from .gen import (  # noqa: F401
    SPECIAL, DIMS, CONFIGS, model_dims, param_spec, init_weights, draw_sources,
    edit_guide, positional_draft,
)
