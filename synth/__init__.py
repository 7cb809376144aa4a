"""Seeded synthetic ERNIE-shaped inputs (weights, kept-row sets, prompts).

This package holds no arithmetic of the method itself: it only draws random
parameters and token ids.  Both the CPU oracle's tests and the HIP path's
tests/bench draw their inputs from here so that they see bit-identical data.
"""
from .ernie_inputs import (CONFIGS, ErnieShape, make_weights, make_kept_ids,
                           make_prompts, full_to_trimmed, trim_table, Workload,
                           make_workload, make_corpus)

__all__ = ["CONFIGS", "ErnieShape", "make_weights", "make_kept_ids",
           "make_prompts", "full_to_trimmed", "trim_table", "Workload",
           "make_workload", "make_corpus"]
