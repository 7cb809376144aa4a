"""CPU oracle for a whole generation job -- TEST INFRASTRUCTURE.

The paper splits serving into a main process, a preprocessing process, a
model-inference process and a post-processing process that run side by side
(Method, "Multi-process parallel processing").  Running the stages side by side
must not change any result, so the oracle is the plain sequential definition:
every request, on its own, goes through preprocessing (full ids -> trimmed ids,
dropped ids become the unknown-word row), generation (the generator of
ernie_oracle.py, free-running greedy) and post-processing (trimmed ids -> full
ids), and results come back in request order.

Nothing in the product package imports this file and it imports nothing from
the product package.  Pins: tests/test_schedule_oracle_pins.py.
"""
from __future__ import annotations

import numpy as np

from . import ernie_oracle as O


def run_job(p: O.Params, prompts_full, full_to_trimmed: np.ndarray, kept_ids: np.ndarray, n_gen: int,
            eos: int | None = None):
    """Returns (tokens_full [n_requests, n_gen] int32, min_gap [n_requests]): min_gap is the smallest top-2 logit
    gap over the computed steps of a request (a trajectory with a large min_gap is unambiguous)."""
    out = np.zeros((len(prompts_full), n_gen), dtype=np.int32)
    gaps = np.zeros(len(prompts_full))
    for r, prompt in enumerate(prompts_full):
        trimmed = full_to_trimmed[np.asarray(prompt, dtype=np.int64)]          # preprocessing
        seen_full = kept_ids[trimmed]                                          # what the model is given, as full ids
        g = O.generate_cached(p, seen_full, n_gen, kept_ids, eos=eos)          # inference
        out[r] = kept_ids[g["tokens"]]                                         # post-processing
        ok = ~np.isnan(g["logits"][:, 0])
        gaps[r] = min(O.top2_gap(z) for z in g["logits"][ok])
    return out, gaps
