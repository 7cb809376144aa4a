"""CPU oracle for length-bucketed batching -- TEST INFRASTRUCTURE.

The paper orders the inputs before inference so that less work is wasted
(Introduction: the allocation of the inference order is optimised; Related
work, "Dynamic Batch Size": the batch size follows the input sizes).  It gives
no procedure; this file defines the plain one the library implements:

  * requests are ordered by prompt length, ascending, equal lengths in their
    original order (a stable sort), so a batch pads every prompt only up to a
    neighbour's length;
  * the ordered list is cut greedily into batches: a batch grows while it has
    fewer than `max_batch` rows AND rows x (longest prompt in it) stays within
    `max_tokens` padded tokens -- short prompts therefore travel in larger
    batches than long ones.

Nothing in the product package imports this file and it imports nothing from
the product package.  Pins: tests/test_schedule_oracle_pins.py.
"""
from __future__ import annotations

import numpy as np


def plan_batches(lens, max_batch: int, max_tokens: int):
    """Returns (order, starts): `order` is the permutation of request indices, `starts` the n_batches + 1
    cut points into it (batch i = order[starts[i]:starts[i + 1]])."""
    lens = [int(x) for x in lens]
    if max_batch < 1 or max_tokens < 1 or any(l < 1 for l in lens):
        raise ValueError("bad limits or lengths")
    if lens and max(lens) > max_tokens:
        raise ValueError("a prompt alone exceeds max_tokens")
    order = sorted(range(len(lens)), key=lambda i: lens[i])      # Python's sort is stable
    starts = [0]
    rows = 0
    for pos, i in enumerate(order):
        # ascending order: the candidate row is the longest of the batch it would join
        if rows + 1 > max_batch or (rows + 1) * lens[i] > max_tokens:
            starts.append(pos)
            rows = 0
        rows += 1
    if lens:
        starts.append(len(lens))
    return np.array(order, dtype=np.int32), np.array(starts, dtype=np.int32)


def padded_tokens(lens, order, starts) -> int:
    """Sum over batches of rows x longest prompt: the token slots a padded implementation touches."""
    lens = np.asarray(lens)
    total = 0
    for a, b in zip(starts[:-1], starts[1:]):
        chunk = lens[np.asarray(order[a:b])]
        total += int(len(chunk) * chunk.max())
    return total
