"""CPU oracle for vocabulary trimming -- TEST INFRASTRUCTURE.

The paper (Method, "Embedding layer pruning") keeps only the frequently used
rows of the word-embedding matrix and drops the rarely used ones.  It prints
no procedure, so this file is the plain definition of the obvious one, in
numpy integer arithmetic (every result here is exact):

  1. count how often each vocabulary id occurs in a corpus;
  2. keep the k most frequent ids (a few reserved ids, such as the unknown-word
     token, are kept whatever their count);
  3. re-index: kept ids get trimmed indices 0..k-1 in ascending id order,
     every dropped id maps to the trimmed index of the unknown-word token;
  4. the trimmed table is rows `kept_ids` of the full table; emitted trimmed
     ids go back to full ids through `kept_ids`.

Readings where the text is silent (choices of this build): frequency is the raw
occurrence count; ids outside [0, V) are not counted; equal counts are ordered
by lower id first; reserved ids come before all others; `kept_ids` is ascending.

Nothing in the product package imports this file and it imports nothing from
the product package.  Pins: tests/test_prune_oracle_pins.py (scalar-loop brute
force, ordering invariants, the closed-form coverage of a Zipf law, round trips).
No function here is "parity unpinned".
"""
from __future__ import annotations

import numpy as np


def count_tokens(ids: np.ndarray, vocab: int, counts: np.ndarray | None = None) -> np.ndarray:
    """Step 1: occurrences of every id in [0, vocab); other values are ignored.  Adds to `counts` if given."""
    ids = np.asarray(ids).reshape(-1).astype(np.int64)
    ok = (ids >= 0) & (ids < vocab)
    c = np.bincount(ids[ok], minlength=vocab).astype(np.uint64)
    return c if counts is None else counts.astype(np.uint64) + c


def select_kept(counts: np.ndarray, k: int, reserved=()) -> np.ndarray:
    """Step 2: ascending ids of the k rows to keep.

    Order of preference: reserved ids, then higher count, then lower id.
    """
    counts = np.asarray(counts).astype(np.uint64)
    vocab = counts.shape[0]
    reserved = [int(r) for r in reserved]
    if not (0 < k <= vocab) or len(set(reserved)) != len(reserved) or len(reserved) > k:
        raise ValueError("bad k or reserved ids")
    if any(r < 0 or r >= vocab for r in reserved):
        raise ValueError("reserved id out of range")
    forced = np.zeros(vocab, dtype=bool)
    forced[reserved] = True
    ids = np.arange(vocab)
    # lexsort: last key is the primary one
    order = np.lexsort((ids, -counts.astype(np.int64), ~forced))
    return np.sort(order[:k]).astype(np.int32)


def full_to_trimmed_map(kept_ids: np.ndarray, vocab: int, unk_full_id: int) -> np.ndarray:
    """Step 3: table [vocab] of trimmed indices; dropped ids point at the unknown-word row."""
    kept_ids = np.asarray(kept_ids).astype(np.int64)
    where = np.nonzero(kept_ids == unk_full_id)[0]
    if where.size != 1:
        raise ValueError("the unknown-word id must be kept exactly once")
    m = np.full(vocab, int(where[0]), dtype=np.int32)
    m[kept_ids] = np.arange(kept_ids.shape[0], dtype=np.int32)
    return m


def remap(ids: np.ndarray, table: np.ndarray, fallback: int) -> np.ndarray:
    """Steps 3/4 applied to data: out = table[id] for ids inside the table, `fallback` otherwise."""
    ids = np.asarray(ids)
    flat = ids.reshape(-1).astype(np.int64)
    ok = (flat >= 0) & (flat < table.shape[0])
    out = np.full(flat.shape, fallback, dtype=np.int32)
    out[ok] = table[flat[ok]]
    return out.reshape(ids.shape)


def trim_rows(table_full: np.ndarray, kept_ids: np.ndarray) -> np.ndarray:
    """Step 4: rows `kept_ids` of the full table, bit for bit."""
    return np.ascontiguousarray(table_full[np.asarray(kept_ids).astype(np.int64)])


def coverage(counts: np.ndarray, kept_ids: np.ndarray) -> float:
    """Share of the counted corpus whose ids survive trimming."""
    counts = np.asarray(counts).astype(np.float64)
    return float(counts[np.asarray(kept_ids).astype(np.int64)].sum() / counts.sum())
