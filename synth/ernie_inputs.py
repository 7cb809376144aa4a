"""Seeded generators for ERNIE-shaped synthetic workloads.

The paper measures on a proprietary summarisation corpus with trained
UNIMO-text weights (Experiments, "Dataset"); neither is available, so these
generators stand in for them.  They reproduce what the text states of the
data's shape -- short inputs against a 512-row position table and a vocabulary
dominated by a small set of frequent rows (Method, "Embedding layer pruning")
-- with the exact shapes of the five benchmark configurations.

Nothing here is part of the method: no matmul, softmax, normalisation or
argmax.  Only random draws, sorting of lengths, and id re-indexing.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, List, Optional

import numpy as np


@dataclass(frozen=True)
class ErnieShape:
    """Static shape of one benchmark configuration."""
    name: str
    cfg: int                 # seed offset
    n_layers: int
    d_model: int
    n_heads: int
    d_ffn: int
    vocab_full: int          # V
    vocab_kept: int          # V'
    max_pos: int             # P
    batch: int               # B (per batch)
    prompt_len: int          # fixed prompt length, or max length when varlen
    n_gen: int               # N tokens generated per sequence (1 prefill + N-1 decode)
    kept: str = "all"        # "all" | "uniform" | "top"
    ids: str = "zipf"        # "zipf" | "uniform_kept"
    varlen_lo: int = 0       # >0: lengths uniform in [varlen_lo, prompt_len]
    varlen_pool: int = 0     # number of sequences drawn before batching
    trivial_affine: bool = True   # LN gamma=1 beta=0, biases 0
    extras: bool = False     # also draw a segment embedding, an output-head transform and an output bias
    ln_eps: float = 1e-5

    @property
    def head_dim(self) -> int:
        return self.d_model // self.n_heads


CONFIGS: Dict[str, ErnieShape] = {
    # cfg 0: tiny prefix-LM, uniformly drawn kept rows
    "tiny": ErnieShape("tiny", 0, 2, 128, 2, 512, 1024, 512, 64, 2, 32, 16,
                       kept="uniform", ids="uniform_kept"),
    # cfg 0b: same shape, non-trivial biases / LN affine so that a dropped bias
    # or swapped gamma/beta cannot pass unnoticed
    "tiny_affine": ErnieShape("tiny_affine", 5, 2, 128, 2, 512, 1024, 512, 64, 2, 32, 16,
                              kept="uniform", ids="uniform_kept", trivial_affine=False),
    # cfg 0c: cfg 0b plus the optional variants (segment embedding, output-head transform, output bias)
    "tiny_head": ErnieShape("tiny_head", 6, 2, 128, 2, 512, 1024, 512, 64, 2, 32, 16,
                            kept="uniform", ids="uniform_kept", trivial_affine=False, extras=True),
    # cfg 1: ERNIE-base, no pruning
    "base": ErnieShape("base", 1, 12, 768, 12, 3072, 18000, 18000, 512, 32, 128, 32),
    # cfg 2: ERNIE-base, pruned to the 6000 most frequent rows, variable lengths
    "base_pruned_varlen": ErnieShape("base_pruned_varlen", 2, 12, 768, 12, 3072, 18000, 6000,
                                     512, 64, 256, 32, kept="top", varlen_lo=16, varlen_pool=512),
    # cfg 3: ERNIE-large (the paper's 24 x 1024 model shape)
    "large": ErnieShape("large", 3, 24, 1024, 16, 4096, 18000, 8000, 512, 128, 256, 64, kept="top"),
    # cfg 4: decode-bound; positions reach 512+128-1 so the table has 640 rows
    "decode_bound": ErnieShape("decode_bound", 4, 12, 768, 12, 3072, 18000, 6000, 640, 256, 512,
                               128, kept="top"),
}


def _normal_f16(rng: np.random.Generator, shape, std: float = 0.02, mean: float = 0.0) -> np.ndarray:
    """fp64 N(mean, std^2) draw rounded to fp16 (round-to-nearest-even)."""
    return (mean + std * rng.standard_normal(shape)).astype(np.float16)


def make_weights(shape: ErnieShape, seed: Optional[int] = None) -> dict:
    """Random fp16 parameters; the fp16 values are the canonical weights.

    Draw order: token table, position table, embedding LN, then per layer
    wqkv, bqkv, wo, bo, ln1, w1, b1, w2, b2, ln2.  All matrices are stored
    [out, in] row-major.  Rows of wqkv: 0..d-1 = Q, d..2d-1 = K, 2d..3d-1 = V.
    """
    rng = np.random.default_rng(np.random.PCG64(1000 + shape.cfg if seed is None else seed))
    d, f = shape.d_model, shape.d_ffn
    triv = shape.trivial_affine

    def gamma(n):
        return np.ones(n, np.float16) if triv else _normal_f16(rng, n, 0.1, 1.0)

    def beta(n):
        return np.zeros(n, np.float16) if triv else _normal_f16(rng, n, 0.1, 0.0)

    def bias(n):
        return np.zeros(n, np.float16) if triv else _normal_f16(rng, n, 0.02, 0.0)

    w = {
        "tok_emb": _normal_f16(rng, (shape.vocab_full, d)),
        "pos_emb": _normal_f16(rng, (shape.max_pos, d)),
        "emb_ln_g": gamma(d), "emb_ln_b": beta(d),
        "layers": [],
    }
    for _ in range(shape.n_layers):
        w["layers"].append({
            "wqkv": _normal_f16(rng, (3 * d, d)), "bqkv": bias(3 * d),
            "wo": _normal_f16(rng, (d, d)), "bo": bias(d),
            "ln1_g": gamma(d), "ln1_b": beta(d),
            "w1": _normal_f16(rng, (f, d)), "b1": bias(f),
            "w2": _normal_f16(rng, (d, f)), "b2": bias(d),
            "ln2_g": gamma(d), "ln2_b": beta(d),
        })
    if shape.extras:
        # drawn after everything else, so the parameters above are the same with and without the variants
        w["type_emb"] = _normal_f16(rng, (2, d))
        w["head_w"] = _normal_f16(rng, (d, d), 0.05)
        w["head_b"] = _normal_f16(rng, d, 0.1)
        w["head_ln_g"] = _normal_f16(rng, d, 0.1, 1.0)
        w["head_ln_b"] = _normal_f16(rng, d, 0.1)
        w["out_bias"] = _normal_f16(rng, shape.vocab_full, 0.1)
    return w


def make_kept_ids(shape: ErnieShape, seed: Optional[int] = None) -> np.ndarray:
    """Ascending full-vocabulary ids of the rows that survive trimming."""
    if shape.kept == "all":
        assert shape.vocab_kept == shape.vocab_full
        return np.arange(shape.vocab_full, dtype=np.int32)
    if shape.kept == "top":
        # Zipf rank r <-> id r-1, so the most frequent rows are the lowest ids
        return np.arange(shape.vocab_kept, dtype=np.int32)
    rng = np.random.default_rng(np.random.PCG64(2000 + shape.cfg if seed is None else seed))
    ids = rng.choice(shape.vocab_full, size=shape.vocab_kept, replace=False)
    return np.sort(ids).astype(np.int32)


def _zipf_p(vocab: int, s: float = 1.1) -> np.ndarray:
    p = np.arange(1, vocab + 1, dtype=np.float64) ** (-s)
    return p / p.sum()


def make_prompts(shape: ErnieShape, kept_ids: np.ndarray, seed: Optional[int] = None,
                 len_seed: Optional[int] = None) -> List[List[np.ndarray]]:
    """Prompt ids in FULL-vocabulary space, grouped into batches.

    Returns a list of batches; each batch is a list of int32 arrays (one per
    sequence, unpadded).  Variable-length configs draw `varlen_pool` lengths,
    sort ascending and cut into batches of `shape.batch`.
    """
    rng = np.random.default_rng(np.random.PCG64(3000 + shape.cfg if seed is None else seed))
    if shape.varlen_lo > 0:
        lrng = np.random.default_rng(np.random.PCG64(4000 + shape.cfg if len_seed is None else len_seed))
        lens = lrng.integers(shape.varlen_lo, shape.prompt_len + 1, size=shape.varlen_pool)
    else:
        lens = np.full(shape.batch, shape.prompt_len, dtype=np.int64)

    if shape.ids == "uniform_kept":
        def draw(n):
            return kept_ids[rng.integers(0, len(kept_ids), size=n)].astype(np.int32)
    else:
        p = _zipf_p(shape.vocab_full)

        def draw(n):
            return rng.choice(shape.vocab_full, size=n, p=p).astype(np.int32)

    seqs = [draw(int(n)) for n in lens]
    if shape.varlen_lo > 0:
        order = np.argsort(lens, kind="stable")
        seqs = [seqs[i] for i in order]
    return [seqs[i:i + shape.batch] for i in range(0, len(seqs), shape.batch)]


def make_corpus(vocab: int, n_tokens: int, seed: int = 5000, s: float = 1.1, shuffle_ranks: bool = True,
                noise_ids: int = 0) -> np.ndarray:
    """A synthetic token stream for frequency counting: bounded Zipf over ranks 1..vocab.

    Rank r is carried by id `perm[r - 1]`, a seeded permutation of the
    vocabulary (identity if `shuffle_ranks` is False), so the frequent rows are
    scattered over the id range.  `noise_ids` values outside [0, vocab) are
    mixed in at seeded positions (malformed input that a counter must ignore).
    """
    rng = np.random.default_rng(np.random.PCG64(seed))
    cdf = np.cumsum(_zipf_p(vocab, s))
    ranks = np.minimum(np.searchsorted(cdf, rng.random(n_tokens), side="right"), vocab - 1)
    perm = rng.permutation(vocab) if shuffle_ranks else np.arange(vocab)
    ids = perm[ranks].astype(np.int32)
    if noise_ids:
        where = rng.choice(n_tokens, size=noise_ids, replace=False)
        ids[where] = np.where(rng.random(noise_ids) < 0.5, -1 - rng.integers(0, 1000, size=noise_ids),
                              vocab + rng.integers(0, 1000, size=noise_ids)).astype(np.int32)
    return ids


def full_to_trimmed(ids_full: np.ndarray, kept_ids: np.ndarray, unk_full_id: int | None = None) -> np.ndarray:
    """Re-index full-vocabulary ids into the trimmed table (input preparation only).

    Ids whose row was dropped map to the trimmed index of the unknown-word id, the rule of the
    trimming step; the synthetic workloads reserve the lowest kept id as that word, so the
    default lands on trimmed index 0.
    """
    kept_ids = np.asarray(kept_ids)
    unk = int(kept_ids[0]) if unk_full_id is None else int(unk_full_id)
    unk_pos = int(np.searchsorted(kept_ids, unk))
    if unk_pos >= len(kept_ids) or int(kept_ids[unk_pos]) != unk:
        raise ValueError("the unknown-word id must be a kept id")
    pos = np.searchsorted(kept_ids, ids_full)
    pos = np.minimum(pos, len(kept_ids) - 1)
    hit = kept_ids[pos] == ids_full
    return np.where(hit, pos, unk_pos).astype(np.int32)


def trim_table(tok_emb: np.ndarray, kept_ids: np.ndarray) -> np.ndarray:
    """Rows `kept_ids` of the full token table (pure indexing)."""
    return np.ascontiguousarray(tok_emb[kept_ids])


@dataclass
class Workload:
    shape: ErnieShape
    weights: dict
    kept_ids: np.ndarray
    # per batch: list of sequences, in trimmed index space and mapped back to
    # full ids (OOV already replaced by UNK on both sides)
    batches_trimmed: List[List[np.ndarray]] = field(default_factory=list)
    batches_full: List[List[np.ndarray]] = field(default_factory=list)

    def padded(self, batch: int = 0):
        """(ids [B, Lmax] int32 right-padded with 0, lens [B] int32) of one batch."""
        seqs = self.batches_trimmed[batch]
        lens = np.array([len(s) for s in seqs], dtype=np.int32)
        ids = np.zeros((len(seqs), int(lens.max())), dtype=np.int32)
        for i, s in enumerate(seqs):
            ids[i, :len(s)] = s
        return ids, lens


def make_workload(name: str, **overrides) -> Workload:
    """Everything one configuration needs, from fixed seeds."""
    shape = CONFIGS[name]
    if overrides:
        shape = replace(shape, **overrides)
    kept = make_kept_ids(shape)
    w = make_weights(shape)
    raw = make_prompts(shape, kept)
    wl = Workload(shape, w, kept)
    for b in raw:
        tb = [full_to_trimmed(s, kept) for s in b]
        wl.batches_trimmed.append(tb)
        wl.batches_full.append([kept[t].astype(np.int32) for t in tb])
    return wl
