"""CPU oracle for the ERNIE / UNIMO-text generation forward -- TEST INFRASTRUCTURE.

This file is the slow, plain reference that the HIP path is checked against.
It is test infrastructure only: nothing in the product package imports it, and
it imports nothing from the product package.  Everything is numpy float64; the
fp16 parameters are upcast exactly, so only activation arithmetic differs from
the GPU.

What the paper fixes and what it leaves open
--------------------------------------------
The paper (Method, "Model-level optimization") describes three exact
reorganisations of a stacked-transformer generation forward -- half-precision
arithmetic, a key/value cache that avoids recomputing earlier positions, and a
word-embedding matrix trimmed to its frequently used rows -- but prints no
equation.  The key/value cache and the trimming do not change the result, so
the oracle is the plain definition they must reproduce:

* `forward_full` recomputes the WHOLE sequence from scratch (no cache);
* `logits_kept` projects onto the FULL table and then selects the kept rows
  (no trimmed table);
* `generate_full_recompute` calls those two once per emitted token.

`CachedSequence` is a second, incremental path (keys and values of earlier
positions are stored and reused, as Method item 3 describes).  It exists to be
tested against the definition, and is the path timed as the CPU baseline.

Readings where the text is silent (each is a choice of this build):
single prefix-LM stack -- bidirectional over the prompt, causal over generated
tokens; token + learned position embedding followed by a LayerNorm; post-LN
sublayers; erf GELU; LayerNorm with population variance and eps inside the
square root; score scale 1/sqrt(head_dim); masked keys excluded from the
softmax; output projection tied to the token table, no bias; greedy argmax
with the lowest index winning exact ties; the first generated token is
emitted from the last prompt position.  Optional variants, off unless the
weight dictionary carries them: a two-row segment embedding (prompt /
generated), an output-head transform LN(gelu(W h + b)) before the tied
projection, and a per-row output bias.  End of sequence (optional `eos`
argument of the generators): a sequence that has emitted the end-of-sequence
token is finished; nothing more is computed for it and it keeps emitting that
token.

Pins: every function here is pinned by tests/test_oracle_*.py (brute force
written independently with scalar loops, closed forms, invariants, torch CPU
fp64 library layers, special weights).  No function is "parity unpinned"
against the mathematics; parity with the paper's own trained system is
unpinned because its weights and data are not public.
"""
from __future__ import annotations

import math

import numpy as np
from scipy.special import erf as _erf


# --------------------------------------------------------------------------
# primitives
# --------------------------------------------------------------------------

def layer_norm(y: np.ndarray, gamma: np.ndarray, beta: np.ndarray, eps: float) -> np.ndarray:
    """Row-wise LayerNorm: gamma * (y - mean) / sqrt(var + eps) + beta, var = population variance."""
    mean = y.mean(axis=-1, keepdims=True)
    var = ((y - mean) ** 2).mean(axis=-1, keepdims=True)
    return gamma * (y - mean) / np.sqrt(var + eps) + beta


def gelu(a: np.ndarray) -> np.ndarray:
    """Exact GELU: a * Phi(a), Phi = standard normal CDF = (1 + erf(a / sqrt 2)) / 2."""
    return a * 0.5 * (1.0 + _erf(a / math.sqrt(2.0)))


def visible(i: int, j: int, L: int) -> bool:
    """Prefix-LM visibility: query i sees key j iff j is in the prompt or j <= i."""
    return (j < L) or (j <= i)


def visibility_matrix(n: int, L: int) -> np.ndarray:
    """[n, n] boolean matrix of `visible(i, j, L)`."""
    i = np.arange(n)[:, None]
    j = np.arange(n)[None, :]
    return (j < L) | (j <= i)


def masked_softmax(scores: np.ndarray, vis: np.ndarray) -> np.ndarray:
    """Softmax along the last axis over visible entries only; invisible entries get exactly 0."""
    out = np.zeros_like(scores)
    for r in range(scores.shape[0]):
        idx = np.nonzero(vis[r])[0]
        s = scores[r, idx]
        e = np.exp(s - s.max())
        out[r, idx] = e / e.sum()
    return out


# --------------------------------------------------------------------------
# parameters
# --------------------------------------------------------------------------

class Params:
    """fp64 copy of a weight dictionary (as produced by the synthetic generator)."""

    def __init__(self, weights: dict, n_heads: int, ln_eps: float = 1e-5, dtype=np.float64):
        c = lambda a: np.asarray(a).astype(dtype)
        self.dtype = dtype
        self.n_heads = int(n_heads)
        self.eps = float(ln_eps)
        self.tok_emb = c(weights["tok_emb"])      # [V, d] FULL table
        self.pos_emb = c(weights["pos_emb"])      # [P, d]
        self.emb_ln_g = c(weights["emb_ln_g"])
        self.emb_ln_b = c(weights["emb_ln_b"])
        self.layers = [{k: c(v) for k, v in lw.items()} for lw in weights["layers"]]
        # optional variants (absent in the paper's description; present in public ERNIE / UNIMO checkpoints):
        # a segment embedding with one row for prompt positions and one for generated positions, a
        # dense + GELU + LayerNorm transform in front of the tied projection, and an output bias per vocabulary row
        opt = lambda k: c(weights[k]) if weights.get(k) is not None else None
        self.type_emb = opt("type_emb")           # [2, d]: row 0 = prompt positions, row 1 = generated positions
        self.head_w, self.head_b = opt("head_w"), opt("head_b")             # [d, d], [d]
        self.head_ln_g, self.head_ln_b = opt("head_ln_g"), opt("head_ln_b")
        self.out_bias = opt("out_bias")           # [V] over the FULL vocabulary
        self.d = self.tok_emb.shape[1]
        assert self.d % self.n_heads == 0
        self.dh = self.d // self.n_heads


# --------------------------------------------------------------------------
# the definition: full recompute
# --------------------------------------------------------------------------

def embed(p: Params, ids_full: np.ndarray, first_pos: int = 0, L: int | None = None) -> np.ndarray:
    """x_i = LN_emb(E[u_i] + Epos[first_pos + i] (+ Etype[0 if position < L else 1])).

    L is the prompt length; it only matters when the model has a segment embedding.
    """
    n = len(ids_full)
    pos = np.arange(first_pos, first_pos + n)
    y = p.tok_emb[ids_full] + p.pos_emb[pos]
    if p.type_emb is not None:
        assert L is not None
        y = y + p.type_emb[(pos >= L).astype(np.int64)]
    return layer_norm(y, p.emb_ln_g, p.emb_ln_b, p.eps)


def attention_full(p: Params, lw: dict, X: np.ndarray, L: int, probs_out: list | None = None) -> np.ndarray:
    """Multi-head self-attention over the whole sequence with the prefix-LM mask.  Returns O [n, d]."""
    n, d = X.shape
    dh = p.dh
    QKV = X @ lw["wqkv"].T + lw["bqkv"]
    Q, K, V = QKV[:, :d], QKV[:, d:2 * d], QKV[:, 2 * d:]
    vis = visibility_matrix(n, L)
    O = np.zeros((n, d), dtype=X.dtype)
    for h in range(p.n_heads):
        sl = slice(h * dh, (h + 1) * dh)
        scores = (Q[:, sl] @ K[:, sl].T) / math.sqrt(float(dh))
        P = masked_softmax(scores, vis)
        if probs_out is not None:
            probs_out.append(P)
        O[:, sl] = P @ V[:, sl]
    return O


def layer_full(p: Params, lw: dict, X: np.ndarray, L: int, probs_out: list | None = None) -> np.ndarray:
    """One post-LN transformer layer on the whole sequence."""
    O = attention_full(p, lw, X, L, probs_out)
    X1 = layer_norm(X + O @ lw["wo"].T + lw["bo"], lw["ln1_g"], lw["ln1_b"], p.eps)
    G = gelu(X1 @ lw["w1"].T + lw["b1"])
    X2 = layer_norm(X1 + G @ lw["w2"].T + lw["b2"], lw["ln2_g"], lw["ln2_b"], p.eps)
    return X2


def forward_full(p: Params, ids_full: np.ndarray, L: int, probs_out: list | None = None) -> np.ndarray:
    """Final-layer hidden states [n, d] of a sequence whose first L tokens are the prompt."""
    ids_full = np.asarray(ids_full)
    assert 1 <= L <= len(ids_full)
    X = embed(p, ids_full, 0, L)
    for lw in p.layers:
        X = layer_full(p, lw, X, L, probs_out)
    return X


def head_transform(p: Params, h: np.ndarray) -> np.ndarray:
    """t = LN_head(gelu(W_head h + b_head)) if the model has an output-head transform, else h."""
    if p.head_w is None:
        return h
    return layer_norm(gelu(p.head_w @ h + p.head_b), p.head_ln_g, p.head_ln_b, p.eps)


def logits_full_vocab(p: Params, h: np.ndarray) -> np.ndarray:
    """z_v = t . E[v] (+ bias_v) over the full, untrimmed table, t = head_transform(h)."""
    z = p.tok_emb @ head_transform(p, h)
    return z if p.out_bias is None else z + p.out_bias


def logits_kept(p: Params, h: np.ndarray, kept_ids: np.ndarray) -> np.ndarray:
    """Logits over the trimmed vocabulary: full-table logits restricted to the kept rows."""
    return logits_full_vocab(p, h)[kept_ids]


def greedy(z: np.ndarray) -> int:
    """Index of the maximum; the lowest index wins exact ties."""
    best, arg = z[0], 0
    for k in range(1, len(z)):
        if z[k] > best:
            best, arg = z[k], k
    return arg


def top2_gap(z: np.ndarray) -> float:
    """Difference between the largest and second-largest logit."""
    part = np.partition(z, len(z) - 2)
    return float(part[-1] - part[-2])


def generate_full_recompute(p: Params, prompt_full: np.ndarray, n_gen: int, kept_ids: np.ndarray,
                            eos: int | None = None):
    """Greedy generation by the definition: every token re-runs the whole forward.

    Returns dict with
      tokens  [n_gen]      trimmed indices k (full id = kept_ids[k])
      hidden  [n_gen, d]   final hidden state at the emitting position
      logits  [n_gen, V']  logits over the kept rows
    `eos` (a trimmed index, optional): once the sequence has emitted it, generation of this sequence is
    over -- nothing more is computed, every later token is `eos` and the later hidden / logits rows are NaN.
    """
    prompt_full = np.asarray(prompt_full)
    L = len(prompt_full)
    seq = list(prompt_full)
    toks, hid, lg = [], [], []
    done = False
    for _ in range(n_gen):
        if done:
            toks.append(eos); hid.append(np.full(p.d, np.nan)); lg.append(np.full(len(kept_ids), np.nan))
            continue
        H = forward_full(p, np.array(seq), L)
        h = H[-1]
        z = logits_kept(p, h, kept_ids)
        k = greedy(z)
        toks.append(k); hid.append(h); lg.append(z)
        if eos is not None and k == eos:
            done = True
        seq.append(int(kept_ids[k]))
    return {"tokens": np.array(toks, dtype=np.int32), "hidden": np.array(hid), "logits": np.array(lg)}


# --------------------------------------------------------------------------
# the incremental path: keys and values of earlier positions are cached
# --------------------------------------------------------------------------

class CachedSequence:
    """One sequence decoded incrementally with a per-layer key/value cache.

    `prefill(prompt)` processes the prompt bidirectionally and stores K, V of
    every prompt position; `step(token)` processes one more token, appending
    its K, V and attending over everything cached (which is exactly what the
    prefix-LM mask allows a generated position to see).
    """

    def __init__(self, p: Params):
        self.p = p
        self.K = [None] * len(p.layers)   # each [n_cached, d]
        self.V = [None] * len(p.layers)
        self.n = 0

    def _attend(self, lw, Q, K, V):
        p = self.p
        dh = p.dh
        O = np.zeros_like(Q)
        for h in range(p.n_heads):
            sl = slice(h * dh, (h + 1) * dh)
            s = (Q[:, sl] @ K[:, sl].T) / math.sqrt(float(dh))
            s = s - s.max(axis=1, keepdims=True)
            e = np.exp(s)
            O[:, sl] = (e / e.sum(axis=1, keepdims=True)) @ V[:, sl]
        return O

    def _layers(self, X):
        p = self.p
        d = p.d
        for li, lw in enumerate(p.layers):
            QKV = X @ lw["wqkv"].T + lw["bqkv"]
            Q, Kn, Vn = QKV[:, :d], QKV[:, d:2 * d], QKV[:, 2 * d:]
            self.K[li] = Kn if self.K[li] is None else np.concatenate([self.K[li], Kn], axis=0)
            self.V[li] = Vn if self.V[li] is None else np.concatenate([self.V[li], Vn], axis=0)
            O = self._attend(lw, Q, self.K[li], self.V[li])
            X1 = layer_norm(X + O @ lw["wo"].T + lw["bo"], lw["ln1_g"], lw["ln1_b"], p.eps)
            G = gelu(X1 @ lw["w1"].T + lw["b1"])
            X = layer_norm(X1 + G @ lw["w2"].T + lw["b2"], lw["ln2_g"], lw["ln2_b"], p.eps)
        return X

    def prefill(self, prompt_full: np.ndarray) -> np.ndarray:
        """Process the whole prompt; returns the final hidden state of its last position."""
        assert self.n == 0
        X = embed(self.p, np.asarray(prompt_full), 0, len(prompt_full))
        H = self._layers(X)
        self.n = self.L = len(prompt_full)
        return H[-1]

    def step(self, token_full: int) -> np.ndarray:
        """Process one generated token at position n; returns its final hidden state."""
        X = embed(self.p, np.array([token_full]), first_pos=self.n, L=self.L)
        H = self._layers(X)
        self.n += 1
        return H[0]


def generate_cached(p: Params, prompt_full: np.ndarray, n_gen: int, kept_ids: np.ndarray,
                    forced_tokens: np.ndarray | None = None, eos: int | None = None):
    """Greedy generation with the key/value cache.  Same return value as the full-recompute form.

    `forced_tokens` (trimmed indices) replaces the fed-back token at each step
    (the emitted argmax is still reported), for teacher-forced comparisons.
    `eos`: the sequence is over once the token fed back is `eos` (free-running: once it has emitted it);
    later tokens are `eos`, later hidden / logits rows NaN, and no further step is computed.
    "steps" in the result counts the forward steps actually run (prefill included).
    """
    cs = CachedSequence(p)
    toks, hid, lg = [], [], []
    h = cs.prefill(prompt_full)
    done, steps = False, 1
    for t in range(n_gen):
        if done:
            toks.append(eos); hid.append(np.full(p.d, np.nan)); lg.append(np.full(len(kept_ids), np.nan))
            continue
        z = logits_kept(p, h, kept_ids)
        k = greedy(z)
        toks.append(k); hid.append(h); lg.append(z)
        if t + 1 < n_gen:
            feed = k if forced_tokens is None else int(forced_tokens[t])
            if eos is not None and feed == eos:
                done = True
            else:
                h = cs.step(int(kept_ids[feed]))
                steps += 1
    return {"tokens": np.array(toks, dtype=np.int32), "hidden": np.array(hid), "logits": np.array(lg),
            "steps": steps}
