"""Planted mistakes in the oracle must be caught by the pins (CPU only).

Each case monkeypatches one oracle function with a plausible wrong version and
asserts that at least one pin from test_oracle_pins.py fails.  This guards the
pins themselves: a pin set that lets one of these through is too weak.
"""
import math

import numpy as np
import pytest

from oracle import ernie_oracle as O
from tests import test_oracle_pins as P


def _small():
    sh = P.small_shape()
    w = P.scaled(P.make_weights(sh, seed=11), 12.0)
    kept = P.make_kept_ids(sh, seed=12)
    return sh, w, kept, O.Params(w, sh.n_heads, sh.ln_eps)


def _run_pins():
    """Run the pins; return the names of those that fail."""
    failed = []
    small = _small()
    for name in sorted(dir(P)):
        if not name.startswith("test_"):
            continue
        fn = getattr(P, name)
        try:
            if "small" in fn.__code__.co_varnames[:fn.__code__.co_argcount]:
                fn(small)
            else:
                fn()
        except AssertionError:
            failed.append(name)
        except Exception:      # a mistake that crashes a pin is also caught
            failed.append(name)
    return failed


def test_pins_pass_unmutated():
    assert _run_pins() == []


def _gelu_tanh(a):
    return 0.5 * a * (1 + np.tanh(math.sqrt(2 / math.pi) * (a + 0.044715 * a ** 3)))


def _ln_unbiased(y, g, b, eps):
    m = y.mean(axis=-1, keepdims=True)
    v = ((y - m) ** 2).sum(axis=-1, keepdims=True) / (y.shape[-1] - 1)
    return g * (y - m) / np.sqrt(v + eps) + b


def _ln_eps_outside(y, g, b, eps):
    m = y.mean(axis=-1, keepdims=True)
    v = ((y - m) ** 2).mean(axis=-1, keepdims=True)
    return g * (y - m) / (np.sqrt(v) + eps) + b


def _ln_swapped_affine(y, g, b, eps):
    m = y.mean(axis=-1, keepdims=True)
    v = ((y - m) ** 2).mean(axis=-1, keepdims=True)
    return b * (y - m) / np.sqrt(v + eps) + g


def _vis_causal(n, L):
    i = np.arange(n)[:, None]; j = np.arange(n)[None, :]
    return j <= i


def _vis_off_by_one(n, L):
    i = np.arange(n)[:, None]; j = np.arange(n)[None, :]
    return (j < L) | (j < i) | (i == j) & (i < L)


def _vis_prompt_sees_all(n, L):
    i = np.arange(n)[:, None]; j = np.arange(n)[None, :]
    return (i < L) | (j <= i)


def _softmax_additive_mask(scores, vis):
    s = np.where(vis, scores, scores - 1e4)
    e = np.exp(s - s.max(axis=1, keepdims=True))
    return e / e.sum(axis=1, keepdims=True)


def _greedy_last(z):
    return int(len(z) - 1 - np.argmax(z[::-1]))


def _logits_kept_prefix(p, h, kept):
    return O.logits_full_vocab(p, h)[:len(kept)]


def _embed_no_offset(p, ids, first_pos=0):
    n = len(ids)
    return O.layer_norm(p.tok_emb[ids] + p.pos_emb[np.arange(n)], p.emb_ln_g, p.emb_ln_b, p.eps)


def _layer_no_second_residual(p, lw, X, L, probs_out=None):
    Oo = O.attention_full(p, lw, X, L, probs_out)
    X1 = O.layer_norm(X + Oo @ lw["wo"].T + lw["bo"], lw["ln1_g"], lw["ln1_b"], p.eps)
    G = O.gelu(X1 @ lw["w1"].T + lw["b1"])
    return O.layer_norm(G @ lw["w2"].T + lw["b2"], lw["ln2_g"], lw["ln2_b"], p.eps)


def _layer_pre_ln(p, lw, X, L, probs_out=None):
    Xn = O.layer_norm(X, lw["ln1_g"], lw["ln1_b"], p.eps)
    X1 = X + O.attention_full(p, lw, Xn, L, probs_out) @ lw["wo"].T + lw["bo"]
    Xn = O.layer_norm(X1, lw["ln2_g"], lw["ln2_b"], p.eps)
    return X1 + O.gelu(Xn @ lw["w1"].T + lw["b1"]) @ lw["w2"].T + lw["b2"]


def _attention_unscaled(p, lw, X, L, probs_out=None):
    n, d = X.shape
    QKV = X @ lw["wqkv"].T + lw["bqkv"]
    Q, K, V = QKV[:, :d], QKV[:, d:2 * d], QKV[:, 2 * d:]
    vis = O.visibility_matrix(n, L)
    out = np.zeros((n, d))
    for h in range(p.n_heads):
        sl = slice(h * p.dh, (h + 1) * p.dh)
        Pm = O.masked_softmax(Q[:, sl] @ K[:, sl].T, vis)
        if probs_out is not None:
            probs_out.append(Pm)
        out[:, sl] = Pm @ V[:, sl]
    return out


def _attention_kv_swapped(p, lw, X, L, probs_out=None):
    n, d = X.shape
    QKV = X @ lw["wqkv"].T + lw["bqkv"]
    Q, V, K = QKV[:, :d], QKV[:, d:2 * d], QKV[:, 2 * d:]
    vis = O.visibility_matrix(n, L)
    out = np.zeros((n, d))
    for h in range(p.n_heads):
        sl = slice(h * p.dh, (h + 1) * p.dh)
        Pm = O.masked_softmax(Q[:, sl] @ K[:, sl].T / math.sqrt(p.dh), vis)
        if probs_out is not None:
            probs_out.append(Pm)
        out[:, sl] = Pm @ V[:, sl]
    return out


MUTATIONS = [
    ("gelu", _gelu_tanh),
    ("layer_norm", _ln_unbiased),
    ("layer_norm", _ln_eps_outside),
    ("layer_norm", _ln_swapped_affine),
    ("visibility_matrix", _vis_causal),
    ("visibility_matrix", _vis_off_by_one),
    ("visibility_matrix", _vis_prompt_sees_all),
    ("masked_softmax", _softmax_additive_mask),
    ("greedy", _greedy_last),
    ("logits_kept", _logits_kept_prefix),
    ("embed", _embed_no_offset),
    ("layer_full", _layer_no_second_residual),
    ("layer_full", _layer_pre_ln),
    ("attention_full", _attention_unscaled),
    ("attention_full", _attention_kv_swapped),
]


@pytest.mark.parametrize("name,wrong", MUTATIONS, ids=[f"{n}:{f.__name__}" for n, f in MUTATIONS])
def test_planted_mistake_is_caught(monkeypatch, name, wrong):
    monkeypatch.setattr(O, name, wrong)
    failed = _run_pins()
    assert failed, f"mutation {wrong.__name__} of {name} passed every pin"


def test_cached_path_mistake_is_caught(monkeypatch):
    """A cache that forgets the newest key (attends over n-1 entries) breaks cached == full."""
    orig = O.CachedSequence._attend

    def wrong(self, lw, Q, K, V):
        if Q.shape[0] == 1 and K.shape[0] > 1:
            return orig(self, lw, Q, K[:-1], V[:-1])
        return orig(self, lw, Q, K, V)

    monkeypatch.setattr(O.CachedSequence, "_attend", wrong)
    assert "test_cached_equals_full_recompute" in _run_pins()
