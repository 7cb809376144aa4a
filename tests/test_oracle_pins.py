"""Pins for the CPU oracle: brute force, closed forms, invariants, library layers.

None of these needs a GPU.  Each pin is chosen so that a plausible mistake in
oracle/ernie_oracle.py (dropped term, wrong sign or index, transposed operand,
wrong mask edge) fails at least one of them; test_oracle_mutations.py plants
such mistakes and checks that they are caught.
"""
import math
import os
from dataclasses import replace

import numpy as np
import pytest
import torch

from oracle import ernie_oracle as O
from synth import CONFIGS, make_weights, make_kept_ids
from tests import bruteforce as BF

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def small_shape(**kw):
    base = dict(n_layers=2, d_model=16, n_heads=2, d_ffn=32, vocab_full=40, vocab_kept=20,
                max_pos=24, batch=2, prompt_len=5, n_gen=4)
    base.update(kw)
    return replace(CONFIGS["tiny_affine"], **base)


def scaled(weights, s):
    """Scale the matrices (not LN/bias) so that attention and GELU are far from linear."""
    out = {k: v for k, v in weights.items() if k != "layers"}
    out["tok_emb"] = (weights["tok_emb"].astype(np.float64) * s).astype(np.float16)
    out["pos_emb"] = (weights["pos_emb"].astype(np.float64) * s).astype(np.float16)
    out["layers"] = []
    for lw in weights["layers"]:
        n = dict(lw)
        for k in ("wqkv", "wo", "w1", "w2"):
            n[k] = (lw[k].astype(np.float64) * s).astype(np.float16)
        out["layers"].append(n)
    return out


@pytest.fixture(scope="module")
def small():
    sh = small_shape()
    w = scaled(make_weights(sh, seed=11), 12.0)
    kept = make_kept_ids(sh, seed=12)
    return sh, w, kept, O.Params(w, sh.n_heads, sh.ln_eps)


# ---------------------------------------------------------------- primitives

def test_gelu_textbook_values():
    # standard normal CDF table values: Phi(1) = 0.8413447460685429, Phi(2) = 0.9772498680518208
    rows = [l.split() for l in open(os.path.join(GOLDEN, "normal_cdf.txt")) if l.strip() and l[0] != "#"]
    for a, phi in rows:
        a, phi = float(a), float(phi)
        assert abs(O.gelu(np.array([a]))[0] - a * phi) < 1e-14
        assert abs(O.gelu(np.array([-a]))[0] - (-a) * (1 - phi)) < 1e-14
    assert O.gelu(np.array([0.0]))[0] == 0.0
    assert abs(O.gelu(np.array([30.0]))[0] - 30.0) < 1e-12
    assert abs(O.gelu(np.array([-30.0]))[0]) < 1e-12
    # against math.erf on random points (library erf vs libm erf)
    x = np.random.default_rng(0).normal(size=200) * 3
    ref = np.array([v * 0.5 * (1 + math.erf(v / math.sqrt(2))) for v in x])
    assert np.max(np.abs(O.gelu(x) - ref)) < 1e-14


def test_gelu_is_not_the_tanh_form():
    a = np.array([1.5])
    tanh_form = 0.5 * a * (1 + np.tanh(np.sqrt(2 / np.pi) * (a + 0.044715 * a ** 3)))
    assert abs(O.gelu(a)[0] - tanh_form[0]) > 1e-5


def test_layer_norm_closed_forms():
    rng = np.random.default_rng(1)
    y = rng.normal(size=(7, 33)) * 3 + 2
    one, zero = np.ones(33), np.zeros(33)
    eps = 1e-5
    out = O.layer_norm(y, one, zero, eps)
    assert np.max(np.abs(out.mean(axis=1))) < 1e-13
    var = y.var(axis=1)                      # population variance
    assert np.allclose(out.var(axis=1), var / (var + eps), rtol=1e-12)
    # constant row -> beta
    beta = rng.normal(size=33)
    const = np.full((1, 33), 4.2)
    assert np.allclose(O.layer_norm(const, rng.normal(size=33), beta, eps), beta, atol=1e-6)
    # positive scale invariance (up to eps), sign flip antisymmetry
    g = rng.normal(size=33)
    assert np.allclose(O.layer_norm(5 * y, g, beta, 0.0), O.layer_norm(y, g, beta, 0.0), atol=1e-12)
    assert np.allclose(O.layer_norm(-y, g, zero, eps), -O.layer_norm(y, g, zero, eps), atol=1e-12)
    # gamma multiplies, beta adds (a swap would fail)
    assert np.allclose(O.layer_norm(y, g, beta, eps), g * out + beta, atol=1e-12)
    # eps sits inside the square root: a tiny-variance row is damped by sqrt(var/(var+eps))
    tiny = np.array([[1e-3, -1e-3]])
    o = O.layer_norm(tiny, np.ones(2), np.zeros(2), 1e-5)
    assert np.allclose(o, tiny / math.sqrt(1e-6 + 1e-5), rtol=1e-12)
    # library cross-check
    t = torch.nn.functional.layer_norm(torch.from_numpy(y), (33,), torch.from_numpy(g),
                                       torch.from_numpy(beta), eps).numpy()
    assert np.max(np.abs(t - O.layer_norm(y, g, beta, eps))) < 1e-12


def test_softmax_rows_sum_to_one_and_closed_forms():
    rng = np.random.default_rng(2)
    n, L = 9, 4
    vis = O.visibility_matrix(n, L)
    s = rng.normal(size=(n, n)) * 5
    P = O.masked_softmax(s, vis)
    assert np.all(P >= 0)
    assert np.max(np.abs(P.sum(axis=1) - 1)) < 1e-12
    assert np.all(P[~vis] == 0.0)
    # equal scores -> uniform over the visible keys
    U = O.masked_softmax(np.full((n, n), 3.3), vis)
    for i in range(n):
        c = vis[i].sum()
        assert np.allclose(U[i, vis[i]], 1.0 / c, atol=1e-15)
    # shift invariance per row
    P2 = O.masked_softmax(s + rng.normal(size=(n, 1)) * 50, vis)
    assert np.max(np.abs(P - P2)) < 1e-12
    # invisible scores are excluded, not merely made small: a huge hidden score changes nothing
    s3 = s.copy(); s3[~vis] = 1e6
    assert np.max(np.abs(O.masked_softmax(s3, vis) - P)) == 0.0
    # library cross-check (masked rows via -inf)
    t = torch.from_numpy(np.where(vis, s, -np.inf)).softmax(dim=-1).numpy()
    assert np.max(np.abs(t - P)) < 1e-14


def test_visibility_rule():
    n, L = 7, 3
    vis = O.visibility_matrix(n, L)
    for i in range(n):
        for j in range(n):
            assert vis[i, j] == O.visible(i, j, L)
            if i < L:
                assert vis[i, j] == (j < L)          # prompt rows see the prompt, nothing generated
            else:
                assert vis[i, j] == (j <= i)         # generated rows are causal
    assert np.array_equal(O.visibility_matrix(5, 1), np.tril(np.ones((5, 5), bool)))   # L=1: purely causal
    assert O.visibility_matrix(5, 5).all()                                            # no generated tokens: encoder


def test_greedy_ties_and_gap():
    assert O.greedy(np.array([1.0, 3.0, 3.0, 2.0])) == 1
    assert O.greedy(np.array([5.0, 5.0])) == 0
    assert O.greedy(np.array([-1.0, -0.5])) == 1
    assert abs(O.top2_gap(np.array([1.0, 3.5, 3.0, 2.0])) - 0.5) < 1e-15
    assert O.top2_gap(np.array([2.0, 2.0, 1.0])) == 0.0


# ---------------------------------------------------------------- whole forward

def test_brute_force_one_layer_d8():
    """1 layer, d = 8, 1 head: scalar-loop implementation agrees to 1e-12."""
    sh = small_shape(n_layers=1, d_model=8, n_heads=1, d_ffn=16, vocab_full=12, vocab_kept=7, max_pos=12)
    w = scaled(make_weights(sh, seed=21), 15.0)
    kept = make_kept_ids(sh, seed=22)
    p = O.Params(w, 1, sh.ln_eps)
    wl = BF.to_lists(w)
    rng = np.random.default_rng(23)
    prompt = kept[rng.integers(0, len(kept), size=4)]
    ids = np.concatenate([prompt, kept[rng.integers(0, len(kept), size=3)]])
    H = O.forward_full(p, ids, 4)
    Hb = np.array(BF.forward(wl, 1, sh.ln_eps, ids.tolist(), 4))
    assert np.max(np.abs(H - Hb)) < 1e-12
    toks_b, logits_b = BF.generate(wl, 1, sh.ln_eps, prompt.tolist(), 4, kept.tolist())
    g = O.generate_full_recompute(p, prompt, 4, kept)
    assert g["tokens"].tolist() == toks_b
    assert np.max(np.abs(g["logits"] - np.array(logits_b))) < 1e-12


def test_brute_force_two_layers_two_heads(small):
    sh, w, kept, p = small
    wl = BF.to_lists(w)
    rng = np.random.default_rng(31)
    ids = rng.integers(0, sh.vocab_full, size=8)
    for L in (1, 3, 8):
        H = O.forward_full(p, ids, L)
        Hb = np.array(BF.forward(wl, sh.n_heads, sh.ln_eps, ids.tolist(), L))
        assert np.max(np.abs(H - Hb)) < 1e-12, L


def test_attention_rows_sum_to_one_in_forward(small):
    sh, w, kept, p = small
    ids = np.random.default_rng(32).integers(0, sh.vocab_full, size=9)
    probs = []
    O.forward_full(p, ids, 4, probs_out=probs)
    assert len(probs) == sh.n_layers * sh.n_heads
    vis = O.visibility_matrix(9, 4)
    for P in probs:
        assert np.max(np.abs(P.sum(axis=1) - 1)) < 1e-12
        assert np.all(P >= 0) and np.all(P[~vis] == 0)
        assert P[vis].min() > 0
    # scaled weights make the rows genuinely non-uniform, otherwise this pin is vacuous
    assert max(P[vis].max() for P in probs) > 0.5


def test_mask_invariances(small):
    sh, w, kept, p = small
    rng = np.random.default_rng(33)
    L, n = 4, 9
    ids = rng.integers(0, sh.vocab_full, size=n)
    H = O.forward_full(p, ids, L)
    # (a) changing a later generated token leaves every earlier position unchanged
    for t in range(L, n):
        ids2 = ids.copy(); ids2[t] = (ids2[t] + 1) % sh.vocab_full
        H2 = O.forward_full(p, ids2, L)
        assert np.max(np.abs(H2[:t] - H[:t])) == 0.0, t
        assert np.max(np.abs(H2[t] - H[t])) > 1e-6
    # (b) appending tokens leaves all existing positions unchanged
    H3 = O.forward_full(p, np.concatenate([ids, [3, 5]]), L)
    assert np.max(np.abs(H3[:n] - H)) < 1e-13
    # (c) truncation: prompt outputs do not depend on anything generated
    H4 = O.forward_full(p, ids[:L], L)
    assert np.max(np.abs(H4 - H[:L])) < 1e-13
    # (d) bidirectional prefix: changing the LAST prompt token changes the FIRST prompt output
    ids5 = ids.copy(); ids5[L - 1] = (ids5[L - 1] + 1) % sh.vocab_full
    H5 = O.forward_full(p, ids5, L)
    assert np.max(np.abs(H5[0] - H[0])) > 1e-6
    # ... while with L = 1 (purely causal) the first output ignores every later token
    Hc = O.forward_full(p, ids, 1)
    Hc5 = O.forward_full(p, ids5, 1)
    assert np.max(np.abs(Hc5[:L - 1] - Hc[:L - 1])) == 0.0


def test_prefix_permutation_symmetry(small):
    """Jointly permuting (token, position-row) pairs of the prompt permutes prompt outputs only."""
    sh, w, kept, p = small
    rng = np.random.default_rng(34)
    L, n = 5, 8
    ids = rng.integers(0, sh.vocab_full, size=n)
    perm = rng.permutation(L)
    w2 = dict(w)
    pe = w["pos_emb"].copy()
    pe[:L] = w["pos_emb"][perm]          # new row i = old row perm[i]
    w2["pos_emb"] = pe
    ids2 = ids.copy(); ids2[:L] = ids[perm]
    H = O.forward_full(p, ids, L)
    H2 = O.forward_full(O.Params(w2, sh.n_heads, sh.ln_eps), ids2, L)
    assert np.max(np.abs(H2[:L] - H[perm])) < 1e-12
    assert np.max(np.abs(H2[L:] - H[L:])) < 1e-12


def test_cached_equals_full_recompute(small):
    sh, w, kept, p = small
    rng = np.random.default_rng(35)
    for L in (1, 2, 6):
        prompt = kept[rng.integers(0, len(kept), size=L)]
        a = O.generate_full_recompute(p, prompt, 6, kept)
        b = O.generate_cached(p, prompt, 6, kept)
        assert np.array_equal(a["tokens"], b["tokens"])
        assert np.max(np.abs(a["hidden"] - b["hidden"])) < 1e-10
        assert np.max(np.abs(a["logits"] - b["logits"])) < 1e-10


def test_cached_teacher_forcing_matches_full_forward(small):
    sh, w, kept, p = small
    rng = np.random.default_rng(36)
    prompt = kept[rng.integers(0, len(kept), size=4)]
    forced = rng.integers(0, len(kept), size=5).astype(np.int32)
    b = O.generate_cached(p, prompt, 5, kept, forced_tokens=forced)
    seq = np.concatenate([prompt, kept[forced[:4]]])
    H = O.forward_full(p, seq, 4)
    assert np.max(np.abs(b["hidden"] - H[3:8])) < 1e-10


def test_cached_on_tiny_config():
    """Same exactness claim at the cfg-0 shape (2 layers, d=128, 2 heads, V' 512 of 1024)."""
    sh = CONFIGS["tiny_affine"]
    w = make_weights(sh)
    kept = make_kept_ids(sh)
    p = O.Params(w, sh.n_heads, sh.ln_eps)
    prompt = kept[np.random.default_rng(37).integers(0, len(kept), size=12)]
    a = O.generate_full_recompute(p, prompt, 5, kept)
    b = O.generate_cached(p, prompt, 5, kept)
    assert np.array_equal(a["tokens"], b["tokens"])
    assert np.max(np.abs(a["hidden"] - b["hidden"])) < 1e-10
    assert np.max(np.abs(a["logits"] - b["logits"])) < 1e-10


def test_pruning_is_row_selection(small):
    sh, w, kept, p = small
    h = np.random.default_rng(38).normal(size=sh.d_model)
    zf = O.logits_full_vocab(p, h)
    zk = O.logits_kept(p, h, kept)
    assert np.array_equal(zk, zf[kept])
    # explicit dot products, one row at a time
    for k, v in enumerate(kept):
        assert abs(zk[k] - float(np.dot(p.tok_emb[v], h))) < 1e-13
    # argmax over trimmed = argmax over the full table restricted to kept rows
    masked = np.full_like(zf, -np.inf); masked[kept] = zf[kept]
    assert kept[O.greedy(zk)] == int(np.argmax(masked))
    # keeping every row is the identity
    allrows = np.arange(sh.vocab_full)
    assert np.array_equal(O.logits_kept(p, h, allrows), zf)


# ---------------------------------------------------------------- special weights

def _zero_layer(lw, keys):
    n = dict(lw)
    for k in keys:
        n[k] = np.zeros_like(lw[k])
    return n


def test_zero_qk_gives_mean_of_visible_values(small):
    sh, w, kept, p = small
    lw = dict(p.layers[0])
    d = sh.d_model
    lw["wqkv"] = lw["wqkv"].copy(); lw["wqkv"][:2 * d] = 0
    lw["bqkv"] = lw["bqkv"].copy(); lw["bqkv"][:2 * d] = 0
    X = np.random.default_rng(39).normal(size=(7, d))
    L = 3
    Oo = O.attention_full(p, lw, X, L)
    V = X @ lw["wqkv"][2 * d:].T + lw["bqkv"][2 * d:]
    for i in range(7):
        c = L if i < L else i + 1
        assert np.max(np.abs(Oo[i] - V[:c].mean(axis=0))) < 1e-13


def test_zero_sublayers_reduce_to_two_layernorms(small):
    sh, w, kept, p = small
    lw = _zero_layer(p.layers[0], ("wqkv", "bqkv", "wo", "bo", "w1", "b1", "w2", "b2"))
    X = np.random.default_rng(40).normal(size=(5, sh.d_model))
    out = O.layer_full(p, lw, X, 2)
    ref = O.layer_norm(O.layer_norm(X, lw["ln1_g"], lw["ln1_b"], p.eps), lw["ln2_g"], lw["ln2_b"], p.eps)
    assert np.max(np.abs(out - ref)) < 1e-13


def test_identity_value_path_hand_computable():
    """1 head, Wq=Wk=0, Wv=Wo=I, FFN zero, LN affine trivial: X1 = LN(X + running/prefix mean of X)."""
    d = 6
    sh = small_shape(n_layers=1, d_model=d, n_heads=1, d_ffn=8, vocab_full=9, vocab_kept=9, max_pos=9)
    w = make_weights(replace(sh, trivial_affine=True), seed=41)
    lw = w["layers"][0]
    lw["wqkv"] = np.concatenate([np.zeros((2 * d, d)), np.eye(d)]).astype(np.float16)
    lw["wo"] = np.eye(d, dtype=np.float16)
    lw["w1"] = np.zeros_like(lw["w1"]); lw["w2"] = np.zeros_like(lw["w2"])
    p = O.Params(w, 1, 0.0)
    X = np.random.default_rng(42).normal(size=(5, d))
    L = 2
    out = O.layer_full(p, p.layers[0], X, L)
    one, zero = np.ones(d), np.zeros(d)
    for i in range(5):
        c = L if i < L else i + 1
        x1 = X[i] + X[:c].mean(axis=0)
        x1 = (x1 - x1.mean()) / x1.std()
        x2 = (x1 - x1.mean()) / x1.std()
        assert np.max(np.abs(out[i] - x2)) < 1e-12


# ---------------------------------------------------------------- library layers

def _torch_layer(sh, lw):
    d = sh.d_model
    layer = torch.nn.TransformerEncoderLayer(d, sh.n_heads, sh.d_ffn, dropout=0.0, activation="gelu",
                                             layer_norm_eps=sh.ln_eps, batch_first=True,
                                             norm_first=False, dtype=torch.float64)
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    with torch.no_grad():
        layer.self_attn.in_proj_weight.copy_(t(lw["wqkv"])); layer.self_attn.in_proj_bias.copy_(t(lw["bqkv"]))
        layer.self_attn.out_proj.weight.copy_(t(lw["wo"])); layer.self_attn.out_proj.bias.copy_(t(lw["bo"]))
        layer.norm1.weight.copy_(t(lw["ln1_g"])); layer.norm1.bias.copy_(t(lw["ln1_b"]))
        layer.linear1.weight.copy_(t(lw["w1"])); layer.linear1.bias.copy_(t(lw["b1"]))
        layer.linear2.weight.copy_(t(lw["w2"])); layer.linear2.bias.copy_(t(lw["b2"]))
        layer.norm2.weight.copy_(t(lw["ln2_g"])); layer.norm2.bias.copy_(t(lw["ln2_b"]))
    layer.train()   # keep the plain (non-fused) code path; dropout is 0
    return layer


def test_layer_against_torch_encoder_layer(small):
    """A post-LN library transformer layer with the prefix-LM mask equals the oracle's layer."""
    sh, w, kept, p = small
    X = np.random.default_rng(43).normal(size=(9, sh.d_model))
    L = 4
    for li in range(sh.n_layers):
        layer = _torch_layer(sh, p.layers[li])
        mask = torch.from_numpy(~O.visibility_matrix(9, L))      # True = not allowed
        with torch.no_grad():
            ref = layer(torch.from_numpy(X)[None], src_mask=mask)[0].numpy()
        out = O.layer_full(p, p.layers[li], X, L)
        assert np.max(np.abs(out - ref)) < 1e-11


def test_matmul_orientation_against_explicit_sums(small):
    """Weights are [out, in]: y_o = sum_i W[o, i] x_i + b_o (guards against a transposed operand)."""
    sh, w, kept, p = small
    lw = p.layers[0]
    x = np.random.default_rng(44).normal(size=sh.d_model)
    y = x @ lw["w1"].T + lw["b1"]
    for o in (0, 7, sh.d_ffn - 1):
        assert abs(y[o] - (sum(lw["w1"][o, i] * x[i] for i in range(sh.d_model)) + lw["b1"][o])) < 1e-13


# ---------------------------------------------------------------- precision

def test_fp32_oracle_is_far_inside_the_gpu_tolerance():
    """The same forward in float32 differs from float64 by << 3e-2 / 1e-2: tolerances measure the GPU."""
    sh = CONFIGS["tiny_affine"]
    w = make_weights(sh)
    kept = make_kept_ids(sh)
    p64 = O.Params(w, sh.n_heads, sh.ln_eps)
    p32 = O.Params(w, sh.n_heads, sh.ln_eps, dtype=np.float32)
    ids = kept[np.random.default_rng(45).integers(0, len(kept), size=40)]
    H64 = O.forward_full(p64, ids, 32)
    H32 = O.forward_full(p32, ids, 32)
    assert H32.dtype == np.float32
    assert np.max(np.abs(H64 - H32)) < 2e-5
    z64 = O.logits_kept(p64, H64[-1], kept)
    z32 = O.logits_kept(p32, H32[-1], kept)
    assert np.max(np.abs(z64 - z32)) < 2e-5


def test_position_rows_are_used(small):
    sh, w, kept, p = small
    ids = np.array([3, 3, 3])
    X = O.embed(p, ids)
    assert np.max(np.abs(X[0] - X[1])) > 1e-6
    X5 = O.embed(p, ids[:1], first_pos=2)
    assert np.array_equal(X5[0], X[2])
