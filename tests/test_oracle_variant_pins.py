"""Pins for the optional model variants of the oracle (segment embedding, output-head transform,
output bias): scalar-loop brute force, reductions to the already pinned plain model, a library layer,
exact bias arithmetic, planted mistakes."""
from dataclasses import replace

import numpy as np
import pytest
import torch

from oracle import ernie_oracle as O
from synth import CONFIGS, make_weights, make_kept_ids, make_workload
from tests import bruteforce as BF
from tests.test_oracle_pins import scaled


def small_extras(**kw):
    base = dict(n_layers=2, d_model=16, n_heads=2, d_ffn=32, vocab_full=40, vocab_kept=20,
                max_pos=24, batch=2, prompt_len=5, n_gen=4)
    base.update(kw)
    return replace(CONFIGS["tiny_head"], **base)


def with_extras(w_scaled, w_raw):
    out = dict(w_scaled)
    for k in ("type_emb", "head_w", "head_b", "head_ln_g", "head_ln_b", "out_bias"):
        out[k] = w_raw[k]
    out["type_emb"] = (w_raw["type_emb"].astype(np.float64) * 12.0).astype(np.float16)
    out["head_w"] = (w_raw["head_w"].astype(np.float64) * 6.0).astype(np.float16)
    return out


@pytest.fixture(scope="module")
def small():
    sh = small_extras()
    raw = make_weights(sh, seed=51)
    w = with_extras(scaled(raw, 12.0), raw)
    kept = make_kept_ids(sh, seed=52)
    return sh, w, kept, O.Params(w, sh.n_heads, sh.ln_eps)


def test_extras_do_not_disturb_the_plain_parameters():
    a = make_weights(CONFIGS["tiny_affine"], seed=3)
    b = make_weights(replace(CONFIGS["tiny_affine"], extras=True), seed=3)
    assert a["tok_emb"].tobytes() == b["tok_emb"].tobytes()
    assert a["layers"][-1]["ln2_b"].tobytes() == b["layers"][-1]["ln2_b"].tobytes()
    assert "head_w" in b and "head_w" not in a


def test_brute_force_with_all_variants(small):
    sh, w, kept, p = small
    wl = BF.to_lists(w)
    rng = np.random.default_rng(53)
    ids = rng.integers(0, sh.vocab_full, size=8)
    for L in (1, 3, 8):
        H = O.forward_full(p, ids, L)
        Hb = np.array(BF.forward(wl, sh.n_heads, sh.ln_eps, ids.tolist(), L))
        assert np.max(np.abs(H - Hb)) < 1e-12, L
    prompt = kept[rng.integers(0, len(kept), size=4)]
    toks_b, logits_b = BF.generate(wl, sh.n_heads, sh.ln_eps, prompt.tolist(), 4, kept.tolist())
    for fn in (O.generate_full_recompute, O.generate_cached):
        g = fn(p, prompt, 4, kept)
        assert g["tokens"].tolist() == toks_b
        assert np.max(np.abs(g["logits"] - np.array(logits_b))) < 1e-11


def test_segment_rows_fold_into_the_position_table(small):
    """For a fixed prompt length L the segment embedding is a position-dependent constant, so the model equals
    a plain model whose position row p carries type row [p >= L] as well."""
    sh, w, kept, p = small
    rng = np.random.default_rng(54)
    ids = rng.integers(0, sh.vocab_full, size=9)
    for L in (2, 9):
        folded = {k: v for k, v in w.items() if k != "type_emb"}
        pe = w["pos_emb"].astype(np.float64).copy()
        te = w["type_emb"].astype(np.float64)
        pe[:L] += te[0]; pe[L:] += te[1]
        folded["pos_emb"] = pe                      # kept in fp64: no rounding of the sum
        q = O.Params(folded, sh.n_heads, sh.ln_eps)
        assert q.type_emb is None
        assert np.max(np.abs(O.forward_full(p, ids, L) - O.forward_full(q, ids, L))) < 1e-12
    # the two rows really differ in effect: swapping them changes the result
    sw = dict(w); sw["type_emb"] = w["type_emb"][::-1].copy()
    assert np.max(np.abs(O.forward_full(O.Params(sw, sh.n_heads, sh.ln_eps), ids, 4) - O.forward_full(p, ids, 4))) > 1e-3


def test_cached_path_switches_segment_at_the_prompt_boundary():
    wl = make_workload("tiny_head")
    p = O.Params(wl.weights, wl.shape.n_heads, wl.shape.ln_eps)
    prompt = wl.batches_full[0][1][:9]
    a = O.generate_full_recompute(p, prompt, 5, wl.kept_ids)
    b = O.generate_cached(p, prompt, 5, wl.kept_ids)
    assert a["tokens"].tolist() == b["tokens"].tolist()
    assert np.max(np.abs(a["logits"] - b["logits"])) < 1e-10 and np.max(np.abs(a["hidden"] - b["hidden"])) < 1e-10


def test_head_transform_against_library_layers_and_special_cases(small):
    sh, w, kept, p = small
    rng = np.random.default_rng(55)
    h = rng.standard_normal(sh.d_model) * 2.0
    t = O.head_transform(p, h)
    ht = torch.tensor(h, dtype=torch.float64)
    lin = torch.nn.functional.linear(ht, torch.tensor(p.head_w), torch.tensor(p.head_b))
    ref = torch.nn.functional.layer_norm(torch.nn.functional.gelu(lin), (sh.d_model,), torch.tensor(p.head_ln_g),
                                         torch.tensor(p.head_ln_b), eps=sh.ln_eps).numpy()
    assert np.max(np.abs(t - ref)) < 1e-12
    # zero matrix: the output no longer depends on h
    z = dict(w); z["head_w"] = np.zeros_like(w["head_w"])
    pz = O.Params(z, sh.n_heads, sh.ln_eps)
    assert np.max(np.abs(O.head_transform(pz, h) - O.head_transform(pz, -3.0 * h))) == 0.0
    # no head: identity
    n = {k: v for k, v in w.items() if not k.startswith("head_")}
    assert np.array_equal(O.head_transform(O.Params(n, sh.n_heads, sh.ln_eps), h), h)
    # order of the three steps matters and is gelu -> LayerNorm: the result has LayerNorm statistics
    g, b = p.head_ln_g, p.head_ln_b
    u = (t - b) / g
    assert abs(u.mean()) < 1e-12 and abs(u.var() - 1.0) < 1e-3


def test_output_bias_is_added_per_full_vocabulary_row(small):
    sh, w, kept, p = small
    rng = np.random.default_rng(56)
    h = rng.standard_normal(sh.d_model)
    nb = {k: v for k, v in w.items() if k != "out_bias"}
    q = O.Params(nb, sh.n_heads, sh.ln_eps)
    diff = O.logits_kept(p, h, kept) - O.logits_kept(q, h, kept)
    assert np.max(np.abs(diff - w["out_bias"].astype(np.float64)[kept])) < 1e-12
    # a dominant bias on one kept row decides every emitted token
    big = dict(w); ob = w["out_bias"].astype(np.float64).copy(); ob[kept[7]] = 1e4; big["out_bias"] = ob
    g = O.generate_cached(O.Params(big, sh.n_heads, sh.ln_eps), kept[:3], 4, kept)
    assert g["tokens"].tolist() == [7, 7, 7, 7]


def test_planted_mistakes_in_the_variants_are_caught(small, monkeypatch):
    sh, w, kept, p = small
    wl = BF.to_lists(w)
    rng = np.random.default_rng(57)
    prompt = kept[rng.integers(0, len(kept), size=4)]
    _, logits_b = BF.generate(wl, sh.n_heads, sh.ln_eps, prompt.tolist(), 3, kept.tolist())
    right = np.array(logits_b)

    def wrong(**patches):
        with monkeypatch.context() as m:
            for name, fn in patches.items():
                m.setattr(O, name, fn)
            return O.generate_full_recompute(p, prompt, 3, kept)["logits"]

    assert np.max(np.abs(O.generate_full_recompute(p, prompt, 3, kept)["logits"] - right)) < 1e-11
    ln, ge = O.layer_norm, O.gelu
    # LayerNorm before GELU
    bad = wrong(head_transform=lambda p_, h: ge(ln(p_.head_w @ h + p_.head_b, p_.head_ln_g, p_.head_ln_b, p_.eps)))
    assert np.max(np.abs(bad - right)) > 1e-3
    # transposed head matrix
    bad = wrong(head_transform=lambda p_, h: ln(ge(p_.head_w.T @ h + p_.head_b), p_.head_ln_g, p_.head_ln_b, p_.eps))
    assert np.max(np.abs(bad - right)) > 1e-3
    # bias indexed by trimmed instead of full id
    bad = wrong(logits_kept=lambda p_, h, k_: (p_.tok_emb @ O.head_transform(p_, h))[k_] + p_.out_bias[:len(k_)])
    assert np.max(np.abs(bad - right)) > 1e-3

    # segment rows swapped (generated positions take row 0)
    def embed_swapped(p_, ids_full, first_pos=0, L=None):
        pos = np.arange(first_pos, first_pos + len(ids_full))
        y = p_.tok_emb[ids_full] + p_.pos_emb[pos] + p_.type_emb[(pos < L).astype(np.int64)]
        return ln(y, p_.emb_ln_g, p_.emb_ln_b, p_.eps)
    bad = wrong(embed=embed_swapped)
    assert np.max(np.abs(bad - right)) > 1e-3
