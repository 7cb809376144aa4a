"""Shared helpers of the GPU parity tests: run the oracle, run the HIP path teacher-forced,
compare under the stated tolerances.  The oracle side never sees a GPU value."""
from __future__ import annotations

import numpy as np

from oracle import ernie_oracle as O

# Acceptance bar (stated with the benchmark definition): with teacher-forced oracle tokens,
# final hidden states and logits within max-abs 3e-2 and relative-L2 1e-2 at every step;
# argmax ids bit-exact wherever the oracle's top-2 logit gap exceeds 0.05.
MAX_ABS = 3e-2
REL_L2 = 1e-2
GAP = 0.05


def oracle_generate(wl, batch: int, rows, n_gen: int, definition: bool = False):
    """Oracle results for the chosen rows of one batch: dict row -> {tokens, hidden, logits}."""
    p = O.Params(wl.weights, wl.shape.n_heads, wl.shape.ln_eps)
    out = {}
    for r in rows:
        prompt = wl.batches_full[batch][r]
        fn = O.generate_full_recompute if definition else O.generate_cached
        out[r] = fn(p, prompt, n_gen, wl.kept_ids)
    return out


def gpu_generate(engine, ids, lens, n_gen: int, forced: dict | None = None, want=True):
    """Run prefill + n_gen-1 decode steps through the C ABI.

    forced: dict row -> [n_gen] oracle tokens to feed for that row (teacher forcing); all other rows
    feed their own previous argmax.  Returns tokens [n_gen, B], hidden [n_gen, B, d], logits [n_gen, B, V'].
    """
    import torch
    tok, lo, ho = engine.prefill(torch.as_tensor(ids), lens, logits=want, hidden=want)
    toks, hid, lg = [tok.cpu().numpy()], [ho.cpu().numpy()], [lo.cpu().numpy()]
    for t in range(1, n_gen):
        feed = tok.clone()
        if forced:
            for r, ft in forced.items():
                feed[r] = int(ft[t - 1])
        tok, lo, ho = engine.decode_step(feed, logits=want, hidden=want)
        toks.append(tok.cpu().numpy()); hid.append(ho.cpu().numpy()); lg.append(lo.cpu().numpy())
    return np.array(toks), np.array(hid), np.array(lg)


def rel_l2(a, ref):
    return float(np.linalg.norm(a - ref) / np.linalg.norm(ref))


def check_rows(orc: dict, toks, hid, lg, label=""):
    """Element-by-element comparison of the HIP outputs with the oracle for the rows in `orc`."""
    stats = {"max_abs_hidden": 0.0, "max_abs_logits": 0.0, "rel_hidden": 0.0, "rel_logits": 0.0,
             "exact_required": 0, "exact_matched": 0, "total": 0}
    for r, o in orc.items():
        n_gen = len(o["tokens"])
        for t in range(n_gen):
            dh = float(np.max(np.abs(hid[t, r] - o["hidden"][t])))
            dl = float(np.max(np.abs(lg[t, r] - o["logits"][t])))
            rh, rl = rel_l2(hid[t, r], o["hidden"][t]), rel_l2(lg[t, r], o["logits"][t])
            stats["max_abs_hidden"] = max(stats["max_abs_hidden"], dh)
            stats["max_abs_logits"] = max(stats["max_abs_logits"], dl)
            stats["rel_hidden"] = max(stats["rel_hidden"], rh)
            stats["rel_logits"] = max(stats["rel_logits"], rl)
            assert dh <= MAX_ABS and rh <= REL_L2, f"{label} hidden row {r} step {t}: max-abs {dh:.3e} rel-L2 {rh:.3e}"
            assert dl <= MAX_ABS and rl <= REL_L2, f"{label} logits row {r} step {t}: max-abs {dl:.3e} rel-L2 {rl:.3e}"
            stats["total"] += 1
            z = o["logits"][t]
            if O.top2_gap(z) > GAP:
                stats["exact_required"] += 1
                assert int(toks[t, r]) == int(o["tokens"][t]), \
                    f"{label} token row {r} step {t}: gpu {int(toks[t, r])} oracle {int(o['tokens'][t])}"
                stats["exact_matched"] += 1
            else:
                # several answers are acceptable: the GPU's choice must be one of the oracle's near-maximal entries
                assert z[int(toks[t, r])] >= z.max() - GAP - 2 * MAX_ABS
            # the emitted id is the argmax of the GPU's own logits, lowest index on ties
            assert int(toks[t, r]) == int(np.argmax(lg[t, r]))
    return stats
