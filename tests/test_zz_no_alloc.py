"""ernie_decode_step_static (the decode step whose temporaries live in static device memory) against
ernie_decode_step, through the C ABI: two calls in a row on one GPU, the second with a smaller batch."""
from dataclasses import replace

import numpy as np
import pytest

from synth import CONFIGS, make_workload, Workload, make_weights, make_kept_ids, full_to_trimmed

pytestmark = pytest.mark.gpu


def _workload(lengths, **kw):
    sh = replace(CONFIGS["tiny_head"], batch=len(lengths), prompt_len=max(lengths), **kw)
    kept = make_kept_ids(sh)
    rng = np.random.default_rng(4242)
    seqs = [kept[rng.integers(0, len(kept), size=n)].astype(np.int32) for n in lengths]
    wl = Workload(sh, make_weights(sh), kept)
    wl.batches_full.append(seqs)
    wl.batches_trimmed.append([full_to_trimmed(s, kept) for s in seqs])
    return wl


def _steps(eng, ids, lens, feeds, static):
    """prefill, then one decode step per entry of `feeds` (teacher-forced ids); returns per-step (tokens, logits, hidden)."""
    import torch
    eng.prefill(torch.as_tensor(ids), lens)
    out = []
    for feed in feeds:
        tok, lo, ho = eng.decode_step(torch.as_tensor(feed), logits=True, hidden=True, static=static)
        out.append((tok.cpu().numpy(), lo.cpu().numpy(), ho.cpu().numpy()))
    return out


def test_static_scratch_decode_step_matches_the_arena_one():
    import torch
    import paper_2407_04991_amd as E
    assert torch.cuda.is_available(), "GPU tests need a GPU: there is no CPU fallback"
    # first call: 40 rows (two row tiles of the decode GEMMs, the model variants on); second call: 3 rows
    big = _workload([5 + (7 * i) % 23 for i in range(40)], max_pos=64, n_gen=4)
    small = _workload([9, 2, 30], max_pos=64, n_gen=4)
    rng = np.random.default_rng(99)
    for wl in (big, small):
        B, V = wl.shape.batch, wl.shape.vocab_kept
        print(f"[no-alloc] batch {B}", flush=True)
        ids, lens = wl.padded(0)
        feeds = [rng.integers(0, V, size=B).astype(np.int32) for _ in range(3)]
        ref_eng = E.engine_from_workload(wl, max_seq=wl.shape.prompt_len + 8)
        ref_eng.tune("persist", 0)      # the five-kernels-per-layer decode step, which is what the static variant runs
        ref = _steps(ref_eng, ids, lens, feeds, static=False)
        ref_eng.close()
        eng = E.engine_from_workload(wl, max_seq=wl.shape.prompt_len + 8)
        got = _steps(eng, ids, lens, feeds, static=True)
        eng.close()
        for t, ((rt, rl, rh), (gt, gl, gh)) in enumerate(zip(ref, got)):
            # same kernels on the same inputs, only the addresses of the temporaries differ: bit-identical
            assert np.array_equal(rt, gt), f"tokens differ at step {t}"
            assert np.array_equal(rl, gl), f"logits differ at step {t}"
            assert np.array_equal(rh, gh), f"hidden states differ at step {t}"
            assert np.all(np.isfinite(gl))


def test_static_scratch_decode_step_refuses_what_does_not_fit():
    import torch
    import paper_2407_04991_amd as E
    wl = _workload([4] * 65, max_pos=16, n_gen=2)          # 65 rows: beyond the static array's batch limit
    eng = E.engine_from_workload(wl, max_seq=8)
    ids, lens = wl.padded(0)
    eng.prefill(torch.as_tensor(ids), lens)
    tok = torch.empty(65, dtype=torch.int32, device="cuda:0")
    assert E.ernie_decode_step_static(eng.handle, None, None, None, tok) == E.ERNIE_ECAPACITY
    assert E.ernie_decode_step(eng.handle, None, None, None, tok) == E.ERNIE_OK      # the arena-backed step still runs
    torch.cuda.synchronize()
    eng.close()
