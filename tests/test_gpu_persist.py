"""The one-launch decode step (all layers of a small-batch step in one persistent kernel with tagged hand-overs):
agreement with the five-kernels-per-layer step, and the bounded waits: a hand-over that never arrives makes every
workgroup give up and leave, the failure is reported, and the handle keeps working afterwards."""
from dataclasses import replace

import numpy as np
import pytest

from oracle import prune_oracle as P
from synth import CONFIGS, make_workload, Workload, make_weights, make_kept_ids, full_to_trimmed

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def E():
    import torch
    import paper_2407_04991_amd as E
    assert torch.cuda.is_available(), "GPU tests need a GPU: there is no CPU fallback"
    E.load_library()
    return E


def _workload(lengths, name="tiny_affine", **kw):
    sh = replace(CONFIGS[name], batch=len(lengths), prompt_len=max(lengths), **kw)
    kept = make_kept_ids(sh)
    rng = np.random.default_rng(31337)
    seqs = [kept[rng.integers(0, len(kept), size=n)].astype(np.int32) for n in lengths]
    wl = Workload(sh, make_weights(sh), kept)
    wl.batches_full.append(seqs)
    wl.batches_trimmed.append([full_to_trimmed(s, kept) for s in seqs])
    return wl


def _run(eng, ids, lens, feeds):
    import torch
    eng.prefill(torch.as_tensor(ids), lens)
    out = []
    for feed in feeds:
        tok, lo, ho = eng.decode_step(torch.as_tensor(feed), logits=True, hidden=True)
        out.append((tok.cpu().numpy(), lo.cpu().numpy(), ho.cpu().numpy()))
    return out


@pytest.mark.parametrize("shape", [dict(lengths=[3, 40, 17, 9, 25], n_layers=3),                         # one row group
                                   dict(lengths=[5 + (11 * i) % 37 for i in range(33)], n_layers=2),   # two rows per wave
                                   dict(lengths=[2 + (5 * i) % 29 for i in range(64)], n_layers=1, d_model=320, n_heads=5,
                                        d_ffn=1152)])
def test_one_launch_step_agrees_with_the_kernel_per_phase_step(E, shape):
    """Same inputs through both small-batch decode paths.  They differ in rounding points only (the one-launch
    kernel keeps the pre-LayerNorm sums in fp16, as the prefill does), so logits agree far inside the oracle tolerance."""
    lengths = shape.pop("lengths")
    wl = _workload(lengths, max_pos=64, n_gen=4, **shape)
    B, V = wl.shape.batch, wl.shape.vocab_kept
    ids, lens = wl.padded(0)
    rng = np.random.default_rng(5)
    feeds = [rng.integers(0, V, size=B).astype(np.int32) for _ in range(3)]
    eng = E.engine_from_workload(wl, max_seq=wl.shape.prompt_len + 8)
    print(f"[persist] B={B} layers={wl.shape.n_layers} d={wl.shape.d_model}", flush=True)
    one = _run(eng, ids, lens, feeds)
    eng.tune("persist", 0)
    five = _run(eng, ids, lens, feeds)
    eng.tune("persist", 1)
    eng.tune("persist_helpers", 0)        # without the workgroups that only warm the L2: identical results
    bare = _run(eng, ids, lens, feeds)
    eng.close()
    for (t1, l1, h1), (t5, l5, h5), (tb, lb, hb) in zip(one, five, bare):
        assert np.max(np.abs(l1 - l5)) < 1e-2 and np.max(np.abs(h1 - h5)) < 1e-2
        assert np.array_equal(l1, lb) and np.array_equal(h1, hb) and np.array_equal(t1, tb)
        assert np.array_equal(t1, np.argmax(l1, axis=1))


@pytest.mark.parametrize("phase", [1, 2, 3, 4, 5])
def test_a_hand_over_that_never_arrives_ends_the_kernel_and_is_reported(E, phase):
    """The output of one phase of layer 0 is withheld (test hook) with a small poll limit: every consumer gives up,
    the kernel ends by itself, the next call reports ERNIE_EHIP once, and the handle works again afterwards."""
    import torch
    wl = _workload([7, 19, 4, 30, 11, 2], max_pos=64, n_gen=4, n_layers=2)
    B, V = wl.shape.batch, wl.shape.vocab_kept
    ids, lens = wl.padded(0)
    feeds = [np.full(B, 3, dtype=np.int32), np.full(B, 5, dtype=np.int32)]
    eng = E.engine_from_workload(wl, max_seq=wl.shape.prompt_len + 8)
    good = _run(eng, ids, lens, feeds)
    eng.tune("persist_spin", 200)
    eng.tune("persist_stall", phase)
    print(f"[persist] withholding phase {phase}", flush=True)
    eng.prefill(torch.as_tensor(ids), lens)
    tok = torch.empty(B, dtype=torch.int32, device="cuda:0")
    assert E.ernie_decode_step(eng.handle, torch.as_tensor(feeds[0]).cuda(), None, None, tok) == E.ERNIE_OK   # enqueued
    torch.cuda.synchronize()                                             # the kernel has ended by itself
    assert E.ernie_decode_step(eng.handle, None, None, None, tok) == E.ERNIE_EHIP      # reported once ...
    assert E.ernie_last_error(eng.handle) == E.ERNIE_OK                                # ... and cleared
    eng.tune("persist_stall", 0)
    eng.tune("persist_spin", 1 << 17)
    again = _run(eng, ids, lens, feeds)
    eng.close()
    for (t0, l0, h0), (t1, l1, h1) in zip(good, again):
        assert np.array_equal(t0, t1) and np.array_equal(l0, l1) and np.array_equal(h0, h1)


@pytest.mark.parametrize("overlap", [False, True])
def test_a_failing_batch_ends_the_job_runner(E, overlap):
    """ernie_run_job with a decode kernel that gives up in every batch: the call returns ERNIE_EHIP (it must not
    hang with its stages side by side either), and the handle runs a clean job afterwards."""
    import torch
    wl = make_workload("tiny_affine")
    sh = wl.shape
    kept = wl.kept_ids
    fmap = P.full_to_trimmed_map(kept, sh.vocab_full, int(kept[0]))
    rng = np.random.default_rng(12)
    prompts = [rng.integers(0, sh.vocab_full, size=int(L)).astype(np.int32) for L in rng.integers(1, 20, size=21)]
    eng = E.engine_from_workload(wl, max_batch=4, max_seq=32)
    ws = torch.empty(E.ernie_job_workspace_bytes(eng.handle, 5), dtype=torch.uint8, device="cuda:0")
    rc, ref, _ = E.ernie_run_job(eng.handle, prompts, fmap, kept, 5, 4, 64, overlap, ws)
    assert rc == E.ERNIE_OK
    eng.tune("persist_spin", 200)
    eng.tune("persist_stall", 4)
    print(f"[persist] failing job, overlap={overlap}", flush=True)
    rc, _, _ = E.ernie_run_job(eng.handle, prompts, fmap, kept, 5, 4, 64, overlap, ws)
    assert rc == E.ERNIE_EHIP
    eng.tune("persist_stall", 0)
    eng.tune("persist_spin", 1 << 17)
    torch.cuda.synchronize()
    E.ernie_last_error(eng.handle)                 # whatever the abandoned batches left behind
    rc, out, _ = E.ernie_run_job(eng.handle, prompts, fmap, kept, 5, 4, 64, overlap, ws)
    assert rc == E.ERNIE_OK and np.array_equal(out, ref)
    eng.close()
