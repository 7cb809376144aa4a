"""Pins for oracle/schedule_oracle.py and the end-of-sequence rule of the generators."""
import itertools

import numpy as np
import pytest

from oracle import ernie_oracle as O
from oracle import schedule_oracle as S
from synth import make_workload


def test_hand_worked_example():
    # lengths            idx: 0  1  2  3  4  5  6
    lens = [5, 2, 9, 2, 7, 3, 9]
    order, starts = S.plan_batches(lens, max_batch=3, max_tokens=16)
    # stable ascending: 1(2) 3(2) 5(3) 0(5) 4(7) 2(9) 6(9)
    assert order.tolist() == [1, 3, 5, 0, 4, 2, 6]
    # [2,2,3] -> 3 rows x 3 = 9 <= 16, full at 3 rows; [5,7]: 2 x 7 = 14, adding 9 would make 27; [9]; [9] (2 x 9 = 18 > 16)
    assert starts.tolist() == [0, 3, 5, 6, 7]
    assert S.padded_tokens(lens, order, starts) == 9 + 14 + 9 + 9


@pytest.mark.parametrize("seed", range(6))
def test_invariants_on_random_lengths(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 200))
    lens = rng.integers(1, 257, size=n)
    mb, mt = int(rng.integers(1, 65)), int(rng.integers(256, 4096))
    order, starts = S.plan_batches(lens, mb, mt)
    assert sorted(order.tolist()) == list(range(n))                         # a permutation
    sl = lens[order]
    assert np.all(np.diff(sl) >= 0)                                         # ascending
    for a, b in zip(np.nonzero(np.diff(sl) == 0)[0], np.nonzero(np.diff(sl) == 0)[0] + 1):
        assert order[a] < order[b]                                          # equal lengths keep their order
    assert starts[0] == 0 and starts[-1] == n and np.all(np.diff(starts) > 0)
    for i, (a, b) in enumerate(zip(starts[:-1], starts[1:])):
        rows, longest = b - a, int(sl[b - 1])
        assert rows <= mb and rows * longest <= mt                          # within both limits
        if b < n:                                                           # greedy: the next row did not fit
            assert rows + 1 > mb or (rows + 1) * int(sl[b]) > mt


def test_sorted_batches_never_pad_more_than_arrival_order_batches():
    rng = np.random.default_rng(9)
    lens = rng.integers(16, 257, size=512)
    order, starts = S.plan_batches(lens, 64, 10 ** 9)                        # token limit off: fixed batches of 64
    assert np.all(np.diff(starts) == 64)
    arrival = np.arange(512, dtype=np.int32)
    assert S.padded_tokens(lens, order, starts) <= S.padded_tokens(lens, arrival, starts)
    # and it is the minimum over contiguous cuts of any ordering for two batches of two (brute force over orders)
    small = [7, 1, 5, 2]
    best = min(S.padded_tokens(small, list(perm), [0, 2, 4]) for perm in itertools.permutations(range(4)))
    o, s = S.plan_batches(small, 2, 10 ** 9)
    assert S.padded_tokens(small, o, s) == best


def test_token_limit_gives_short_prompts_larger_batches():
    lens = [10] * 40 + [100] * 40
    order, starts = S.plan_batches(lens, max_batch=32, max_tokens=800)
    sizes = np.diff(starts).tolist()
    assert sizes[0] == 32 and max(sizes[2:]) == 8                            # 32 x 10 <= 800; 8 x 100 = 800


def test_bad_arguments():
    for args in [([3, 0], 4, 10), ([3], 0, 10), ([3], 4, 0), ([11], 4, 10)]:
        with pytest.raises(ValueError):
            S.plan_batches(*args)
    o, s = S.plan_batches([], 4, 10)
    assert o.size == 0 and s.tolist() == [0]


# ---------------------------------------------------------------- end of sequence

@pytest.fixture(scope="module")
def tiny():
    wl = make_workload("tiny_affine")
    return wl, O.Params(wl.weights, wl.shape.n_heads, wl.shape.ln_eps)


def test_eos_stops_the_sequence_where_it_is_emitted(tiny):
    wl, p = tiny
    prompt = wl.batches_full[0][0]
    free = O.generate_cached(p, prompt, 8, wl.kept_ids)
    eos = int(free["tokens"][3])
    first = int(np.nonzero(free["tokens"] == eos)[0][0])
    for fn in (O.generate_cached, O.generate_full_recompute):
        g = fn(p, prompt, 8, wl.kept_ids, eos=eos)
        assert g["tokens"][:first + 1].tolist() == free["tokens"][:first + 1].tolist()      # identical up to and including it
        assert np.all(g["tokens"][first:] == eos)
        assert np.allclose(g["logits"][:first + 1], free["logits"][:first + 1], atol=1e-10)
        assert np.isnan(g["logits"][first + 1:]).all() and np.isnan(g["hidden"][first + 1:]).all()
    assert O.generate_cached(p, prompt, 8, wl.kept_ids, eos=eos)["steps"] == first + 1   # prefill + `first` decode steps
    # an id that never appears changes nothing
    never = int(np.setdiff1d(np.arange(len(wl.kept_ids)), free["tokens"])[0])
    g = O.generate_cached(p, prompt, 8, wl.kept_ids, eos=never)
    assert g["tokens"].tolist() == free["tokens"].tolist() and g["steps"] == 8


def test_eos_under_teacher_forcing_follows_the_fed_token(tiny):
    wl, p = tiny
    prompt = wl.batches_full[0][1]
    eos = 17
    forced = np.array([5, 9, eos, 3, 4, 6, 7, 8])
    g = O.generate_cached(p, prompt, 8, wl.kept_ids, forced_tokens=forced, eos=eos)
    ref = O.generate_cached(p, prompt, 8, wl.kept_ids, forced_tokens=forced)
    assert np.allclose(g["logits"][:3], ref["logits"][:3], atol=1e-12)       # steps fed 5, 9 ran; feeding eos ends it
    assert np.isnan(g["logits"][3:]).all() and np.all(g["tokens"][3:] == eos) and g["steps"] == 3


# ---------------------------------------------------------------- whole job

def test_job_is_per_request_preprocess_generate_postprocess(tiny):
    from oracle import job_oracle as J
    from oracle import prune_oracle as P
    wl, p = tiny
    kept = wl.kept_ids
    V = wl.shape.vocab_full
    unk = int(kept[3])
    fmap = P.full_to_trimmed_map(kept, V, unk)
    rng = np.random.default_rng(4)
    prompts = [rng.integers(0, V, size=n).astype(np.int32) for n in (3, 11, 6)]       # contain dropped ids
    assert any(np.setdiff1d(q, kept).size for q in prompts)
    toks, gaps = J.run_job(p, prompts, fmap, kept, 5)
    assert toks.shape == (3, 5) and toks.dtype == np.int32 and np.all(gaps > 0)
    assert np.all(np.isin(toks, kept))                                                # full ids of kept rows only
    for r, q in enumerate(prompts):
        seen = np.where(np.isin(q, kept), q, unk)                                     # dropped ids -> unknown-word id
        g = O.generate_full_recompute(p, seen, 5, kept)                               # the definition, not the cached path
        assert toks[r].tolist() == kept[g["tokens"]].tolist()
    # request order is the caller's order whatever the lengths
    toks2, _ = J.run_job(p, prompts[::-1], fmap, kept, 5)
    assert np.array_equal(toks2, toks[::-1])
