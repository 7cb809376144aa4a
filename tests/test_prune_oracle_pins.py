"""Pins for oracle/prune_oracle.py (Method, "Embedding layer pruning"): brute force with scalar loops,
ordering invariants, the closed-form coverage of a Zipf law, round trips, planted mistakes."""
import numpy as np
import pytest

from oracle import prune_oracle as P
from synth import make_corpus


def _count_loop(ids, vocab):
    c = [0] * vocab
    for t in ids:
        t = int(t)
        if 0 <= t < vocab:
            c[t] += 1
    return c


def _select_loop(counts, k, reserved):
    """Repeatedly pick the best remaining id: reserved first, then larger count, then smaller id."""
    left = set(range(len(counts)))
    out = []
    for _ in range(k):
        best = None
        for i in left:
            if best is None:
                best = i
                continue
            a = (i in reserved, counts[i], -i)
            b = (best in reserved, counts[best], -best)
            if a > b:
                best = i
        out.append(best)
        left.remove(best)
    return sorted(out)


def test_counts_match_a_scalar_loop_and_ignore_out_of_range_ids():
    ids = make_corpus(97, 5000, seed=1, noise_ids=200)
    assert (ids < 0).any() and (ids >= 97).any()
    got = P.count_tokens(ids, 97)
    assert got.dtype == np.uint64
    assert got.tolist() == _count_loop(ids, 97)
    assert int(got.sum()) == 5000 - 200


def test_counts_accumulate_over_calls():
    ids = make_corpus(50, 3000, seed=2)
    whole = P.count_tokens(ids, 50)
    part = P.count_tokens(ids[:1234], 50)
    part = P.count_tokens(ids[1234:], 50, part)
    assert np.array_equal(whole, part)


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_selection_matches_greedy_brute_force_with_many_ties(seed):
    rng = np.random.default_rng(seed)
    vocab, k = 60, 17
    counts = rng.integers(0, 6, size=vocab)          # few distinct values: ties everywhere
    reserved = [int(x) for x in rng.choice(vocab, size=3, replace=False)]
    got = P.select_kept(counts, k, reserved)
    assert got.dtype == np.int32
    assert got.tolist() == _select_loop(counts.tolist(), k, set(reserved))


def test_selection_invariants():
    vocab, k = 2000, 300
    counts = P.count_tokens(make_corpus(vocab, 200000, seed=5), vocab)
    reserved = [7, 1999]
    kept = P.select_kept(counts, k, reserved)
    assert len(kept) == k and np.all(np.diff(kept) > 0)          # ascending, unique
    assert set(reserved) <= set(kept.tolist())
    dropped = np.setdiff1d(np.arange(vocab), kept)
    free = np.setdiff1d(kept, reserved)
    assert counts[dropped].max() <= counts[free].min()
    # boundary ties: among ids with the boundary count, the kept ones are the lowest ids
    edge = counts[free].min()
    tie_kept = [i for i in free if counts[i] == edge]
    tie_drop = [i for i in dropped if counts[i] == edge]
    if tie_kept and tie_drop:
        assert max(tie_kept) < min(tie_drop)


def test_all_equal_counts_keep_the_lowest_ids_and_k_equal_vocab_keeps_everything():
    assert P.select_kept(np.full(10, 4), 3).tolist() == [0, 1, 2]
    assert P.select_kept(np.full(10, 4), 3, reserved=[9]).tolist() == [0, 1, 9]
    assert P.select_kept(np.arange(10), 10).tolist() == list(range(10))
    assert P.select_kept(np.arange(10), 2).tolist() == [8, 9]       # larger count wins


def test_bad_arguments_raise():
    c = np.ones(10)
    for k, res in [(0, ()), (11, ()), (2, (1, 1)), (1, (1, 2)), (3, (10,)), (3, (-1,))]:
        with pytest.raises(ValueError):
            P.select_kept(c, k, res)
    with pytest.raises(ValueError):
        P.full_to_trimmed_map(np.array([1, 2, 3]), 10, unk_full_id=5)    # unknown-word row not kept


def test_zipf_expected_counts_keep_the_top_ranks_and_cover_the_closed_form_share():
    """With counts proportional to r^-1.1 the k most frequent ids are ranks 1..k and the kept share of the
    corpus is the ratio of two partial sums of the law: 93.6 % for 6000 of 18000, 95.4 % for 8000."""
    V = 18000
    w = np.arange(1, V + 1, dtype=np.float64) ** -1.1
    counts = np.round(w / w.sum() * 1e12).astype(np.uint64)
    for k, share in [(6000, 0.936), (8000, 0.954)]:
        kept = P.select_kept(counts, k)
        assert np.array_equal(kept, np.arange(k))
        # partial sums written as an explicit loop over ranks
        num = sum(r ** -1.1 for r in range(1, k + 1))
        den = sum(r ** -1.1 for r in range(1, V + 1))
        assert abs(P.coverage(counts, kept) - num / den) < 1e-9
        assert abs(num / den - share) < 5e-4


def test_sampled_zipf_corpus_recovers_the_frequent_ranks_wherever_they_sit():
    V, k = 3000, 200
    ids = make_corpus(V, 2_000_000, seed=11, shuffle_ranks=True)
    rng = np.random.default_rng(np.random.PCG64(11))
    rng.random(2_000_000)
    perm = rng.permutation(V)                       # same draw order as the generator
    kept = P.select_kept(P.count_tokens(ids, V), k)
    top = set(perm[:k // 2].tolist())               # the 100 most frequent ranks are far from the boundary
    assert top <= set(kept.tolist())


def test_maps_round_trip_and_unknown_routing():
    vocab = 500
    counts = P.count_tokens(make_corpus(vocab, 50000, seed=3), vocab)
    unk = 123
    kept = P.select_kept(counts, 64, reserved=[unk])
    m = P.full_to_trimmed_map(kept, vocab, unk)
    assert m.dtype == np.int32 and m.shape == (vocab,)
    assert np.array_equal(m[kept], np.arange(64))                       # kept ids: their rank in kept_ids
    unk_t = int(np.searchsorted(kept, unk))
    dropped = np.setdiff1d(np.arange(vocab), kept)
    assert np.all(m[dropped] == unk_t)
    # trimmed -> full -> trimmed is the identity; full -> trimmed -> full fixes kept ids and sends the rest to unk
    t = np.arange(64, dtype=np.int32)
    assert np.array_equal(P.remap(P.remap(t, kept, -1), m, unk_t), t)
    f = np.arange(vocab, dtype=np.int32)
    back = P.remap(P.remap(f, m, unk_t), kept, -1)
    assert np.array_equal(back[kept], kept) and np.all(back[dropped] == unk)
    # out-of-table values take the fallback, shape is preserved
    x = np.array([[0, -1], [vocab, 5]], dtype=np.int32)
    y = P.remap(x, m, unk_t)
    assert y.shape == x.shape and y[0, 1] == unk_t and y[1, 0] == unk_t and y[0, 0] == m[0] and y[1, 1] == m[5]


def test_input_generator_reindexes_by_the_same_rule():
    """synth.full_to_trimmed prepares the prompts of both sides of the generation parity tests: it must route
    dropped ids to the unknown-word row exactly like the oracle's map (default: the lowest kept id is that word)."""
    from synth.ernie_inputs import full_to_trimmed
    vocab = 400
    counts = P.count_tokens(make_corpus(vocab, 30000, seed=5), vocab)
    ids = np.arange(vocab, dtype=np.int32)
    for unk in (0, 57):
        kept = P.select_kept(counts, 48, reserved=[unk])
        m = P.full_to_trimmed_map(kept, vocab, unk)
        assert np.array_equal(full_to_trimmed(ids, kept, unk_full_id=unk), m)
    kept = P.select_kept(counts, 48, reserved=[0])
    assert np.array_equal(full_to_trimmed(ids, kept), P.full_to_trimmed_map(kept, vocab, int(kept[0])))
    with pytest.raises(ValueError):
        full_to_trimmed(ids, np.array([1, 2, 3]), unk_full_id=5)


def test_trim_rows_is_bitwise_row_selection():
    rng = np.random.default_rng(0)
    tab = rng.standard_normal((40, 16)).astype(np.float16)
    kept = np.array([0, 3, 4, 39], dtype=np.int32)
    out = P.trim_rows(tab, kept)
    assert out.flags["C_CONTIGUOUS"] and out.dtype == np.float16
    for i, r in enumerate(kept):
        assert out[i].tobytes() == tab[r].tobytes()


def test_trimmed_projection_equals_selected_rows_of_the_full_projection():
    """Why trimming is exact for the kept rows: h . E'[i] = (h . E^T)[kept_ids[i]]."""
    rng = np.random.default_rng(1)
    E = rng.standard_normal((50, 8))
    h = rng.standard_normal(8)
    kept = np.array([2, 5, 7, 30, 49])
    full = np.array([sum(h[j] * E[r, j] for j in range(8)) for r in range(50)])
    trimmed = P.trim_rows(E, kept) @ h
    assert np.allclose(trimmed, full[kept], rtol=0, atol=1e-12)


def test_planted_mistakes_are_caught():
    """Each plausible slip changes the answer on the tie-heavy case used above."""
    rng = np.random.default_rng(0)
    vocab, k = 60, 17
    counts = rng.integers(0, 6, size=vocab)
    reserved = [4, 50]
    right = P.select_kept(counts, k, reserved).tolist()
    ids = np.arange(vocab)
    forced = np.zeros(vocab, dtype=bool); forced[reserved] = True
    wrong_variants = {
        "ascending counts": np.lexsort((ids, counts, ~forced)),
        "ties by higher id": np.lexsort((-ids, -counts, ~forced)),
        "reserved ignored": np.lexsort((ids, -counts)),
        "reserved last": np.lexsort((ids, -counts, forced)),
    }
    for name, order in wrong_variants.items():
        assert sorted(order[:k].tolist()) != right, name
