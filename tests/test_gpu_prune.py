"""Bit-exact parity of the vocabulary-trimming kernels with oracle/prune_oracle.py, through the C ABI."""
from dataclasses import replace

import numpy as np
import pytest

from oracle import prune_oracle as P
from synth import CONFIGS, make_corpus, make_weights, Workload
from tests.parity_util import oracle_generate, gpu_generate, check_rows

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def E():
    import torch
    import paper_2407_04991_amd as E
    assert torch.cuda.is_available(), "GPU tests need a GPU: there is no CPU fallback"
    E.load_library()
    return E


def _say(msg):
    print(msg, flush=True)


def _dev(a):
    import torch
    return torch.as_tensor(np.ascontiguousarray(a)).to("cuda:0")


def _counts(tr):
    return tr.counts.cpu().numpy().view(np.uint64)


@pytest.mark.parametrize("vocab,n", [(18000, 3_000_017), (50000, 400_003), (97, 70_001), (1, 1000)])
def test_counts_are_exact_on_ragged_unaligned_pieces(E, vocab, n):
    """Zipf stream with out-of-range ids mixed in, fed in three pieces whose starts are 4-, 8- and 16-byte aligned;
    vocab 50000 takes the path without an LDS histogram."""
    ids = make_corpus(vocab, n, seed=21, noise_ids=n // 50)
    want = P.count_tokens(ids, vocab)
    d = _dev(ids)
    tr = E.VocabTrimmer(vocab)
    cuts = [0, 1 + (n // 3 // 4) * 4, 2 + (2 * n // 3 // 4) * 4, n]
    _say(f"[prune] count vocab {vocab} n {n} cuts {cuts}")
    for a, b in zip(cuts[:-1], cuts[1:]):
        tr.count(d[a:b])
    assert np.array_equal(_counts(tr), want)


@pytest.mark.parametrize("n", [0, 1, 3, 4, 5, 7, 8, 9, 2051])
def test_counts_of_tiny_streams(E, n):
    ids = make_corpus(300, max(n, 1), seed=n)[:n]
    tr = E.VocabTrimmer(300)
    import torch
    buf = _dev(np.concatenate([[7, 7, 7], ids, [7, 7, 7]]).astype(np.int32))     # neighbours must not be counted
    for off in (3,):
        tr.count(buf[off:off + n]) if n else E.ernie_vocab_count(None, 0, 300, tr.counts)
    torch.cuda.synchronize()
    assert np.array_equal(_counts(tr), P.count_tokens(ids, 300))


def _select_case(E, counts, k, reserved, unk):
    vocab = len(counts)
    tr = E.VocabTrimmer(vocab)
    tr.counts.copy_(_dev(np.asarray(counts).astype(np.uint64).view(np.int64)))
    kept = tr.select(k, reserved, unk).cpu().numpy()
    fmap = tr.full_to_trimmed.cpu().numpy()
    want = P.select_kept(counts, k, reserved)
    assert kept.dtype == np.int32 and np.array_equal(kept, want)
    assert np.array_equal(fmap, P.full_to_trimmed_map(want, vocab, unk))
    return tr


@pytest.mark.parametrize("vocab,k,seed", [(60, 17, 0), (1024, 1, 1), (1025, 1025, 2), (2049, 700, 3), (5000, 4999, 4),
                                          (1, 1, 5), (18000, 6000, 6)])
def test_selection_with_ties_everywhere(E, vocab, k, seed):
    """Counts drawn from a handful of values, so the boundary always falls inside a run of equal counts."""
    rng = np.random.default_rng(seed)
    counts = rng.integers(0, 5, size=vocab).astype(np.uint64)
    n_res = min(k, 3, vocab)
    reserved = [int(x) for x in rng.choice(vocab, size=n_res, replace=False)]
    _say(f"[prune] select vocab {vocab} k {k} reserved {reserved}")
    _select_case(E, counts, k, reserved, reserved[-1])


def test_selection_on_counted_zipf_corpus_and_huge_counts(E):
    vocab = 18000
    ids = make_corpus(vocab, 2_000_000, seed=31)
    counts = P.count_tokens(ids, vocab)
    _select_case(E, counts, 6000, [0, 17999, 5], 5)
    big = counts * np.uint64(1 << 40) + np.uint64(3)              # values far beyond 32 bits
    _select_case(E, big, 8000, [100], 100)


def test_gather_rows_and_remaps_are_bit_copies(E):
    import torch
    vocab, d, k = 5000, 128, 777
    rng = np.random.default_rng(9)
    table = rng.standard_normal((vocab, d)).astype(np.float16)
    table[3, 5] = np.float16(np.nan); table[4, 6] = np.float16(-0.0)             # bit patterns, not values
    counts = P.count_tokens(make_corpus(vocab, 300_000, seed=9), vocab)
    unk = 1234
    tr = _select_case(E, counts, k, [unk, 3, 4], unk)
    kept = tr.kept_ids.cpu().numpy()
    got = tr.trim_table(_dev(table)).cpu().numpy()
    assert got.tobytes() == P.trim_rows(table, kept).tobytes()
    # full -> trimmed (out-of-range ids included), unaligned start, then in place
    ids = make_corpus(vocab, 100_003, seed=10, noise_ids=500)
    fmap = P.full_to_trimmed_map(kept, vocab, unk)
    unk_t = int(fmap[unk])
    d_ids = _dev(ids)
    for off in (0, 1, 2, 3):
        out = tr.to_trimmed(d_ids[off:]).cpu().numpy()
        assert np.array_equal(out, P.remap(ids[off:], fmap, unk_t))
    buf = d_ids.clone()
    assert E.ernie_remap_ids(buf, buf.numel(), tr.full_to_trimmed, vocab, unk_t, buf) == E.ERNIE_OK
    assert np.array_equal(buf.cpu().numpy(), P.remap(ids, fmap, unk_t))
    # trimmed -> full
    t = rng.integers(-2, k + 2, size=4099).astype(np.int32)
    assert np.array_equal(tr.to_full(_dev(t)).cpu().numpy(), P.remap(t, kept, -1))
    torch.cuda.synchronize()


def test_trimmed_vocabulary_feeds_the_generation_path(E):
    """End to end at the tiny shape: count a corpus, keep 300 of 1024 rows, trim the table, map prompts in,
    generate, map tokens out -- against the oracle's definition (full-table projection, kept rows selected)."""
    import torch
    sh = replace(CONFIGS["tiny_affine"], vocab_kept=300)
    w = make_weights(sh)
    corpus = make_corpus(sh.vocab_full, 200_000, seed=41)
    unk = 100
    tr = E.VocabTrimmer(sh.vocab_full)
    tr.count(_dev(corpus))
    kept_dev = tr.select(300, [unk], unk)
    kept = kept_dev.cpu().numpy()
    assert np.array_equal(kept, P.select_kept(P.count_tokens(corpus, sh.vocab_full), 300, [unk]))
    table_kept = tr.trim_table(_dev(w["tok_emb"])).cpu().numpy()
    # prompts: raw corpus slices in full ids (they contain dropped ids)
    rng = np.random.default_rng(5)
    raw = [corpus[s:s + sh.prompt_len].copy() for s in rng.integers(0, 100_000, size=sh.batch)]
    assert any(np.setdiff1d(r, kept).size for r in raw)
    ids_t = tr.to_trimmed(_dev(np.stack(raw)))
    fmap = P.full_to_trimmed_map(kept, sh.vocab_full, unk)
    assert np.array_equal(ids_t.cpu().numpy(), P.remap(np.stack(raw), fmap, int(fmap[unk])))
    # what the model then sees, in full ids: dropped ids replaced by the unknown-word id
    seen_full = [kept[fmap[r]] for r in raw]
    wl = Workload(sh, w, kept)
    wl.batches_full.append(seen_full)
    wl.batches_trimmed.append([fmap[r] for r in raw])
    weights = dict(w); weights["tok_emb_kept"] = table_kept
    eng = E.ErnieEngine(n_layers=sh.n_layers, d_model=sh.d_model, n_heads=sh.n_heads, d_ffn=sh.d_ffn,
                        vocab_full=sh.vocab_full, vocab_kept=300, max_pos=sh.max_pos, max_batch=sh.batch,
                        max_seq=sh.prompt_len + sh.n_gen, ln_eps=sh.ln_eps, weights=weights, kept_ids=kept)
    orc = oracle_generate(wl, 0, range(sh.batch), sh.n_gen, definition=True)
    lens = np.full(sh.batch, sh.prompt_len, dtype=np.int32)
    toks, hid, lg = gpu_generate(eng, ids_t.cpu().numpy(), lens, sh.n_gen, {r: orc[r]["tokens"] for r in orc})
    st = check_rows(orc, toks, hid, lg, "trimmed-by-gpu")
    _say(f"[prune] end to end: {st}")
    full_out = tr.to_full(_dev(toks.astype(np.int32))).cpu().numpy()
    assert np.array_equal(full_out, kept[toks])
    eng.close()
    torch.cuda.synchronize()


def test_argument_errors_with_live_buffers(E):
    import torch
    tr = E.VocabTrimmer(100)
    ids = _dev(np.arange(50, dtype=np.int32))
    k = torch.empty(10, dtype=torch.int32, device="cuda:0")
    assert E.ernie_vocab_count(ids, -1, 100, tr.counts) == E.ERNIE_EINVAL
    assert E.ernie_vocab_count(ids, 50, 0, tr.counts) == E.ERNIE_EINVAL
    assert E.ernie_vocab_count(ids, 50, 300000, tr.counts) == E.ERNIE_EINVAL
    assert E.ernie_vocab_count(None, 50, 100, tr.counts) == E.ERNIE_EINVAL
    for kk, res, unk in [(0, [1], 1), (101, [1], 1), (10, [1, 1], 1), (10, [100], 100), (10, [1], 2), (10, [], 1),
                         (2, [1, 2, 3], 1), (10, list(range(17)), 1)]:
        assert E.ernie_vocab_select(tr.counts, 100, kk, np.array(res, dtype=np.int32), unk, k, tr.full_to_trimmed) \
            == E.ERNIE_EINVAL, (kk, res, unk)
    tab = torch.zeros((100, 12), dtype=torch.float16, device="cuda:0")
    assert E.ernie_vocab_gather_rows(tab, 100, 12, k, 10, tab) == E.ERNIE_EINVAL          # d not a multiple of 8
    assert E.ernie_remap_ids(ids, 50, tr.full_to_trimmed, 0, 0, ids) == E.ERNIE_EINVAL
    torch.cuda.synchronize()
    assert int(_counts(tr).sum()) == 0                                                     # nothing was enqueued
