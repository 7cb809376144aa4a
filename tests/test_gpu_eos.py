"""End of sequence, batch compaction and batch planning through the C ABI, against the oracle."""
import numpy as np
import pytest

from oracle import ernie_oracle as O
from tests.parity_util import oracle_generate, gpu_generate, check_rows
from tests.test_gpu_parity import _ragged_workload

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


def _oracle_rows(wl, rows, n_gen, forced=None, eos=None):
    p = O.Params(wl.weights, wl.shape.n_heads, wl.shape.ln_eps)
    return {r: O.generate_cached(p, wl.batches_full[0][r], n_gen, wl.kept_ids,
                                 None if forced is None else forced[r], eos) for r in rows}


def _valid_prefix(o):
    """The steps of an oracle result that were really computed (rows after the end token are NaN)."""
    m = int(np.sum(~np.isnan(o["logits"][:, 0])))
    return {k: o[k][:m] for k in ("tokens", "hidden", "logits")}, m


def test_teacher_forced_end_tokens_stop_rows_independently(E):
    lengths = [5, 1, 17, 30, 9, 12]
    n_gen = 8
    wl = _ragged_workload(lengths, max_pos=64, n_gen=n_gen)
    B = len(lengths)
    free = _oracle_rows(wl, range(B), n_gen)
    used = set(int(t) for r in free for t in free[r]["tokens"])
    eos = next(i for i in range(len(wl.kept_ids)) if i not in used)
    # row r is fed the end token as its stop[r]-th fed-back token (None: never)
    stop = {0: None, 1: 0, 2: 3, 3: 6, 4: 1, 5: None}
    forced = {}
    for r in range(B):
        f = free[r]["tokens"].copy()
        if stop[r] is not None:
            f[stop[r]] = eos
        forced[r] = f
    orc = _oracle_rows(wl, range(B), n_gen, forced, eos)
    eng = E.engine_from_workload(wl, max_seq=max(lengths) + n_gen)
    eng.set_eos(eos)
    ids, lens = wl.padded(0)
    _say(f"[eos] teacher-forced stops {stop} eos {eos}")
    toks, hid, lg = gpu_generate(eng, ids, lens, n_gen, forced)
    for r in range(B):
        o, m = _valid_prefix(orc[r])
        assert m == (n_gen if stop[r] is None else stop[r] + 1) == orc[r]["steps"]
        check_rows({r: o}, toks, hid, lg, f"eos-row{r}")
        assert np.all(toks[m:, r] == eos)
    lens_d, fin_d = eng.state()
    want_len = [lengths[r] + orc[r]["steps"] - 1 for r in range(B)]
    assert lens_d.cpu().numpy().tolist() == want_len                       # a finished row's cache stops growing
    assert fin_d.cpu().numpy().tolist() == [0 if stop[r] is None else 1 for r in range(B)]
    # a new prefill clears the flags
    eng.prefill(__import__("torch").as_tensor(ids), lens)
    assert eng.state()[1].cpu().numpy().sum() == 0
    eng.close()


def test_free_running_rows_stop_at_their_own_end_token(E):
    """Without teacher forcing the end token is whatever a row emits: with the id set, every row repeats its
    own free-running trajectory up to and including its first end token and emits only that afterwards."""
    import torch
    lengths = [7, 19, 3, 26]
    n_gen = 10
    wl = _ragged_workload(lengths, max_pos=64, n_gen=n_gen)
    eng = E.engine_from_workload(wl, max_seq=max(lengths) + n_gen)
    ids, lens = wl.padded(0)
    base, _, _ = gpu_generate(eng, ids, lens, n_gen)
    eos = int(base[3, 0])                                # row 0 emits it at step 3 (or earlier)
    eng.set_eos(eos)
    got, _, _ = gpu_generate(eng, ids, lens, n_gen)
    for r in range(len(lengths)):
        hits = np.nonzero(base[:, r] == eos)[0]
        m = n_gen if hits.size == 0 else int(hits[0]) + 1
        assert np.array_equal(got[:m, r], base[:m, r]) and np.all(got[m:, r] == eos), r
    assert np.all(got[3:, 0] == eos)
    eng.set_eos(-1)
    again, _, _ = gpu_generate(eng, ids, lens, n_gen)
    assert np.array_equal(again, base)
    eng.close()
    torch.cuda.synchronize()


@pytest.mark.parametrize("B,keep1,keep2", [(8, [1, 4, 6], [0, 2]), (70, list(range(3, 70, 2))[:30] + [69], [0, 5, 30])])
def test_compaction_keeps_the_surviving_rows_exact(E, B, keep1, keep2):
    """Rows dropped between steps: the survivors continue exactly as if nothing had happened (their cache rows
    are reached through the row map).  The 70-row case moves from the large-batch to the small-batch decode path."""
    import torch
    rng = np.random.default_rng(B)
    lengths = [int(x) for x in rng.integers(2, 40, size=B)]
    n_gen = 9
    wl = _ragged_workload(lengths, max_pos=64, n_gen=n_gen)
    final_rows = [keep1[i] for i in keep2]
    orc = oracle_generate(wl, 0, keep1 if B <= 8 else final_rows, n_gen)
    eng = E.engine_from_workload(wl, max_seq=max(lengths) + n_gen)
    ids, lens = wl.padded(0)
    _say(f"[eos] compaction {B} -> {len(keep1)} -> {len(keep2)}")
    tok, lo, ho = eng.prefill(torch.as_tensor(ids), lens, logits=True, hidden=True)
    rows = list(range(B))                                # original row of each current batch row
    got = {r: {"tokens": [], "hidden": [], "logits": []} for r in range(B)}

    def record():
        t, l, h = tok.cpu().numpy(), lo.cpu().numpy(), ho.cpu().numpy()
        for i, r in enumerate(rows):
            got[r]["tokens"].append(t[i]); got[r]["hidden"].append(h[i]); got[r]["logits"].append(l[i])

    record()
    for step in range(1, n_gen):
        if step == 3:
            eng.compact(keep1); rows = [rows[i] for i in keep1]; tok = tok[torch.as_tensor(keep1, device=tok.device)]
        if step == 6:
            eng.compact(keep2); rows = [rows[i] for i in keep2]; tok = tok[torch.as_tensor(keep2, device=tok.device)]
        feed = tok.clone()
        for i, r in enumerate(rows):
            if r in orc:
                feed[i] = int(orc[r]["tokens"][step - 1])
        tok, lo, ho = eng.decode_step(feed, logits=True, hidden=True)
        assert tok.shape[0] == len(rows)
        record()
    for r in orc:
        n = len(got[r]["tokens"])
        assert n == (n_gen if r in final_rows else 6)
        o = {k: orc[r][k][:n] for k in ("tokens", "hidden", "logits")}
        toks = np.array(got[r]["tokens"])[:, None]; hid = np.array(got[r]["hidden"])[:, None]
        lg = np.array(got[r]["logits"])[:, None]
        check_rows({0: o}, toks, hid, lg, f"compact-row{r}")
    lens_d, _ = eng.state()
    assert lens_d.cpu().numpy().tolist() == [lengths[r] + n_gen - 1 for r in rows]
    # identity list: nothing to do; then a fresh prefill restores the full batch
    eng.compact(list(range(len(rows))))
    tok2, _, _ = eng.prefill(torch.as_tensor(ids), lens)
    assert tok2.shape[0] == B and np.array_equal(tok2.cpu().numpy(), np.array([got[r]["tokens"][0] for r in range(B)]))
    eng.close()


def test_state_and_compaction_errors(E):
    import torch
    wl = _ragged_workload([4, 5, 6], max_pos=32, n_gen=3)
    eng = E.engine_from_workload(wl)
    assert E.ernie_compact(eng.handle, [0]) == E.ERNIE_ESEQUENCE
    assert E.ernie_batch_state(eng.handle, None, None) == E.ERNIE_ESEQUENCE
    ids, lens = wl.padded(0)
    eng.prefill(torch.as_tensor(ids), lens)
    for bad in ([], [0, 0], [1, 0], [3], [-1], [0, 1, 2, 2]):
        assert E.ernie_compact(eng.handle, bad) == E.ERNIE_EINVAL, bad
    for bad in (-2, len(wl.kept_ids)):
        assert E.ernie_set_eos(eng.handle, bad) == E.ERNIE_EINVAL
    assert E.ernie_set_eos(eng.handle, 0) == E.ERNIE_OK and E.ernie_set_eos(eng.handle, -1) == E.ERNIE_OK
    assert eng.state()[0].cpu().numpy().tolist() == [4, 5, 6]
    eng.close()
