"""Parity of the HIP path with the CPU oracle, through the C ABI, on seeded synthetic inputs."""
from dataclasses import replace

import numpy as np
import pytest

from synth import CONFIGS, make_workload, Workload, make_weights, make_kept_ids, full_to_trimmed
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


@pytest.mark.parametrize("name", ["tiny", "tiny_affine", "tiny_head"])
def test_tiny_all_rows_against_the_definition(E, name):
    """cfg 0 / 0b / 0c (0b plus segment embedding, output-head transform and output bias): every row, every step,
    against the full-recompute definition."""
    _say(f"[parity] {name}")
    wl = make_workload(name)
    sh = wl.shape
    eng = E.engine_from_workload(wl)
    ids, lens = wl.padded(0)
    orc = oracle_generate(wl, 0, range(sh.batch), sh.n_gen, definition=True)
    forced = {r: orc[r]["tokens"] for r in orc}
    toks, hid, lg = gpu_generate(eng, ids, lens, sh.n_gen, forced)
    st = check_rows(orc, toks, hid, lg, name)
    _say(f"[parity] {name}: {st}")
    assert st["exact_required"] > 0
    eng.close()


def test_free_running_matches_teacher_forced(E):
    """Feeding back the on-device argmax (tok_in = NULL) gives the same trajectory as feeding the same ids."""
    import torch
    wl = make_workload("tiny_affine")
    sh = wl.shape
    eng = E.engine_from_workload(wl)
    ids, lens = wl.padded(0)
    tok, lo, _ = eng.prefill(torch.as_tensor(ids), lens, logits=True)
    free_toks, free_logits = [tok.cpu().numpy()], [lo.cpu().numpy()]
    for _ in range(1, sh.n_gen):
        tok, lo, _ = eng.decode_step(None, logits=True)
        free_toks.append(tok.cpu().numpy()); free_logits.append(lo.cpu().numpy())
    tok, lo, _ = eng.prefill(torch.as_tensor(ids), lens, logits=True)
    for t in range(1, sh.n_gen):
        assert np.array_equal(tok.cpu().numpy(), free_toks[t - 1])
        tok, lo, _ = eng.decode_step(torch.as_tensor(free_toks[t - 1]), logits=True)
        assert np.array_equal(lo.cpu().numpy(), free_logits[t])      # same kernels, same inputs: bit-identical
    eng.close()


def _ragged_workload(lengths, name="tiny_affine", **kw):
    """A batch with the given prompt lengths at the tiny shape (d = 128, 2 heads)."""
    sh = replace(CONFIGS[name], batch=len(lengths), prompt_len=max(lengths), **kw)
    kept = make_kept_ids(sh)
    w = make_weights(sh)
    rng = np.random.default_rng(777)
    seqs = [kept[rng.integers(0, len(kept), size=n)].astype(np.int32) for n in lengths]
    wl = Workload(sh, w, kept)
    wl.batches_full.append(seqs)
    wl.batches_trimmed.append([full_to_trimmed(s, kept) for s in seqs])
    return wl


def test_ragged_batch_spanning_tiles(E):
    """Variable lengths 1..200: several 128-row GEMM tiles, several attention key blocks, ragged tails, L = 1."""
    lengths = [1, 2, 31, 33, 64, 65, 127, 130, 200]
    n_gen = 6
    wl = _ragged_workload(lengths, max_pos=256, n_gen=n_gen)
    eng = E.engine_from_workload(wl, max_seq=max(lengths) + n_gen)
    ids, lens = wl.padded(0)
    _say(f"[parity] ragged lengths {lengths}")
    orc = oracle_generate(wl, 0, range(len(lengths)), n_gen)
    forced = {r: orc[r]["tokens"] for r in orc}
    toks, hid, lg = gpu_generate(eng, ids, lens, n_gen, forced)
    st = check_rows(orc, toks, hid, lg, "ragged")
    _say(f"[parity] ragged: {st}")
    eng.close()


def test_padding_and_batch_neighbours_do_not_matter(E):
    """A sequence's outputs are independent of pad width, pad values, batch order and the other sequences."""
    import torch
    lengths = [40, 7, 90]
    n_gen = 4
    wl = _ragged_workload(lengths, max_pos=256, n_gen=n_gen)
    eng = E.engine_from_workload(wl, max_batch=4, max_seq=160)
    ids, lens = wl.padded(0)
    a_t, a_h, a_l = gpu_generate(eng, ids, lens, n_gen)
    # wider padding filled with junk ids, reversed batch order, one extra neighbour
    wide = np.full((4, 150), 3, dtype=np.int32)
    order = [2, 1, 0]
    for i, r in enumerate(order):
        wide[i, :lengths[r]] = ids[r, :lengths[r]]
    wide[3, :5] = 1
    lens2 = np.array([lengths[r] for r in order] + [5], dtype=np.int32)
    b_t, b_h, b_l = gpu_generate(eng, wide, lens2, n_gen)
    for i, r in enumerate(order):
        assert np.array_equal(a_t[:, r], b_t[:, i])
        assert np.max(np.abs(a_l[:, r] - b_l[:, i])) <= 1e-5
        assert np.max(np.abs(a_h[:, r] - b_h[:, i])) <= 1e-5
    eng.close()


def test_kv_cache_contents_and_lengths(E):
    """The cache holds K, V of exactly the valid positions, head-major, and lengths advance by one per step."""
    import ctypes as C
    import torch
    from oracle import ernie_oracle as O
    lengths = [5, 37]
    wl = _ragged_workload(lengths, max_pos=64, n_gen=3)
    sh = wl.shape
    S = 48
    eng = E.engine_from_workload(wl, max_seq=S)
    ids, lens = wl.padded(0)
    orc = oracle_generate(wl, 0, range(2), 3)
    gpu_generate(eng, ids, lens, 3, {r: orc[r]["tokens"] for r in orc})
    ptr, nbytes = eng.debug_buffer("kv")
    H, d = sh.n_heads, sh.d_model
    assert nbytes == sh.n_layers * 2 * 2 * S * d * 2
    buf = torch.empty(nbytes // 2, dtype=torch.float16, device="cuda:0")
    C.CDLL("libamdhip64.so.7").hipMemcpy(C.c_void_p(buf.data_ptr()), C.c_void_p(ptr), C.c_size_t(nbytes), 3)
    kv = buf.cpu().numpy().astype(np.float64).reshape(sh.n_layers, 2, 2, H, S, 64)
    lptr, _ = eng.debug_buffer("lens")
    lens_dev = torch.empty(2, dtype=torch.int32, device="cuda:0")
    C.CDLL("libamdhip64.so.7").hipMemcpy(C.c_void_p(lens_dev.data_ptr()), C.c_void_p(lptr), C.c_size_t(8), 3)
    assert lens_dev.cpu().tolist() == [lengths[0] + 2, lengths[1] + 2]
    # layer-0 keys/values of the prompt straight from the definition
    p = O.Params(wl.weights, sh.n_heads, sh.ln_eps)
    for b, L in enumerate(lengths):
        X = O.embed(p, wl.batches_full[0][b])
        lw = p.layers[0]
        QKV = X @ lw["wqkv"].T + lw["bqkv"]
        K, V = QKV[:, d:2 * d], QKV[:, 2 * d:]
        for h in range(H):
            assert np.max(np.abs(kv[0, 0, b, h, :L] - K[:, 64 * h:64 * h + 64])) < 5e-3
            assert np.max(np.abs(kv[0, 1, b, h, :L] - V[:, 64 * h:64 * h + 64])) < 5e-3
    eng.close()


def test_error_paths_with_a_live_handle(E):
    import torch
    wl = make_workload("tiny")
    eng = E.engine_from_workload(wl, max_batch=2, max_seq=34)
    ids, lens = wl.padded(0)
    dev_ids = torch.as_tensor(ids).cuda()
    tok = torch.empty(2, dtype=torch.int32, device="cuda:0")
    h = eng.handle
    assert E.ernie_decode_step(h, None, None, None, tok) == E.ERNIE_ESEQUENCE          # before any prefill
    assert E.ernie_prefill(h, 3, 32, dev_ids, np.array([32, 32, 32]), None, None, tok) == E.ERNIE_ECAPACITY
    assert E.ernie_prefill(h, 2, 35, dev_ids, lens, None, None, tok) == E.ERNIE_ECAPACITY      # Lmax > max_seq
    assert E.ernie_prefill(h, 2, 32, dev_ids, np.array([0, 32]), None, None, tok) == E.ERNIE_EINVAL
    assert E.ernie_prefill(h, 2, 32, dev_ids, np.array([33, 32]), None, None, tok) == E.ERNIE_EINVAL
    assert E.ernie_prefill(h, 2, 32, dev_ids, lens, None, None, None) == E.ERNIE_EINVAL
    assert E.ernie_decode_step(h, None, None, None, tok) == E.ERNIE_ESEQUENCE          # failed calls left no state
    assert E.ernie_prefill(h, 2, 32, dev_ids, lens, None, None, tok) == E.ERNIE_OK
    assert E.ernie_decode_step(h, None, None, None, tok) == E.ERNIE_OK                 # slot 32
    assert E.ernie_decode_step(h, None, None, None, tok) == E.ERNIE_OK                 # slot 33
    assert E.ernie_decode_step(h, None, None, None, tok) == E.ERNIE_ECAPACITY          # slot 34 does not exist
    torch.cuda.synchronize()
    # arena too small / misaligned
    rc, need, _ = E.ernie_init_weights(eng.cfg, None, None)
    assert rc == E.ERNIE_OK and need == eng.arena_bytes
    eng.close()


def test_argmax_ties_pick_the_lowest_index(E):
    """Two identical rows in the trimmed table give exactly equal logits: the lower index must win."""
    import torch
    wl = make_workload("tiny")
    kept = wl.kept_ids
    # make kept row 400 a copy of kept row 17, and make both dominate: scale that row up
    te = wl.weights["tok_emb"].copy()
    te[kept[17]] = (te[kept[17]].astype(np.float32) * 40).astype(np.float16)
    te[kept[400]] = te[kept[17]]
    wl.weights["tok_emb"] = te
    eng = E.engine_from_workload(wl)
    ids, lens = wl.padded(0)
    tok, lo, ho = eng.prefill(torch.as_tensor(ids), lens, logits=True, hidden=True)
    lo = lo.cpu().numpy(); tok = tok.cpu().numpy()
    assert np.array_equal(lo[:, 17], lo[:, 400])
    for b in range(2):
        assert tok[b] == int(np.argmax(lo[b]))
        if np.argmax(lo[b]) in (17, 400):
            assert tok[b] == 17
    eng.close()


def test_base_shape_sampled_rows(E):
    """cfg 1 (ERNIE-base, batch 32, prompt 128, 32 tokens) at full size, in the launch configuration the
    benchmark times; the oracle computes a sample of rows one by one."""
    wl = make_workload("base")
    sh = wl.shape
    eng = E.engine_from_workload(wl)
    ids, lens = wl.padded(0)
    rows = [0, 13, 31]
    _say(f"[parity] base rows {rows}")
    orc = oracle_generate(wl, 0, rows, sh.n_gen)
    forced = {r: orc[r]["tokens"] for r in orc}
    toks, hid, lg = gpu_generate(eng, ids, lens, sh.n_gen, forced)
    st = check_rows(orc, toks, hid, lg, "base")
    _say(f"[parity] base: {st}")
    assert st["exact_required"] >= st["total"] // 4
    eng.close()
    # the L2 warm-up workgroups (on by default at this shape) load and discard: any count gives the same bits
    for count, kv in ((0, 0), (8, 8), (200, 1000)):
        eng = E.engine_from_workload(wl)
        eng.tune("dec_prefetch", count); eng.tune("kv_prefetch", kv)
        toks2, hid2, lg2 = gpu_generate(eng, ids, lens, 6, forced)
        assert np.array_equal(lg2, lg[:6]) and np.array_equal(toks2, toks[:6]), f"dec_prefetch={count} kv_prefetch={kv} changed results"
        eng.close()


@pytest.mark.parametrize("B", [40, 70, 130, 256])
def test_decode_paths_by_batch_size(E, B):
    """Batch sizes that select each decode kernel variant (1, 2, 4, 8 row tiles; fused and per-operation paths)."""
    rng = np.random.default_rng(B)
    lengths = [int(x) for x in rng.integers(3, 40, size=B)]
    n_gen = 4
    wl = _ragged_workload(lengths, max_pos=64, n_gen=n_gen)
    eng = E.engine_from_workload(wl, max_seq=max(lengths) + n_gen)
    ids, lens = wl.padded(0)
    rows = [0, B // 3, B // 2, B - 1]
    _say(f"[parity] batch {B} rows {rows}")
    orc = oracle_generate(wl, 0, rows, n_gen)
    toks, hid, lg = gpu_generate(eng, ids, lens, n_gen, {r: orc[r]["tokens"] for r in orc})
    st = check_rows(orc, toks, hid, lg, f"batch{B}")
    _say(f"[parity] batch {B}: {st}")
    eng.close()


@pytest.mark.parametrize("keys", [("type_emb",), ("head_w", "head_b", "head_ln_g", "head_ln_b"), ("out_bias",)])
def test_each_optional_variant_alone(E, keys):
    """One variant switched on at a time, ragged lengths: a variant wired to the wrong place cannot hide behind another."""
    lengths = [1, 9, 33, 40]
    n_gen = 5
    wl = _ragged_workload(lengths, name="tiny_head", max_pos=64, n_gen=n_gen)
    for k in ("type_emb", "head_w", "head_b", "head_ln_g", "head_ln_b", "out_bias"):
        if k not in keys:
            wl.weights.pop(k)
    eng = E.engine_from_workload(wl, max_seq=max(lengths) + n_gen)
    ids, lens = wl.padded(0)
    _say(f"[parity] variant {keys[0]} alone")
    orc = oracle_generate(wl, 0, range(len(lengths)), n_gen, definition=True)
    toks, hid, lg = gpu_generate(eng, ids, lens, n_gen, {r: orc[r]["tokens"] for r in orc})
    check_rows(orc, toks, hid, lg, f"variant-{keys[0]}")
    eng.close()


@pytest.mark.parametrize("B", [70, 256])
def test_variants_on_the_large_batch_decode_path(E, B):
    rng = np.random.default_rng(1000 + B)
    lengths = [int(x) for x in rng.integers(3, 40, size=B)]
    n_gen = 4
    wl = _ragged_workload(lengths, name="tiny_head", max_pos=64, n_gen=n_gen)
    eng = E.engine_from_workload(wl, max_seq=max(lengths) + n_gen)
    ids, lens = wl.padded(0)
    rows = [0, B // 2, B - 1]
    _say(f"[parity] variants, batch {B} rows {rows}")
    orc = oracle_generate(wl, 0, rows, n_gen)
    toks, hid, lg = gpu_generate(eng, ids, lens, n_gen, {r: orc[r]["tokens"] for r in orc})
    check_rows(orc, toks, hid, lg, f"variants-batch{B}")
    eng.close()


def test_partial_head_parameters_are_rejected(E):
    wl = make_workload("tiny_head")
    wl.weights.pop("head_ln_b")
    with pytest.raises(E.ErnieError):
        E.engine_from_workload(wl)


@pytest.mark.parametrize("vocab_kept,knobs", [(512, {"big_logits_gemm": 0, "big_ln_rows": 4}),
                                              (512, {"big_f1_fused": 0, "big_warm": 0, "big_ln_rows": 2}),
                                              (300, {"big_warm": 200}), (512, {"big_f1_tile": 1}), (512, {"big_f1_tile": 2, "big_narrow": 0, "big_mfast": 0})])
def test_large_batch_path_alternatives(E, vocab_kept, knobs):
    """B > 64 with each alternative of the large-batch path switched: projection by the skinny kernel instead of
    the GEMM pipeline, first FFN GEMM split with a separate GELU kernel, and a kept-row count that is not a
    multiple of 8 (which the GEMM-pipeline projection cannot take); the small-vector warm-up hosted by the attention
    is off, default or large; the LayerNorm row kernels run with four, two or one row per workgroup; the unsplit
    FFN1 GEMM and the split projections run on 64 x 32 or 64 x 64 tiles."""
    B = 130
    rng = np.random.default_rng(4242)
    lengths = [int(x) for x in rng.integers(3, 40, size=B)]
    n_gen = 4
    wl = _ragged_workload(lengths, max_pos=64, n_gen=n_gen, vocab_kept=vocab_kept)
    eng = E.engine_from_workload(wl, max_seq=max(lengths) + n_gen)
    for k, v in knobs.items():
        eng.tune(k, v)
    ids, lens = wl.padded(0)
    rows = [0, 64, B - 1]
    _say(f"[parity] large-batch alternatives V'={vocab_kept} {knobs}")
    orc = oracle_generate(wl, 0, rows, n_gen)
    toks, hid, lg = gpu_generate(eng, ids, lens, n_gen, {r: orc[r]["tokens"] for r in orc})
    check_rows(orc, toks, hid, lg, f"big-alt-{vocab_kept}")
    eng.close()


def test_host_lengths_survive_unsynchronised_calls_and_graph_replays(E):
    """The prompt lengths travel through library-owned pinned memory.  (a) Twenty prefills of two alternating
    ragged batches issued back to back without synchronisation: the last one decides the state.  (b) A prefill
    captured into a graph keeps reading the lengths of capture time, however many eager calls with other lengths
    follow.  (c) The ninth captured prefill on one handle is refused with the capacity error."""
    import torch
    la = [5, 17, 9, 30, 3, 12]
    lb = [30, 4, 22, 7, 15, 6]
    wl_a = _ragged_workload(la, max_pos=64, n_gen=3, vocab_kept=512)
    ids_a, _ = wl_a.padded(0)
    rng = np.random.default_rng(99)
    ids_b = rng.integers(0, 512, size=ids_a.shape).astype(np.int32)
    eng = E.engine_from_workload(wl_a, max_seq=40)
    ref = E.engine_from_workload(wl_a, max_seq=40)
    dev_a, dev_b = torch.as_tensor(ids_a).cuda(), torch.as_tensor(ids_b).cuda()
    tok = torch.empty(len(la), dtype=torch.int32, device="cuda:0")
    tok_ref = torch.empty_like(tok)
    _say("[parity] twenty unsynchronised prefills")
    for i in range(20):
        ids, lens = (dev_a, la) if i % 2 else (dev_b, lb)
        assert E.ernie_prefill(eng.handle, len(lens), ids.shape[1], ids, lens, None, None, tok) == 0
    assert E.ernie_decode_step(eng.handle, None, None, None, tok) == 0
    assert E.ernie_prefill(ref.handle, len(la), dev_a.shape[1], dev_a, la, None, None, tok_ref) == 0
    assert E.ernie_decode_step(ref.handle, None, None, None, tok_ref) == 0
    torch.cuda.synchronize()
    assert torch.equal(tok, tok_ref)
    lens_dev = torch.empty(len(la), dtype=torch.int32, device="cuda:0")
    assert E.ernie_batch_state(eng.handle, lens_dev, None) == 0
    assert lens_dev.cpu().tolist() == [x + 1 for x in la]

    _say("[parity] captured prefill replayed after ten eager prefills with other lengths")
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    tok_g = torch.empty_like(tok)
    with torch.cuda.graph(g, stream=side):
        assert E.ernie_prefill(eng.handle, len(la), dev_a.shape[1], dev_a, la, None, None, tok_g) == 0
        assert E.ernie_decode_step(eng.handle, None, None, None, tok_g) == 0
    for i in range(10):
        assert E.ernie_prefill(eng.handle, len(lb), dev_b.shape[1], dev_b, lb, None, None, tok) == 0
    torch.cuda.synchronize()
    for _ in range(2):
        tok_g.zero_()
        with torch.cuda.stream(side):
            g.replay()
        side.synchronize()
        assert torch.equal(tok_g, tok_ref)

    _say("[parity] capture slots run out")
    codes = []
    g2 = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g2, stream=side):
        for i in range(8):
            codes.append(E.ernie_prefill(eng.handle, len(la), dev_a.shape[1], dev_a, la, None, None, tok_g))
    assert codes == [0] * 7 + [E.ERNIE_ECAPACITY], codes
    torch.cuda.synchronize()
    eng.close(); ref.close()


@pytest.mark.parametrize("seed", [11, 12, 13, 14, 15, 16, 17, 18])
def test_seeded_random_small_configurations(E, seed):
    """Model width, FFN width, depth, batch, ragged lengths, kept-row count and generated length drawn from a seed:
    shapes that no named configuration has (one head, widths that are not powers of two, a single layer, batches
    on both decode paths), three sampled rows against the oracle."""
    rng = np.random.default_rng(seed)
    heads = int(rng.choice([1, 2, 3, 5]))
    d_ffn = int(rng.choice([64, 192, 320, 512]))
    layers = int(rng.integers(1, 4))
    B = int(rng.choice([1, 2, 7, 33, 64, 65, 90]))
    lengths = [int(x) for x in rng.integers(1, 45, size=B)]
    n_gen = int(rng.integers(1, 5))
    vocab_kept = int(rng.integers(65, 700))
    wl = _ragged_workload(lengths, max_pos=64, n_gen=n_gen, vocab_kept=vocab_kept, n_layers=layers,
                          d_model=64 * heads, n_heads=heads, d_ffn=d_ffn)
    eng = E.engine_from_workload(wl, max_seq=max(lengths) + n_gen)
    ids, lens = wl.padded(0)
    rows = sorted({0, B // 2, B - 1})
    _say(f"[parity] seed {seed}: layers={layers} d={64 * heads} ffn={d_ffn} B={B} V'={vocab_kept} n_gen={n_gen}")
    orc = oracle_generate(wl, 0, rows, n_gen)
    toks, hid, lg = gpu_generate(eng, ids, lens, n_gen, {r: orc[r]["tokens"] for r in orc})
    check_rows(orc, toks, hid, lg, f"seeded-{seed}")
    eng.close()


@pytest.mark.parametrize("d_model,heads,B", [(1280, 20, 3), (1280, 20, 70), (2048, 32, 5), (2048, 32, 66), (4096, 64, 2)])
def test_model_widths_above_1024(E, d_model, heads, B):
    """Widths the named configurations do not reach: the row kernels' 4- and 8-chunk instantiations, prefill GEMMs with
    a contraction above 1024, and small batches on the large-batch decode path (the small-batch paths stop at 1024)."""
    rng = np.random.default_rng(d_model + B)
    lengths = [int(x) for x in rng.integers(1, 40, size=B)]
    n_gen = 3
    wl = _ragged_workload(lengths, max_pos=64, n_gen=n_gen, vocab_kept=200, n_layers=1, d_model=d_model, n_heads=heads,
                          d_ffn=256)
    eng = E.engine_from_workload(wl, max_seq=max(lengths) + n_gen)
    ids, lens = wl.padded(0)
    rows = sorted({0, B - 1})
    _say(f"[parity] width {d_model}, batch {B}")
    orc = oracle_generate(wl, 0, rows, n_gen)
    toks, hid, lg = gpu_generate(eng, ids, lens, n_gen, {r: orc[r]["tokens"] for r in orc})
    check_rows(orc, toks, hid, lg, f"width-{d_model}")
    eng.close()


@pytest.mark.parametrize("seed", [1001, 1002, 1003, 1004])
def test_seeded_random_wide_configurations(E, seed):
    """As above at widths and lengths of the benchmark models: 8-16 heads, FFN width up to 4096, prompts up to 300
    (several attention key blocks and GEMM tiles), batches up to 256, with or without the optional model variants."""
    rng = np.random.default_rng(seed)
    heads = int(rng.choice([8, 12, 16]))
    d_ffn = int(rng.choice([1024, 3072, 4096]))
    layers = int(rng.integers(1, 3))
    B = int(rng.choice([8, 40, 70, 140, 256]))
    lmax = int(rng.choice([130, 300]))
    lengths = [int(x) for x in rng.integers(1, lmax + 1, size=B)]
    n_gen = int(rng.integers(1, 4))
    vocab_kept = int(rng.integers(1000, 9000))
    name = str(rng.choice(["tiny_affine", "tiny_head"]))
    wl = _ragged_workload(lengths, name=name, max_pos=lmax + 8, n_gen=n_gen, vocab_kept=vocab_kept, vocab_full=12000,
                          n_layers=layers, d_model=64 * heads, n_heads=heads, d_ffn=d_ffn)
    eng = E.engine_from_workload(wl, max_seq=max(lengths) + n_gen)
    ids, lens = wl.padded(0)
    rows = sorted({0, B - 1})
    _say(f"[parity] seed {seed}: {name} layers={layers} d={64 * heads} ffn={d_ffn} B={B} lmax={lmax} V'={vocab_kept} n_gen={n_gen}")
    orc = oracle_generate(wl, 0, rows, n_gen)
    toks, hid, lg = gpu_generate(eng, ids, lens, n_gen, {r: orc[r]["tokens"] for r in orc})
    check_rows(orc, toks, hid, lg, f"seeded-wide-{seed}")
    eng.close()


def test_prefill_gemm_tile_shapes_agree(E):
    """Every tile shape of the prefill GEMM (chosen by problem size, here forced: 256 x 256, 128 x 128, 64 x 64) meets
    the oracle on a ragged batch whose packed token count spans several tiles with a partial last one and whose
    widths are below one large tile, and all shapes give bit-identical logits (the contraction order per output
    element does not depend on the tile)."""
    B = 70
    rng = np.random.default_rng(777)
    lengths = [int(x) for x in rng.integers(3, 40, size=B)]
    wl = _ragged_workload(lengths, max_pos=64, n_gen=2, vocab_kept=512)
    ids, lens = wl.padded(0)
    rows = [0, 33, B - 1]
    orc = oracle_generate(wl, 0, rows, 2)
    ref = None
    for tile in (0, 1, 2, 3):
        eng = E.engine_from_workload(wl, max_seq=max(lengths) + 2)
        eng.tune("pf_tile", tile)
        _say(f"[parity] prefill GEMM tile shape {tile}, {sum(lengths)} packed tokens")
        toks, hid, lg = gpu_generate(eng, ids, lens, 2, {r: orc[r]["tokens"] for r in orc})
        check_rows(orc, toks, hid, lg, f"pf-tile-{tile}")
        if ref is None:
            ref = lg
        else:
            assert np.array_equal(np.asarray(ref), np.asarray(lg)), f"tile shape {tile} changed the logits"
        eng.close()


def test_decode_tuning_variants_agree(E):
    """Every split-K setting and both decode paths meet the oracle and agree with each other closely."""
    wl = make_workload("tiny_affine")
    sh = wl.shape
    ids, lens = wl.padded(0)
    orc = oracle_generate(wl, 0, range(sh.batch), sh.n_gen)
    forced = {r: orc[r]["tokens"] for r in orc}
    ref = None
    for fused, sk_out, sk_f2, ln_ns in [(1, 1, 1, 1), (0, 1, 1, 1), (1, 2, 2, 1), (1, 4, 2, 2), (1, 1, 4, 4), (1, 2, 4, 2)]:
        eng = E.engine_from_workload(wl)
        eng.tune("fused_decode", fused); eng.tune("sk_out", sk_out); eng.tune("sk_f2", sk_f2); eng.tune("ln_ns", ln_ns)
        eng.tune("dec_nw16", (sk_out + sk_f2 + ln_ns) % 4)        # every setting of the wave-count knob appears once
        eng.tune("dec_prefetch", (0, 8, 64, 200, 24, 1024)[(sk_out * 2 + sk_f2 + ln_ns) % 6])   # L2 warm-up workgroups: none .. many
        eng.tune("kv_prefetch", (1, 0, 16, 2048, 1, 40)[(sk_out + sk_f2 * 2 + ln_ns) % 6])
        _say(f"[parity] variant fused={fused} sk_out={sk_out} sk_f2={sk_f2} ln_ns={ln_ns}")
        toks, hid, lg = gpu_generate(eng, ids, lens, sh.n_gen, forced)
        check_rows(orc, toks, hid, lg, f"variant{(fused, sk_out, sk_f2, ln_ns)}")
        if ref is None:
            ref = lg
        assert np.max(np.abs(lg - ref)) < 2e-3
        eng.close()
    eng = E.engine_from_workload(wl)
    with pytest.raises(E.ErnieError):
        eng.tune("sk_out", 3)         # only 1, 2 and 4 partial buffers are supported
    with pytest.raises(E.ErnieError):
        eng.tune("no_such_knob", 1)
    eng.close()


def test_decode_attention_shapes_and_poisoned_cache_tail(E):
    """Every decode-attention shape meets the oracle on caches that straddle its batch sizes (128, 192, 256 keys),
    with every cache slot past the valid lengths holding NaN bit patterns."""
    import ctypes as C
    import torch
    lengths = [1, 7, 63, 125, 127, 128, 190, 193, 250]
    n_gen = 6
    wl = _ragged_workload(lengths, max_pos=256, n_gen=n_gen)
    ids, lens = wl.padded(0)
    orc = oracle_generate(wl, 0, range(len(lengths)), n_gen)
    forced = {r: orc[r]["tokens"] for r in orc}
    hip = C.CDLL("libamdhip64.so.7")
    for variant, nt in ((0, 1), (1, 0), (1, 1), (2, 0), (3, 0), (4, 1), (5, 1)):
        eng = E.engine_from_workload(wl, max_seq=max(lengths) + n_gen)
        eng.tune("attn_dec", variant)
        eng.tune("attn_nt", nt)              # cache rows read with / without the streaming (non-temporal) hint
        ptr, nbytes = eng.debug_buffer("kv")
        torch.cuda.synchronize()
        assert hip.hipMemset(C.c_void_p(ptr), 0xFF, C.c_size_t(nbytes)) == 0     # fp16 0xFFFF is a NaN
        torch.cuda.synchronize()
        _say(f"[parity] decode attention shape {variant}, poisoned cache")
        toks, hid, lg = gpu_generate(eng, ids, lens, n_gen, forced)
        assert np.isfinite(lg).all() and np.isfinite(hid).all()
        check_rows(orc, toks, hid, lg, f"attn_dec{variant}")
        eng.close()
    eng = E.engine_from_workload(wl, max_seq=max(lengths) + n_gen)
    with pytest.raises(E.ErnieError):
        eng.tune("attn_dec", 6)
    eng.close()


def test_profile_hooks_count_launches(E):
    """ernie_profile brackets every launch of a kernel family; counts and algorithmic bytes match the step structure,
    with the layers of a step as one kernel (default) and as five kernels per layer."""
    import torch
    wl = make_workload("tiny_affine")
    sh = wl.shape
    eng = E.engine_from_workload(wl)
    ids, lens = wl.padded(0)
    Nl, d, f = sh.n_layers, sh.d_model, sh.d_ffn
    w_layer = (4 * d * d + 2 * d * f) * 2
    kv = sum(2 * (int(lens.sum()) + sh.batch * (t + 1)) * d * 2 for t in range(3)) * Nl
    for persist in (1, 0):
        eng.tune("persist", persist)
        eng.profile(True)
        tok, _, _ = eng.prefill(torch.as_tensor(ids), lens)
        for _ in range(3):
            eng.decode_step(None)
        torch.cuda.synchronize()
        p = eng.profile_read()
        assert p["gemm_prefill"][1] == 4 * Nl and p["attn_prefill"][1] == Nl
        assert p["logits"][1] == 3
        if persist:
            assert p["dec_persist"][1] == 3 and p["attn_dec"][1] == 0 and p["gemm_dec"][1] == 0 and p["gemm_dec_ln"][1] == 0
            assert p["row_dec"][1] == 3                                          # second argmax stage
            assert abs(p["dec_persist"][2] - (3 * Nl * w_layer + kv)) < 1
            assert p["dec_persist"][0] > 0.0
        else:
            assert p["dec_persist"][1] == 0 and p["attn_dec"][1] == 3 * Nl
            assert p["gemm_dec"][1] + p["gemm_dec_ln"][1] == 3 * 4 * Nl          # four projections per layer per step
            assert p["gemm_dec_ln"][1] == 3 * 2 * Nl                             # every QKV (layer 0: embedding prologue) and FFN1
            assert p["row_dec"][1] == 3 * 2                                      # final LayerNorm and second argmax stage per step
            assert abs(p["gemm_dec"][2] + p["gemm_dec_ln"][2] - 3 * Nl * w_layer) < 1
            assert abs(p["attn_dec"][2] - kv) < 1
            for name in ("attn_dec", "gemm_dec", "gemm_dec_ln"):
                assert p[name][0] > 0.0
        assert abs(p["gemm_prefill"][3] - 2 * int(lens.sum()) * Nl * (4 * d * d + 2 * d * f)) < 1
        for name in ("gemm_prefill", "attn_prefill", "logits"):
            assert p[name][0] > 0.0
    eng.profile(False)
    eng.decode_step(None)
    torch.cuda.synchronize()
    assert eng.profile_read()["attn_dec"][1] == 0        # switched off: nothing recorded after the reset
    eng.close()


@pytest.mark.parametrize("name,rows,batch", [
    ("base_pruned_varlen", [0, 31, 63], 0),      # cfg 2, shortest batch (lengths 16..)
    ("base_pruned_varlen", [0, 40, 63], 7),      # cfg 2, longest batch (lengths ..256)
    ("large", [5, 127], 0),                      # cfg 3: 24 layers x 1024, batch 128, prompt 256, 64 tokens
    ("decode_bound", [17, 255], 0),              # cfg 4: batch 256, prompt 512, 128 tokens
])
def test_full_size_configs_sampled_rows(E, name, rows, batch):
    """The remaining benchmark configurations at full size; the oracle computes a sample of rows one by one."""
    wl = make_workload(name)
    sh = wl.shape
    eng = E.engine_from_workload(wl)
    ids, lens = wl.padded(batch)
    _say(f"[parity] {name} batch {batch} rows {rows} lens {[int(lens[r]) for r in rows]}")
    orc = oracle_generate(wl, batch, rows, sh.n_gen)
    forced = {r: orc[r]["tokens"] for r in orc}
    toks, hid, lg = gpu_generate(eng, ids, lens, sh.n_gen, forced)
    st = check_rows(orc, toks, hid, lg, name)
    _say(f"[parity] {name}: {st}")
    eng.close()


@pytest.mark.parametrize("batch,nw16", [(48, 2), (48, 0), (24, 0)])
def test_wide_model_on_the_small_batch_path(E, batch, nw16):
    """ERNIE-large widths (d = 1024, FFN 4096) at batch sizes that take the fused small-batch decode kernels: the
    activation tile of the second FFN GEMM then needs 8 (16 waves) or 16 (8 waves) pieces per thread, i.e. the
    straight-line first batch of loads plus, with 8 waves, the loop for the remainder."""
    wl = make_workload("large", n_layers=2, batch=batch, prompt_len=48, n_gen=4, vocab_full=4096, vocab_kept=2048)
    sh = wl.shape
    eng = E.engine_from_workload(wl)
    eng.tune("dec_nw16", nw16)
    ids, lens = wl.padded(0)
    rows = [0, batch // 2, batch - 1]
    _say(f"[parity] wide small-batch B={batch} dec_nw16={nw16} rows {rows}")
    orc = oracle_generate(wl, 0, rows, sh.n_gen)
    toks, hid, lg = gpu_generate(eng, ids, lens, sh.n_gen, {r: orc[r]["tokens"] for r in orc})
    st = check_rows(orc, toks, hid, lg, f"wide-B{batch}")
    _say(f"[parity] wide small-batch: {st}")
    eng.close()
