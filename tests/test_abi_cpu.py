"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
declared symbol, sizes the arena and rejects bad configurations before any device call."""
import ctypes as C
import os
import re

import pytest

import paper_2407_04991_amd as E

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = "".join(open(os.path.join(ROOT, "include", f)).read()
                   for f in sorted(os.listdir(os.path.join(ROOT, "include"))) if f.endswith(".h"))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ernie_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = E.load_library()
    names = declared_symbols()
    assert set(names) == set(E.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_library_exports_nothing_else():
    """Hidden visibility: the dynamic symbol table defines the declared entry points and no other function or object
    (no kernel stubs, no helpers)."""
    import subprocess
    from paper_2407_04991_amd import binding
    out = subprocess.run(["nm", "-D", "--defined-only", binding.LIB_PATH], capture_output=True, text=True, check=True).stdout
    defined = {line.split()[-1] for line in out.splitlines() if line.strip()}
    assert defined == set(declared_symbols()), sorted(defined ^ set(declared_symbols()))


def base_cfg(**kw):
    v = dict(n_layers=12, d_model=768, n_heads=12, d_ffn=3072, vocab_full=18000, vocab_kept=18000, max_pos=512,
             max_batch=32, max_seq=160, ln_eps=1e-5)
    v.update(kw)
    return E.ErnieConfig(*[v[k] for k in ("n_layers", "d_model", "n_heads", "d_ffn", "vocab_full", "vocab_kept",
                                          "max_pos", "max_batch", "max_seq", "ln_eps")])


def test_size_query_counts_cache_and_weights():
    rc, need, handle = E.ernie_init_weights(base_cfg(), None, None)
    assert rc == E.ERNIE_OK and handle is None
    kv = 12 * 2 * 32 * 160 * 768 * 2
    weights = 12 * (4 * 768 * 768 + 2 * 768 * 3072) * 2 + 2 * 18000 * 768 * 2
    assert need >= kv + weights
    rc2, need2, _ = E.ernie_init_weights(base_cfg(max_seq=320), None, None)
    assert rc2 == E.ERNIE_OK and need2 - need >= kv          # cache doubles (activations grow too)


@pytest.mark.parametrize("kw", [
    dict(n_heads=11),                  # head_dim != 64
    dict(d_model=0), dict(n_layers=0), dict(d_ffn=100), dict(vocab_kept=0),
    dict(vocab_kept=18001),            # more kept rows than the full table
    dict(max_batch=0), dict(max_batch=257), dict(max_seq=0), dict(max_pos=0), dict(ln_eps=0.0),
    dict(d_model=8192, n_heads=128),   # wider than one wave normalises
])
def test_bad_config_is_einval(kw):
    rc, need, _ = E.ernie_init_weights(base_cfg(**kw), None, None)
    assert rc == E.ERNIE_EINVAL


def test_null_arguments_are_rejected_on_the_host():
    lib = E.load_library()
    assert lib.ernie_init_weights(None, None, None, 0, None, None, None) == E.ERNIE_EINVAL
    cfg = base_cfg()
    assert lib.ernie_init_weights(C.byref(cfg), None, None, 0, None, None, None) == E.ERNIE_EINVAL  # nowhere to write the size
    assert lib.ernie_prefill(None, 1, 1, None, None, None, None, None, None) == E.ERNIE_EINVAL
    assert lib.ernie_decode_step(None, None, None, None, None, None) == E.ERNIE_EINVAL
    assert lib.ernie_decode_step_static(None, None, None, None, None, None) == E.ERNIE_EINVAL
    lib.ernie_free(None)     # no-op
    assert lib.ernie_profile(None, 1) == E.ERNIE_EINVAL
    assert lib.ernie_debug_tune(None, b"sk_out", 1) == E.ERNIE_EINVAL
    ms = C.c_double(); cnt = C.c_int64()
    assert lib.ernie_profile_read(None, 0, C.byref(ms), C.byref(cnt), None, None) == E.ERNIE_EINVAL
    out = C.c_void_p(); n = C.c_size_t()
    assert lib.ernie_debug_buffer(None, b"x", C.byref(out), C.byref(n)) == E.ERNIE_EINVAL


def test_error_strings():
    assert E.error_string(0) == "ok"
    for code in (-1, -2, -3, -4, -5):
        assert E.error_string(code) not in ("ok", "unknown error")
    assert E.error_string(-99) == "unknown error"


def test_trimming_entry_points_reject_bad_arguments_before_any_device_call():
    """ernie_prune.h: every ERNIE_EINVAL is decided on the host, so these calls are safe without a GPU
    (the fake addresses are never dereferenced)."""
    lib = E.load_library()
    fake, odd = 0x10000, 0x10002
    res = (C.c_int32 * 2)(3, 4)
    assert lib.ernie_vocab_count(None, 5, 100, fake, None) == E.ERNIE_EINVAL          # NULL stream of ids
    assert lib.ernie_vocab_count(fake, 5, 100, None, None) == E.ERNIE_EINVAL          # NULL bins
    assert lib.ernie_vocab_count(odd, 5, 100, fake, None) == E.ERNIE_EINVAL           # misaligned ids
    assert lib.ernie_vocab_count(fake, 5, 100, fake + 4, None) == E.ERNIE_EINVAL      # misaligned bins
    assert lib.ernie_vocab_count(fake, 5, 0, fake, None) == E.ERNIE_EINVAL
    assert lib.ernie_vocab_count(fake, 5, 262145, fake, None) == E.ERNIE_EINVAL
    assert lib.ernie_vocab_count(fake, -1, 100, fake, None) == E.ERNIE_EINVAL
    assert lib.ernie_vocab_count(fake, (1 << 40) + 1, 100, fake, None) == E.ERNIE_EINVAL
    assert lib.ernie_vocab_select(None, 100, 10, res, 2, 3, fake, fake, None) == E.ERNIE_EINVAL
    assert lib.ernie_vocab_select(fake, 100, 10, None, 2, 3, fake, fake, None) == E.ERNIE_EINVAL
    assert lib.ernie_vocab_select(fake, 100, 0, res, 2, 3, fake, fake, None) == E.ERNIE_EINVAL
    assert lib.ernie_vocab_select(fake, 100, 101, res, 2, 3, fake, fake, None) == E.ERNIE_EINVAL
    assert lib.ernie_vocab_select(fake, 100, 1, res, 2, 3, fake, fake, None) == E.ERNIE_EINVAL    # more reserved than k
    assert lib.ernie_vocab_select(fake, 100, 10, res, 2, 5, fake, fake, None) == E.ERNIE_EINVAL   # unk not reserved
    assert lib.ernie_vocab_select(fake, 4, 3, res, 2, 3, fake, fake, None) == E.ERNIE_EINVAL      # reserved id 4 >= V
    assert lib.ernie_vocab_gather_rows(None, 100, 64, fake, 10, fake, None) == E.ERNIE_EINVAL
    assert lib.ernie_vocab_gather_rows(fake, 100, 60, fake, 10, fake, None) == E.ERNIE_EINVAL     # d % 8 != 0
    assert lib.ernie_vocab_gather_rows(fake, 100, 64, fake, 10, fake + 8, None) == E.ERNIE_EINVAL  # misaligned table
    assert lib.ernie_vocab_gather_rows(fake, 100, 64, fake, 0, fake, None) == E.ERNIE_EINVAL
    assert lib.ernie_remap_ids(fake, 5, None, 10, 0, fake, None) == E.ERNIE_EINVAL
    assert lib.ernie_remap_ids(fake, 5, fake, 0, 0, fake, None) == E.ERNIE_EINVAL
    assert lib.ernie_remap_ids(None, 5, fake, 10, 0, fake, None) == E.ERNIE_EINVAL
    assert lib.ernie_remap_ids(fake, -1, fake, 10, 0, fake, None) == E.ERNIE_EINVAL
    assert lib.ernie_remap_ids(None, 0, fake, 10, 0, None, None) == E.ERNIE_OK                    # empty stream: no-op
    assert lib.ernie_vocab_count(None, 0, 100, fake, None) == E.ERNIE_OK


def test_variant_size_query_and_partial_head():
    """ernie_init_weights_ex: each optional variant adds its repacked parameters to the arena; the four head
    parameters come together or not at all (only NULL-ness matters for the size query)."""
    cfg = base_cfg()
    rc, plain, _ = E.ernie_init_weights_ex(cfg, None, None, None)
    assert rc == E.ERNIE_OK and plain == E.ernie_init_weights(cfg, None, None)[1]
    d, V = 768, 18000
    for fields, extra in [(("type_emb",), 2 * d * 2), (("out_bias",), V * 4),
                          (("head_w", "head_b", "head_ln_g", "head_ln_b"), d * d * 2 + 3 * d * 4)]:
        var = E.ErnieVariants()
        for f in fields:
            setattr(var, f, 0x1000)
        rc, need, _ = E.ernie_init_weights_ex(cfg, None, var, None)
        assert rc == E.ERNIE_OK and extra <= need - plain <= extra + 6 * 256, (fields, need - plain)
    var = E.ErnieVariants()
    var.head_w = 0x1000; var.head_b = 0x1000
    assert E.ernie_init_weights_ex(cfg, None, var, None)[0] == E.ERNIE_EINVAL


def test_batch_planning_matches_the_oracle_bit_for_bit():
    """ernie_plan_batches is host-only C++: compared with oracle/schedule_oracle.py on random and edge inputs."""
    import numpy as np
    from oracle import schedule_oracle as S
    rng = np.random.default_rng(0)
    cases = [([5, 2, 9, 2, 7, 3, 9], 3, 16), ([1], 1, 1), ([], 4, 10), ([7] * 50, 8, 10 ** 9)]
    for _ in range(40):
        n = int(rng.integers(1, 300))
        cases.append((rng.integers(1, 257, size=n).tolist(), int(rng.integers(1, 65)), int(rng.integers(256, 5000))))
    for lens, mb, mt in cases:
        rc, order, starts = E.ernie_plan_batches(lens, mb, mt)
        o, s = S.plan_batches(lens, mb, mt)
        assert rc == E.ERNIE_OK and np.array_equal(order, o) and np.array_equal(starts, s), (lens[:8], mb, mt)
    for lens, mb, mt in [([3, 0], 4, 10), ([3], 0, 10), ([3], 4, 0), ([11], 4, 10)]:
        assert E.ernie_plan_batches(lens, mb, mt)[0] == E.ERNIE_EINVAL
    lib = E.load_library()
    assert lib.ernie_plan_batches(None, 3, 4, 10, None, None, None) == E.ERNIE_EINVAL
    assert lib.ernie_set_eos(None, 0) == E.ERNIE_EINVAL
    assert lib.ernie_compact(None, 1, None, None) == E.ERNIE_EINVAL
    assert lib.ernie_batch_state(None, None, None, None) == E.ERNIE_EINVAL


def test_job_entry_points_reject_null_handles():
    lib = E.load_library()
    assert lib.ernie_job_workspace_bytes(None, 4) == 0
    assert lib.ernie_get_config(None, None) == E.ERNIE_EINVAL
    assert lib.ernie_run_job(None, None, None, None) == E.ERNIE_EINVAL


def test_missing_library_and_missing_gpu_fail_loudly(tmp_path):
    """There is no CPU fallback: a missing shared library raises on load, and without a GPU the engine refuses to start."""
    import torch
    from synth import make_workload
    with pytest.raises(FileNotFoundError, match="no CPU fallback"):
        E.load_library(str(tmp_path / "libernie_hip_absent.so"))
    if not torch.cuda.is_available():
        with pytest.raises(RuntimeError, match="needs a GPU"):
            E.engine_from_workload(make_workload("tiny"))
