"""ctypes binding of the C ABI in include/ernie.h.

Argument marshalling only: every step of the hot path runs in the HIP
library.  PyTorch supplies device memory (tensors) and streams; no torch op
takes part in the computation.  If the library has not been built, loading
fails with an error -- there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np
import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libernie_hip.so")

ERNIE_OK, ERNIE_EINVAL, ERNIE_ECAPACITY, ERNIE_EARENA, ERNIE_ESEQUENCE, ERNIE_EHIP = 0, -1, -2, -3, -4, -5

EXPORTS = ("ernie_init_weights", "ernie_init_weights_ex", "ernie_prefill", "ernie_decode_step", "ernie_decode_step_static", "ernie_last_error", "ernie_free",
           "ernie_debug_buffer", "ernie_debug_tune", "ernie_debug_handover", "ernie_profile", "ernie_profile_read",
           "ernie_error_string", "ernie_get_config", "ernie_job_workspace_bytes", "ernie_run_job", "ernie_set_eos", "ernie_batch_state", "ernie_compact", "ernie_plan_batches",
           "ernie_vocab_count", "ernie_vocab_select", "ernie_vocab_gather_rows", "ernie_remap_ids")

PROF_CATEGORIES = ("gemm_dec", "gemm_dec_ln", "attn_dec", "gemm_prefill", "attn_prefill", "logits",
                   "row_dec", "row_prefill", "dec_persist")


class ErnieConfig(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32), ("d_ffn", C.c_int32),
                ("vocab_full", C.c_int32), ("vocab_kept", C.c_int32), ("max_pos", C.c_int32),
                ("max_batch", C.c_int32), ("max_seq", C.c_int32), ("ln_eps", C.c_float)]


_PP = C.POINTER(C.c_void_p)


class ErnieWeights(C.Structure):
    _fields_ = [("tok_emb_kept", C.c_void_p), ("kept_ids", C.c_void_p), ("pos_emb", C.c_void_p),
                ("emb_ln_g", C.c_void_p), ("emb_ln_b", C.c_void_p),
                ("wqkv", _PP), ("bqkv", _PP), ("wo", _PP), ("bo", _PP), ("ln1_g", _PP), ("ln1_b", _PP),
                ("w1", _PP), ("b1", _PP), ("w2", _PP), ("b2", _PP), ("ln2_g", _PP), ("ln2_b", _PP)]


class ErnieVariants(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("type_emb", "head_w", "head_b", "head_ln_g", "head_ln_b", "out_bias")]


VARIANT_KEYS = ("type_emb", "head_w", "head_b", "head_ln_g", "head_ln_b", "out_bias_kept")


class ErnieJob(C.Structure):
    _fields_ = [("n_requests", C.c_int32), ("prompt_offsets_host", C.POINTER(C.c_int32)),
                ("prompt_ids_host", C.POINTER(C.c_int32)), ("full_to_trimmed_host", C.POINTER(C.c_int32)),
                ("kept_ids_host", C.POINTER(C.c_int32)), ("n_gen", C.c_int32), ("max_batch", C.c_int32),
                ("max_tokens", C.c_int64), ("overlap", C.c_int32), ("workspace_dev", C.c_void_p),
                ("workspace_bytes", C.c_size_t), ("tokens_out_host", C.POINTER(C.c_int32))]


class ErnieJobStats(C.Structure):
    _fields_ = [("pre_s", C.c_double), ("enqueue_s", C.c_double), ("post_s", C.c_double), ("wall_s", C.c_double),
                ("n_batches", C.c_int32)]


class ErnieError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__(f"{what}: {error_string(code)} ({code})")


_lib = None


def load_library(path: Optional[str] = None) -> C.CDLL:
    """Load libernie_hip.so (built in-tree by paper_2407_04991_amd.build)."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    p = path or os.environ.get("ERNIE_HIP_LIB") or LIB_PATH     # the variable selects another build of the same library
    if not os.path.exists(p):
        raise FileNotFoundError(
            f"{p} not found: build it with `python -m paper_2407_04991_amd.build` (there is no CPU fallback)")
    lib = C.CDLL(p)
    lib.ernie_init_weights.restype = C.c_int
    lib.ernie_init_weights.argtypes = [C.POINTER(ErnieConfig), C.POINTER(ErnieWeights), C.c_void_p, C.c_size_t,
                                       C.POINTER(C.c_size_t), C.c_void_p, C.POINTER(C.c_void_p)]
    lib.ernie_init_weights_ex.restype = C.c_int
    lib.ernie_init_weights_ex.argtypes = [C.POINTER(ErnieConfig), C.POINTER(ErnieWeights), C.POINTER(ErnieVariants),
                                          C.c_void_p, C.c_size_t, C.POINTER(C.c_size_t), C.c_void_p,
                                          C.POINTER(C.c_void_p)]
    lib.ernie_prefill.restype = C.c_int
    lib.ernie_prefill.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.POINTER(C.c_int32),
                                  C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.ernie_decode_step.restype = C.c_int
    lib.ernie_decode_step.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.ernie_decode_step_static.restype = C.c_int
    lib.ernie_decode_step_static.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.ernie_last_error.restype = C.c_int
    lib.ernie_last_error.argtypes = [C.c_void_p]
    lib.ernie_free.restype = None
    lib.ernie_free.argtypes = [C.c_void_p]
    lib.ernie_debug_buffer.restype = C.c_int
    lib.ernie_debug_buffer.argtypes = [C.c_void_p, C.c_char_p, C.POINTER(C.c_void_p), C.POINTER(C.c_size_t)]
    lib.ernie_debug_tune.restype = C.c_int
    lib.ernie_debug_tune.argtypes = [C.c_void_p, C.c_char_p, C.c_int]
    lib.ernie_debug_handover.restype = C.c_int
    lib.ernie_debug_handover.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_size_t, C.c_void_p,
                                         C.POINTER(C.c_double), C.POINTER(C.c_int64)]
    lib.ernie_profile.restype = C.c_int
    lib.ernie_profile.argtypes = [C.c_void_p, C.c_int]
    lib.ernie_profile_read.restype = C.c_int
    lib.ernie_profile_read.argtypes = [C.c_void_p, C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_int64),
                                       C.POINTER(C.c_double), C.POINTER(C.c_double)]
    lib.ernie_error_string.restype = C.c_char_p
    lib.ernie_error_string.argtypes = [C.c_int]
    lib.ernie_get_config.restype = C.c_int
    lib.ernie_get_config.argtypes = [C.c_void_p, C.POINTER(ErnieConfig)]
    lib.ernie_job_workspace_bytes.restype = C.c_size_t
    lib.ernie_job_workspace_bytes.argtypes = [C.c_void_p, C.c_int32]
    lib.ernie_run_job.restype = C.c_int
    lib.ernie_run_job.argtypes = [C.c_void_p, C.POINTER(ErnieJob), C.POINTER(ErnieJobStats), C.c_void_p]
    lib.ernie_set_eos.restype = C.c_int
    lib.ernie_set_eos.argtypes = [C.c_void_p, C.c_int32]
    lib.ernie_batch_state.restype = C.c_int
    lib.ernie_batch_state.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.ernie_compact.restype = C.c_int
    lib.ernie_compact.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_int32), C.c_void_p]
    lib.ernie_plan_batches.restype = C.c_int
    lib.ernie_plan_batches.argtypes = [C.POINTER(C.c_int32), C.c_int32, C.c_int32, C.c_int64, C.POINTER(C.c_int32),
                                       C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
    lib.ernie_vocab_count.restype = C.c_int
    lib.ernie_vocab_count.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_void_p]
    lib.ernie_vocab_select.restype = C.c_int
    lib.ernie_vocab_select.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(C.c_int32), C.c_int32, C.c_int32,
                                       C.c_void_p, C.c_void_p, C.c_void_p]
    lib.ernie_vocab_gather_rows.restype = C.c_int
    lib.ernie_vocab_gather_rows.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p,
                                            C.c_void_p]
    lib.ernie_remap_ids.restype = C.c_int
    lib.ernie_remap_ids.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
    if path is None:
        _lib = lib
    return lib


def error_string(code: int) -> str:
    return load_library().ernie_error_string(int(code)).decode()


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream_ptr(stream: Optional[torch.cuda.Stream]) -> Optional[int]:
    s = stream if stream is not None else torch.cuda.current_stream()
    return s.cuda_stream or None


# ---- thin wrappers with the C names -----------------------------------------

def ernie_init_weights(cfg: ErnieConfig, weights: Optional[ErnieWeights], arena: Optional[torch.Tensor],
                       stream=None):
    """Returns (rc, arena_needed, handle)."""
    lib = load_library()
    need = C.c_size_t(0)
    out = C.c_void_p(None)
    rc = lib.ernie_init_weights(C.byref(cfg), C.byref(weights) if weights is not None else None,
                                _ptr(arena), arena.numel() if arena is not None else 0, C.byref(need),
                                _stream_ptr(stream) if arena is not None else None, C.byref(out))
    return rc, need.value, out.value


def ernie_init_weights_ex(cfg: ErnieConfig, weights: Optional[ErnieWeights], variants: Optional[ErnieVariants],
                          arena: Optional[torch.Tensor], stream=None):
    """Returns (rc, arena_needed, handle)."""
    lib = load_library()
    need = C.c_size_t(0)
    out = C.c_void_p(None)
    rc = lib.ernie_init_weights_ex(C.byref(cfg), C.byref(weights) if weights is not None else None,
                                   C.byref(variants) if variants is not None else None,
                                   _ptr(arena), arena.numel() if arena is not None else 0, C.byref(need),
                                   _stream_ptr(stream) if arena is not None else None, C.byref(out))
    return rc, need.value, out.value


def ernie_prefill(handle, B: int, Lmax: int, ids_dev: torch.Tensor, prompt_lens_host: np.ndarray,
                  logits_out: Optional[torch.Tensor], hidden_out: Optional[torch.Tensor], tok_out: torch.Tensor,
                  stream=None) -> int:
    lens = np.ascontiguousarray(prompt_lens_host, dtype=np.int32)
    return load_library().ernie_prefill(handle, B, Lmax, _ptr(ids_dev), lens.ctypes.data_as(C.POINTER(C.c_int32)),
                                        _ptr(logits_out), _ptr(hidden_out), _ptr(tok_out), _stream_ptr(stream))


def ernie_decode_step(handle, tok_in: Optional[torch.Tensor], logits_out: Optional[torch.Tensor],
                      hidden_out: Optional[torch.Tensor], tok_out: torch.Tensor, stream=None) -> int:
    return load_library().ernie_decode_step(handle, _ptr(tok_in), _ptr(logits_out), _ptr(hidden_out),
                                            _ptr(tok_out), _stream_ptr(stream))


def ernie_decode_step_static(handle, tok_in: Optional[torch.Tensor], logits_out: Optional[torch.Tensor],
                             hidden_out: Optional[torch.Tensor], tok_out: torch.Tensor, stream=None) -> int:
    return load_library().ernie_decode_step_static(handle, _ptr(tok_in), _ptr(logits_out), _ptr(hidden_out),
                                                   _ptr(tok_out), _stream_ptr(stream))


def ernie_last_error(handle) -> int:
    return load_library().ernie_last_error(handle)


def ernie_debug_handover(mode: int, n_workgroups: int, stages: int, pieces: int, out_units: int, ws: torch.Tensor,
                         stream=None):
    """Returns (rc, microseconds per stage, units with a wrong payload)."""
    us, bad = C.c_double(0.0), C.c_int64(0)
    rc = load_library().ernie_debug_handover(mode, n_workgroups, stages, pieces, out_units, _ptr(ws), ws.numel(),
                                             _stream_ptr(stream), C.byref(us), C.byref(bad))
    return rc, us.value, bad.value


def ernie_free(handle) -> None:
    load_library().ernie_free(handle)


def ernie_get_config(handle):
    """Returns (rc, ErnieConfig)."""
    cfg = ErnieConfig()
    return load_library().ernie_get_config(handle, C.byref(cfg)), cfg


def ernie_job_workspace_bytes(handle, n_gen: int) -> int:
    return load_library().ernie_job_workspace_bytes(handle, int(n_gen))


def ernie_run_job(handle, prompts_full, full_to_trimmed_host, kept_ids_host, n_gen: int, max_batch: int,
                  max_tokens: int, overlap: bool, workspace: Optional[torch.Tensor], stream=None):
    """Marshals a list of int32 prompt arrays into the ragged layout of ErnieJob and runs it.
    Returns (rc, tokens [n_requests, n_gen] int32 full ids, ErnieJobStats)."""
    n = len(prompts_full)
    offs = np.zeros(n + 1, dtype=np.int32)
    offs[1:] = np.cumsum([len(q) for q in prompts_full])
    flat = np.ascontiguousarray(np.concatenate(prompts_full) if n else np.zeros(0), dtype=np.int32)
    fmap = np.ascontiguousarray(full_to_trimmed_host, dtype=np.int32)
    kept = np.ascontiguousarray(kept_ids_host, dtype=np.int32)
    out = np.zeros((n, n_gen), dtype=np.int32)
    P32 = C.POINTER(C.c_int32)
    job = ErnieJob(n, offs.ctypes.data_as(P32), flat.ctypes.data_as(P32), fmap.ctypes.data_as(P32),
                   kept.ctypes.data_as(P32), int(n_gen), int(max_batch), int(max_tokens), int(bool(overlap)),
                   _ptr(workspace), workspace.numel() if workspace is not None else 0, out.ctypes.data_as(P32))
    stats = ErnieJobStats()
    rc = load_library().ernie_run_job(handle, C.byref(job), C.byref(stats), _stream_ptr(stream))
    return rc, out, stats


def ernie_set_eos(handle, eos_id: int) -> int:
    return load_library().ernie_set_eos(handle, int(eos_id))


def ernie_batch_state(handle, lens_out: Optional[torch.Tensor], finished_out: Optional[torch.Tensor], stream=None) -> int:
    return load_library().ernie_batch_state(handle, _ptr(lens_out), _ptr(finished_out), _stream_ptr(stream))


def ernie_compact(handle, keep_rows_host, stream=None) -> int:
    keep = np.ascontiguousarray(keep_rows_host, dtype=np.int32)
    return load_library().ernie_compact(handle, keep.size, keep.ctypes.data_as(C.POINTER(C.c_int32)),
                                        _stream_ptr(stream))


def ernie_plan_batches(lens_host, max_batch: int, max_tokens: int):
    """Host-only.  Returns (rc, order [n], starts [n_batches + 1])."""
    lens = np.ascontiguousarray(lens_host, dtype=np.int32)
    n = lens.size
    order = np.zeros(max(n, 1), dtype=np.int32)
    starts = np.zeros(n + 1, dtype=np.int32)
    nb = C.c_int32(0)
    rc = load_library().ernie_plan_batches(lens.ctypes.data_as(C.POINTER(C.c_int32)), n, int(max_batch), int(max_tokens),
                                           order.ctypes.data_as(C.POINTER(C.c_int32)),
                                           starts.ctypes.data_as(C.POINTER(C.c_int32)), C.byref(nb))
    return rc, order[:n], starts[:nb.value + 1]


# ---- vocabulary trimming (include/ernie_prune.h) ------------------------------

def ernie_vocab_count(ids_dev: Optional[torch.Tensor], n: int, vocab_full: int, counts_dev: Optional[torch.Tensor],
                      stream=None) -> int:
    """counts_dev: int64 tensor viewed as uint64 bins (torch has no unsigned 64-bit arithmetic; the bits are the same)."""
    return load_library().ernie_vocab_count(_ptr(ids_dev), n, vocab_full, _ptr(counts_dev), _stream_ptr(stream))


def ernie_vocab_select(counts_dev, vocab_full: int, k: int, reserved_host, unk_full_id: int, kept_ids_dev,
                       full_to_trimmed_dev, stream=None) -> int:
    res = None if reserved_host is None else np.ascontiguousarray(reserved_host, dtype=np.int32)
    return load_library().ernie_vocab_select(_ptr(counts_dev), vocab_full, k,
                                             None if res is None else res.ctypes.data_as(C.POINTER(C.c_int32)),
                                             0 if res is None else res.size, unk_full_id, _ptr(kept_ids_dev),
                                             _ptr(full_to_trimmed_dev), _stream_ptr(stream))


def ernie_vocab_gather_rows(table_full_dev, vocab_full: int, d: int, kept_ids_dev, k: int, table_kept_dev,
                            stream=None) -> int:
    return load_library().ernie_vocab_gather_rows(_ptr(table_full_dev), vocab_full, d, _ptr(kept_ids_dev), k,
                                                  _ptr(table_kept_dev), _stream_ptr(stream))


def ernie_remap_ids(in_dev, n: int, map_dev, map_len: int, fallback: int, out_dev, stream=None) -> int:
    return load_library().ernie_remap_ids(_ptr(in_dev), n, _ptr(map_dev), map_len, fallback, _ptr(out_dev),
                                          _stream_ptr(stream))


def _check(rc: int, what: str):
    if rc != ERNIE_OK:
        raise ErnieError(rc, what)


class VocabTrimmer:
    """Buffers + call sequence of the trimming step; every result is computed by the library's kernels.

    count(ids) may be called any number of times (a corpus streamed in pieces);
    select(k, reserved, unk) then fixes kept_ids [k] and full_to_trimmed [V] on the device.
    """

    def __init__(self, vocab_full: int, device="cuda:0"):
        load_library()
        self.V = int(vocab_full)
        self.device = torch.device(device)
        self.counts = torch.zeros(self.V, dtype=torch.int64, device=self.device)
        self.kept_ids = None
        self.full_to_trimmed = torch.empty(self.V, dtype=torch.int32, device=self.device)
        self.unk_trimmed = None

    def count(self, ids: torch.Tensor, stream=None):
        assert ids.dtype == torch.int32 and ids.is_contiguous() and ids.device == self.device
        _check(ernie_vocab_count(ids, ids.numel(), self.V, self.counts, stream), "ernie_vocab_count")

    def select(self, k: int, reserved, unk_full_id: int, stream=None):
        self.kept_ids = torch.empty(int(k), dtype=torch.int32, device=self.device)
        _check(ernie_vocab_select(self.counts, self.V, int(k), reserved, int(unk_full_id), self.kept_ids,
                                  self.full_to_trimmed, stream), "ernie_vocab_select")
        self.unk_full, self.unk_trimmed = int(unk_full_id), None
        return self.kept_ids

    def trim_table(self, table_full: torch.Tensor, stream=None) -> torch.Tensor:
        assert table_full.dtype == torch.float16 and table_full.is_contiguous() and table_full.shape[0] == self.V
        k, d = self.kept_ids.numel(), table_full.shape[1]
        out = torch.empty((k, d), dtype=torch.float16, device=self.device)
        _check(ernie_vocab_gather_rows(table_full, self.V, d, self.kept_ids, k, out, stream), "ernie_vocab_gather_rows")
        return out

    def to_trimmed(self, ids_full: torch.Tensor, stream=None) -> torch.Tensor:
        """Full -> trimmed ids; dropped and out-of-range ids become the unknown-word row."""
        if self.unk_trimmed is None:
            self.unk_trimmed = int(self.full_to_trimmed[self.unk_full].item())
        out = torch.empty_like(ids_full)
        _check(ernie_remap_ids(ids_full, ids_full.numel(), self.full_to_trimmed, self.V, self.unk_trimmed, out, stream),
               "ernie_remap_ids")
        return out

    def to_full(self, ids_trimmed: torch.Tensor, stream=None) -> torch.Tensor:
        out = torch.empty_like(ids_trimmed)
        _check(ernie_remap_ids(ids_trimmed, ids_trimmed.numel(), self.kept_ids, self.kept_ids.numel(), -1, out, stream),
               "ernie_remap_ids")
        return out


# ---- convenience object ------------------------------------------------------

_LAYER_KEYS = ("wqkv", "bqkv", "wo", "bo", "ln1_g", "ln1_b", "w1", "b1", "w2", "b2", "ln2_g", "ln2_b")


class ErnieEngine:
    """Owns the arena tensor and the handle; forwards to the C entry points.

    `weights` is a dict of numpy/torch fp16 arrays laid out as the synthetic
    generator produces them, with the token table ALREADY trimmed to the kept
    rows under key "tok_emb_kept".  Optional variants are switched on by the
    keys "type_emb", "head_w" + "head_b" + "head_ln_g" + "head_ln_b", and
    "out_bias_kept" (the output bias already gathered to the kept rows).
    """

    def __init__(self, *, n_layers, d_model, n_heads, d_ffn, vocab_full, vocab_kept, max_pos, max_batch, max_seq,
                 ln_eps, weights: dict, kept_ids, device="cuda:0"):
        if not torch.cuda.is_available():
            raise RuntimeError("ErnieEngine needs a GPU: the HIP library is the only implementation")
        self.device = torch.device(device)
        self.cfg = ErnieConfig(n_layers, d_model, n_heads, d_ffn, vocab_full, vocab_kept, max_pos, max_batch,
                               max_seq, ln_eps)
        self.handle = None
        var = None
        if any(weights.get(k) is not None for k in VARIANT_KEYS):
            var = ErnieVariants()
            for k in VARIANT_KEYS:          # the size query looks at NULL-ness only
                setattr(var, k.replace("_kept", ""), 1 if weights.get(k) is not None else None)
        rc, need, _ = ernie_init_weights_ex(self.cfg, None, var, None)
        if rc != ERNIE_OK:
            raise ErnieError(rc, "ernie_init_weights_ex(size query)")
        self.arena_bytes = need
        self.arena = torch.empty(need, dtype=torch.uint8, device=self.device)
        assert self.arena.data_ptr() % 256 == 0

        def dev(a, dtype=torch.float16):
            t = torch.as_tensor(np.ascontiguousarray(a)) if not isinstance(a, torch.Tensor) else a
            return t.to(device=self.device, dtype=dtype).contiguous()

        keep = []       # device originals stay alive until the repack has run
        w = ErnieWeights()
        for name, key, dt in (("tok_emb_kept", "tok_emb_kept", torch.float16), ("pos_emb", "pos_emb", torch.float16),
                              ("emb_ln_g", "emb_ln_g", torch.float16), ("emb_ln_b", "emb_ln_b", torch.float16)):
            t = dev(weights[key], dt); keep.append(t); setattr(w, name, t.data_ptr())
        t = dev(kept_ids, torch.int32); keep.append(t); w.kept_ids = t.data_ptr()
        arrays = {}
        for k in _LAYER_KEYS:
            arr = (C.c_void_p * n_layers)()
            for l in range(n_layers):
                t = dev(weights["layers"][l][k]); keep.append(t); arr[l] = t.data_ptr()
            arrays[k] = arr
            setattr(w, k, C.cast(arr, _PP))
        if var is not None:
            for k in VARIANT_KEYS:
                if weights.get(k) is not None:
                    t = dev(weights[k]); keep.append(t); setattr(var, k.replace("_kept", ""), t.data_ptr())
        rc, _, handle = ernie_init_weights_ex(self.cfg, w, var, self.arena)
        if rc != ERNIE_OK:
            raise ErnieError(rc, "ernie_init_weights_ex")
        torch.cuda.synchronize(self.device)
        del keep
        self.handle = handle
        self.B = 0

    # outputs are allocated by the caller-side helper, never by the library
    def prefill(self, ids: torch.Tensor, lens, *, logits=False, hidden=False, stream=None):
        B, Lmax = ids.shape
        ids = ids.to(device=self.device, dtype=torch.int32).contiguous()
        lo = torch.empty(B, self.cfg.vocab_kept, dtype=torch.float32, device=self.device) if logits else None
        ho = torch.empty(B, self.cfg.d_model, dtype=torch.float32, device=self.device) if hidden else None
        tok = torch.empty(B, dtype=torch.int32, device=self.device)
        rc = ernie_prefill(self.handle, B, Lmax, ids, np.asarray(lens, dtype=np.int32), lo, ho, tok, stream)
        if rc != ERNIE_OK:
            raise ErnieError(rc, "ernie_prefill")
        self.B = B
        return tok, lo, ho

    def decode_step(self, tok_in: Optional[torch.Tensor] = None, *, logits=False, hidden=False, stream=None,
                    out=None, static=False):
        B = self.B
        if tok_in is not None:
            tok_in = tok_in.to(device=self.device, dtype=torch.int32).contiguous()
        if out is None:
            lo = torch.empty(B, self.cfg.vocab_kept, dtype=torch.float32, device=self.device) if logits else None
            ho = torch.empty(B, self.cfg.d_model, dtype=torch.float32, device=self.device) if hidden else None
            tok = torch.empty(B, dtype=torch.int32, device=self.device)
        else:
            tok, lo, ho = out
        fn = ernie_decode_step_static if static else ernie_decode_step
        rc = fn(self.handle, tok_in, lo, ho, tok, stream)
        if rc != ERNIE_OK:
            raise ErnieError(rc, fn.__name__)
        return tok, lo, ho

    def set_eos(self, eos_id: int):
        _check(ernie_set_eos(self.handle, eos_id), "ernie_set_eos")

    def state(self):
        """(cached lengths, finished flags) of the batch in flight, as device int32 tensors."""
        lens = torch.empty(self.B, dtype=torch.int32, device=self.device)
        fin = torch.empty(self.B, dtype=torch.int32, device=self.device)
        _check(ernie_batch_state(self.handle, lens, fin), "ernie_batch_state")
        return lens, fin

    def compact(self, keep_rows):
        _check(ernie_compact(self.handle, keep_rows), "ernie_compact")
        self.B = len(keep_rows)

    def debug_buffer(self, name: str):
        ptr = C.c_void_p(None); n = C.c_size_t(0)
        rc = load_library().ernie_debug_buffer(self.handle, name.encode(), C.byref(ptr), C.byref(n))
        if rc != ERNIE_OK:
            raise ErnieError(rc, "ernie_debug_buffer")
        return ptr.value, n.value

    def profile(self, enable: bool):
        rc = load_library().ernie_profile(self.handle, int(bool(enable)))
        if rc != ERNIE_OK:
            raise ErnieError(rc, "ernie_profile")

    def profile_read(self) -> dict:
        """{category: (total_ms, launches, algorithmic bytes, algorithmic flops)} of the profiled launches."""
        out = {}
        for i, name in enumerate(PROF_CATEGORIES):
            ms, n, by, fl = C.c_double(0), C.c_int64(0), C.c_double(0), C.c_double(0)
            rc = load_library().ernie_profile_read(self.handle, i, C.byref(ms), C.byref(n), C.byref(by), C.byref(fl))
            if rc != ERNIE_OK:
                raise ErnieError(rc, "ernie_profile_read")
            out[name] = (ms.value, n.value, by.value, fl.value)
        return out

    def tune(self, key: str, value: int):
        rc = load_library().ernie_debug_tune(self.handle, key.encode(), int(value))
        if rc != ERNIE_OK:
            raise ErnieError(rc, f"ernie_debug_tune({key}, {value})")

    def close(self):
        if self.handle is not None:
            ernie_free(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def engine_from_workload(wl, *, max_batch=None, max_seq=None, device="cuda:0") -> ErnieEngine:
    """Engine for a synthetic workload object (shape, weights, kept_ids)."""
    sh = wl.shape
    weights = dict(wl.weights)
    weights["tok_emb_kept"] = np.ascontiguousarray(wl.weights["tok_emb"][wl.kept_ids])
    if wl.weights.get("out_bias") is not None:
        weights["out_bias_kept"] = np.ascontiguousarray(wl.weights["out_bias"][wl.kept_ids])
    return ErnieEngine(n_layers=sh.n_layers, d_model=sh.d_model, n_heads=sh.n_heads, d_ffn=sh.d_ffn,
                       vocab_full=sh.vocab_full, vocab_kept=sh.vocab_kept, max_pos=sh.max_pos,
                       max_batch=max_batch or sh.batch, max_seq=max_seq or (sh.prompt_len + sh.n_gen),
                       ln_eps=sh.ln_eps, weights=weights, kept_ids=wl.kept_ids, device=device)
