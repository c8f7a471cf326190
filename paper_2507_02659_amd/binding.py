"""ctypes binding of libotverify.so: same entry points as include/otverify.h, argument marshalling only.

Every step of the verification path runs in the library's HIP kernels.  There is no fallback: if the shared
library has not been built, importing a symbol raises with the build command.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libotverify.so")

OT_OK = 0
OT_ERR_NULL, OT_ERR_SHAPE, OT_ERR_DTYPE, OT_ERR_MAP = -1, -2, -3, -4
OT_ERR_NGRAM, OT_ERR_CTX_MISMATCH, OT_ERR_HIP, OT_ERR_NOMEM = -5, -6, -7, -8
OT_BF16, OT_F32 = 0, 1
OT_FLAG_UNMAPPABLE, OT_FLAG_RESID_ZERO, OT_FLAG_BAD_ID = 1, 2, 4
OT_MAX_NGRAM_LEN, OT_MAX_K = 8, 63
OT_STATIC_MAX_BATCH = 4096
OT_N_STAGES = 4
STAGE_NAMES = ("lm_head", "softmax_stats", "translate_accept", "residual_draw")

OT_EVICT_NONE, OT_EVICT_LRU, OT_EVICT_LFU = 0, 1, 2
OT_DRAFT_SIDE_AUTO, OT_DRAFT_SIDE_IN_LM_HEAD, OT_DRAFT_SIDE_SEPARATE = 0, 1, 2
OT_LAMBDA_FIXED, OT_LAMBDA_TARGET_PROB = 0, 1
OT_NGRAM_TERM_NLL, OT_NGRAM_TERM_APPROX_KL = 0, 1

EXPORTS = (
    "ot_verify_init", "ot_verify_destroy", "ot_ngram_cache_build", "ot_ngram_cache_create", "ot_ngram_cache_insert",
    "ot_ngram_cache_size", "ot_ngram_cache_export", "ot_ngram_cache_import", "ot_ngram_cache_destroy", "ot_verify_step",
    "ot_verify_step_from_logits", "ot_distill_loss", "ot_adaptive_drafting", "ot_adaptive_drafting_static", "ot_verify_workspace", "ot_verify_profile",
    "ot_verify_profile_read", "ot_last_error", "ot_version",
)


class OtError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"otverify error {code}: {message}")
        self.code = code
        self.message = message


class ot_verify_config(C.Structure):
    _fields_ = [
        ("d", C.c_int32), ("V_t", C.c_int32), ("V_d", C.c_int32), ("max_batch", C.c_int32), ("max_k", C.c_int32),
        ("dtype", C.c_int32), ("max_ngram_len", C.c_int32), ("draft_side", C.c_int32),
        ("W", C.c_void_p), ("direct_map", C.c_void_p), ("stream", C.c_void_p),
    ]


class ot_step_in(C.Structure):
    _fields_ = [
        ("B", C.c_int32), ("step", C.c_uint32),
        ("row_off", C.c_void_p), ("row_off_host", C.c_void_p), ("hidden", C.c_void_p), ("draft_logits", C.c_void_p),
        ("draft_ids", C.c_void_p), ("temperature", C.c_void_p), ("draft_temperature", C.c_void_p),
        ("seq_id", C.c_void_p), ("seed", C.c_uint64),
    ]


OUT_INT_B = ("n_mapped", "n_accept", "n_accept_draft", "n_emit", "hits_proposed", "hits_accepted", "flags")
OUT_INT_M = ("out_tokens", "mapped_ids", "span_start", "span_len")
OUT_F32_M = ("p_tok", "q_tok", "ratio")


class ot_step_out(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in OUT_INT_B + OUT_INT_M + OUT_F32_M]


class ot_loss_config(C.Structure):
    _fields_ = [("lambda", C.c_float), ("lambda_mode", C.c_int32), ("ngram_term", C.c_int32), ("accepted_only", C.c_int32)]


LOSS_OUT = ("kind", "kl", "nll", "weight", "totals", "qprime")


class ot_loss_out(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in LOSS_OUT]


class ot_adapt_in(C.Structure):
    _fields_ = [("B", C.c_int32), ("gamma", C.c_float), ("w_accept", C.c_float), ("w_reject", C.c_float), ("reserved", C.c_int32),
                ("row_off", C.c_void_p), ("row_off_host", C.c_void_p), ("head_logits", C.c_void_p), ("labels", C.c_void_p),
                ("n_valid", C.c_void_p)]


class ot_adapt_out(C.Structure):
    _fields_ = [("p_accept", C.c_void_p), ("p_any_reject", C.c_void_p), ("n_keep", C.c_void_p), ("bce", C.c_void_p)]


class ot_workspace_view(C.Structure):
    _fields_ = [
        ("logits", C.c_void_p), ("ld_logits", C.c_int64), ("row_max", C.c_void_p), ("row_sumexp", C.c_void_p),
        ("row_argmax", C.c_void_p), ("draft_row_max", C.c_void_p), ("draft_row_sumexp", C.c_void_p),
        ("draft_row_argmax", C.c_void_p),
    ]


_lib = None


def load_library() -> C.CDLL:
    """Loads the in-tree shared library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2507_02659_amd.build` "
                           "(there is no CPU fallback)")
    lib = C.CDLL(LIB_PATH)
    lib.ot_verify_init.argtypes = [C.POINTER(ot_verify_config), C.POINTER(C.c_void_p)]
    lib.ot_verify_init.restype = C.c_int
    lib.ot_verify_destroy.argtypes = [C.c_void_p]
    lib.ot_verify_destroy.restype = None
    lib.ot_ngram_cache_build.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(C.c_void_p)]
    lib.ot_ngram_cache_build.restype = C.c_int
    lib.ot_ngram_cache_destroy.argtypes = [C.c_void_p]
    lib.ot_ngram_cache_destroy.restype = None
    lib.ot_ngram_cache_create.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(C.c_void_p)]
    lib.ot_ngram_cache_create.restype = C.c_int
    lib.ot_ngram_cache_insert.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(C.c_int32)]
    lib.ot_ngram_cache_insert.restype = C.c_int
    lib.ot_ngram_cache_size.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
    lib.ot_ngram_cache_size.restype = C.c_int
    lib.ot_ngram_cache_export.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                          C.c_void_p, C.c_void_p]
    lib.ot_ngram_cache_export.restype = C.c_int
    lib.ot_ngram_cache_import.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.ot_ngram_cache_import.restype = C.c_int
    lib.ot_verify_step.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(ot_step_in), C.POINTER(ot_step_out)]
    lib.ot_verify_step.restype = C.c_int
    lib.ot_verify_step_from_logits.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(ot_step_in), C.c_void_p, C.POINTER(ot_step_out)]
    lib.ot_verify_step_from_logits.restype = C.c_int
    lib.ot_distill_loss.argtypes = [C.c_void_p, C.POINTER(ot_step_in), C.POINTER(ot_step_out), C.c_void_p,
                                    C.POINTER(ot_loss_config), C.POINTER(ot_loss_out)]
    lib.ot_distill_loss.restype = C.c_int
    lib.ot_adaptive_drafting.argtypes = [C.c_void_p, C.POINTER(ot_adapt_in), C.POINTER(ot_adapt_out)]
    lib.ot_adaptive_drafting.restype = C.c_int
    lib.ot_adaptive_drafting_static.argtypes = [C.POINTER(ot_adapt_in), C.POINTER(ot_adapt_out), C.c_void_p]
    lib.ot_adaptive_drafting_static.restype = C.c_int
    lib.ot_verify_workspace.argtypes = [C.c_void_p, C.POINTER(ot_workspace_view)]
    lib.ot_verify_workspace.restype = C.c_int
    lib.ot_verify_profile.argtypes = [C.c_void_p, C.c_int32]
    lib.ot_verify_profile.restype = C.c_int
    lib.ot_verify_profile_read.argtypes = [C.c_void_p, C.POINTER(C.c_float), C.POINTER(C.c_int32)]
    lib.ot_verify_profile_read.restype = C.c_int
    lib.ot_last_error.argtypes = []
    lib.ot_last_error.restype = C.c_char_p
    lib.ot_version.argtypes = []
    lib.ot_version.restype = C.c_char_p
    _lib = lib
    return lib


def _ptr(x) -> Optional[int]:
    """Address of a torch tensor, a numpy array, or a raw integer address; None stays NULL."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if isinstance(x, np.ndarray):
        assert x.flags["C_CONTIGUOUS"]
        return x.ctypes.data
    if hasattr(x, "data_ptr"):
        assert x.is_contiguous()
        return x.data_ptr()
    raise TypeError(f"cannot take the address of {type(x)}")


def _check(rc: int):
    if rc != OT_OK:
        raise OtError(rc, ot_last_error())


def ot_last_error() -> str:
    return load_library().ot_last_error().decode()


def ot_version() -> str:
    return load_library().ot_version().decode()


def ot_verify_init(*, d, V_t, V_d, max_batch, max_k, dtype, max_ngram_len, W, direct_map, stream=None, draft_side=0):
    """W: device tensor/address [d, V_t]; direct_map: host int32 array [V_d].  Returns the context handle."""
    dm = None if direct_map is None else np.ascontiguousarray(direct_map, dtype=np.int32)
    cfg = ot_verify_config(d, V_t, V_d, max_batch, max_k, dtype, max_ngram_len, int(draft_side), _ptr(W), _ptr(dm), _ptr(stream))
    ctx = C.c_void_p()
    _check(load_library().ot_verify_init(C.byref(cfg), C.byref(ctx)))
    return ctx


def ot_verify_destroy(ctx):
    load_library().ot_verify_destroy(ctx)


def ot_ngram_cache_build(ctx, key_off, key_ids, target_ids):
    """Host int32 CSR arrays of the cache entries.  Returns the cache handle."""
    ko = np.ascontiguousarray(key_off, dtype=np.int32)
    ki = np.ascontiguousarray(key_ids, dtype=np.int32)
    ti = np.ascontiguousarray(target_ids, dtype=np.int32)
    out = C.c_void_p()
    _check(load_library().ot_ngram_cache_build(ctx, int(ti.size), _ptr(ko), _ptr(ki), _ptr(ti), C.byref(out)))
    return out


def ot_ngram_cache_destroy(cache):
    load_library().ot_ngram_cache_destroy(cache)


def ot_ngram_cache_create(ctx, capacity: int, policy: int):
    out = C.c_void_p()
    _check(load_library().ot_ngram_cache_create(ctx, int(capacity), int(policy), C.byref(out)))
    return out


def ot_ngram_cache_insert(cache, key_off, key_ids, target_ids) -> int:
    """Host int32 CSR arrays of the pairs to add; returns the number of evicted entries."""
    ko = np.ascontiguousarray(key_off, dtype=np.int32)
    ki = np.ascontiguousarray(key_ids, dtype=np.int32)
    ti = np.ascontiguousarray(target_ids, dtype=np.int32)
    ev = C.c_int32()
    _check(load_library().ot_ngram_cache_insert(cache, int(ti.size), _ptr(ko), _ptr(ki), _ptr(ti), C.byref(ev)))
    return int(ev.value)


def ot_ngram_cache_import(cache, key_off, key_ids, target_ids, uses, last_used) -> None:
    """Brings saved entries back with their statistics (the arrays ot_ngram_cache_export returns)."""
    ko = np.ascontiguousarray(key_off, dtype=np.int32)
    ki = np.ascontiguousarray(key_ids, dtype=np.int32)
    ti = np.ascontiguousarray(target_ids, dtype=np.int32)
    us = np.ascontiguousarray(uses, dtype=np.int64)
    lu = np.ascontiguousarray(last_used, dtype=np.int64)
    _check(load_library().ot_ngram_cache_import(cache, int(ti.size), _ptr(ko), _ptr(ki), _ptr(ti), _ptr(us), _ptr(lu)))


def ot_ngram_cache_size(cache):
    """(number of entries, total number of key ids)."""
    n, ids = C.c_int32(), C.c_int32()
    _check(load_library().ot_ngram_cache_size(cache, C.byref(n), C.byref(ids)))
    return int(n.value), int(ids.value)


def ot_ngram_cache_export(cache) -> dict:
    """Entries in insertion order with their use counts and last-use clocks (numpy arrays)."""
    n, ids = ot_ngram_cache_size(cache)
    out = {"key_off": np.zeros(n + 1, np.int32), "key_ids": np.zeros(max(ids, 1), np.int32),
           "target_ids": np.zeros(max(n, 1), np.int32), "uses": np.zeros(max(n, 1), np.int64),
           "last_used": np.zeros(max(n, 1), np.int64)}
    _check(load_library().ot_ngram_cache_export(cache, n, ids, _ptr(out["key_off"]), _ptr(out["key_ids"]),
                                                _ptr(out["target_ids"]), _ptr(out["uses"]), _ptr(out["last_used"])))
    out["key_ids"], out["target_ids"] = out["key_ids"][:ids], out["target_ids"][:n]
    out["uses"], out["last_used"] = out["uses"][:n], out["last_used"][:n]
    return out


def make_step_in(*, B, step, row_off, row_off_host, hidden, draft_logits, draft_ids, temperature,
                 draft_temperature, seq_id, seed) -> ot_step_in:
    return ot_step_in(int(B), int(step) & 0xFFFFFFFF, _ptr(row_off), _ptr(row_off_host), _ptr(hidden),
                      _ptr(draft_logits), _ptr(draft_ids), _ptr(temperature), _ptr(draft_temperature), _ptr(seq_id),
                      int(seed) & 0xFFFFFFFFFFFFFFFF)


def make_step_out(buffers: dict) -> ot_step_out:
    """buffers: name -> device tensor/address for every field of ot_step_out."""
    return ot_step_out(*[_ptr(buffers.get(n)) for n in OUT_INT_B + OUT_INT_M + OUT_F32_M])


def ot_verify_step(ctx, cache, step_in: ot_step_in, step_out: ot_step_out):
    _check(load_library().ot_verify_step(ctx, cache, C.byref(step_in), C.byref(step_out)))


def ot_verify_step_from_logits(ctx, cache, step_in: ot_step_in, target_logits, step_out: ot_step_out):
    _check(load_library().ot_verify_step_from_logits(ctx, cache, C.byref(step_in), _ptr(target_logits), C.byref(step_out)))


def ot_distill_loss(ctx, step_in: ot_step_in, step_out: ot_step_out, target_logits, *, lam: float, lambda_mode: int,
                    ngram_term: int, accepted_only: bool, buffers: dict):
    """buffers: name -> device tensor/address for the fields of ot_loss_out ("qprime" may be absent)."""
    cfg = ot_loss_config(float(lam), int(lambda_mode), int(ngram_term), 1 if accepted_only else 0)
    out = ot_loss_out(*[_ptr(buffers.get(n)) for n in LOSS_OUT])
    _check(load_library().ot_distill_loss(ctx, C.byref(step_in), C.byref(step_out), _ptr(target_logits), C.byref(cfg),
                                          C.byref(out)))


def ot_adaptive_drafting(ctx, *, B, gamma, w_accept=1.0, w_reject=1.0, row_off, row_off_host, head_logits, labels=None,
                         n_valid=None, p_accept, p_any_reject, n_keep, bce=None, reserved=0):
    ain = ot_adapt_in(int(B), float(gamma), float(w_accept), float(w_reject), int(reserved), _ptr(row_off), _ptr(row_off_host),
                      _ptr(head_logits), _ptr(labels), _ptr(n_valid))
    aout = ot_adapt_out(_ptr(p_accept), _ptr(p_any_reject), _ptr(n_keep), _ptr(bce))
    _check(load_library().ot_adaptive_drafting(ctx, C.byref(ain), C.byref(aout)))


def ot_adaptive_drafting_static(*, B, gamma, w_accept=1.0, w_reject=1.0, row_off, row_off_host, head_logits, labels=None,
                                n_valid=None, p_accept, p_any_reject, n_keep, bce=None, reserved=0, stream=None):
    """The allocation-free twin of ot_adaptive_drafting: no context, scratch inside the library, work on `stream`."""
    ain = ot_adapt_in(int(B), float(gamma), float(w_accept), float(w_reject), int(reserved), _ptr(row_off), _ptr(row_off_host),
                      _ptr(head_logits), _ptr(labels), _ptr(n_valid))
    aout = ot_adapt_out(_ptr(p_accept), _ptr(p_any_reject), _ptr(n_keep), _ptr(bce))
    _check(load_library().ot_adaptive_drafting_static(C.byref(ain), C.byref(aout), C.c_void_p(stream or 0)))


def ot_verify_workspace(ctx) -> ot_workspace_view:
    v = ot_workspace_view()
    _check(load_library().ot_verify_workspace(ctx, C.byref(v)))
    return v


def ot_verify_profile(ctx, enable: bool):
    _check(load_library().ot_verify_profile(ctx, 1 if enable else 0))


def ot_verify_profile_read(ctx):
    """Returns (dict stage -> accumulated milliseconds, number of steps covered)."""
    ms = (C.c_float * OT_N_STAGES)()
    n = C.c_int32()
    _check(load_library().ot_verify_profile_read(ctx, ms, C.byref(n)))
    return {STAGE_NAMES[i]: float(ms[i]) for i in range(OT_N_STAGES)}, int(n.value)
