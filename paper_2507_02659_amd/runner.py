"""Device-memory plumbing around the C ABI: uploads a batch with PyTorch-ROCm, owns output buffers, calls the step.

PyTorch is used for device allocations, host<->device copies and the stream only.  No arithmetic of the
verification path happens here; every stage runs in libotverify's kernels.
"""
from __future__ import annotations

import ctypes as C
from typing import Optional

import numpy as np
import torch

from . import binding as ot


def _to_device(x: np.ndarray, dtype: str, device) -> torch.Tensor:
    """float32 array, or uint16 bfloat16 bit patterns, to a device tensor of the same bits."""
    if dtype == "bf16":
        return torch.from_numpy(np.ascontiguousarray(x).view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(device)


def read_device(ptr: int, count: int, np_dtype) -> np.ndarray:
    """Copies `count` elements from a raw device address (used for the library's workspace view)."""
    out = np.empty(count, dtype=np_dtype)
    if count:
        hip = C.CDLL("libamdhip64.so")
        hip.hipMemcpy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int]
        hip.hipMemcpy.restype = C.c_int
        rc = hip.hipMemcpy(out.ctypes.data, C.c_void_p(ptr), out.nbytes, 2)  # hipMemcpyDeviceToHost
        if rc != 0:
            raise RuntimeError(f"hipMemcpy failed with {rc}")
    return out


class Verifier:
    """One library context plus (optionally) one n-gram cache, for batches of a fixed model shape."""

    def __init__(self, *, d, V_t, V_d, dtype: str, W, direct_map, max_batch, max_k, max_ngram_len=2,
                 device="cuda:0", stream: Optional[torch.cuda.Stream] = None, draft_side: int = ot.OT_DRAFT_SIDE_AUTO):
        if not torch.cuda.is_available():
            raise RuntimeError("otverify needs a GPU: there is no CPU path")
        self.device = torch.device(device)
        self.dtype = dtype
        self.d, self.V_t, self.V_d = d, V_t, V_d
        self.stream = stream
        torch.cuda.set_device(self.device)
        W_dev = W if isinstance(W, torch.Tensor) else _to_device(W, dtype, self.device)
        assert tuple(W_dev.shape) == (d, V_t)
        torch.cuda.synchronize(self.device)
        self.ctx = ot.ot_verify_init(d=d, V_t=V_t, V_d=V_d, max_batch=max_batch, max_k=max_k,
                                     dtype=ot.OT_BF16 if dtype == "bf16" else ot.OT_F32, max_ngram_len=max_ngram_len,
                                     W=W_dev, direct_map=direct_map,
                                     stream=None if stream is None else stream.cuda_stream, draft_side=draft_side)
        del W_dev                                   # init keeps a private re-tiled copy
        self.cache = None
        self._keep = None

    @classmethod
    def for_case(cls, case, **kw) -> "Verifier":
        kw.setdefault("max_batch", max(1, case.B))
        kw.setdefault("max_k", int(case.k.max()) if case.B else 0)
        kw.setdefault("max_ngram_len", case.max_ngram_len)
        W = case.W
        if W is None:                               # logits-only cases still need an LM head to create a context
            W = np.zeros((case.d, case.V_t), dtype=np.float32 if case.dtype == "f32" else np.uint16)
        v = cls(d=case.d, V_t=case.V_t, V_d=case.V_d, dtype=case.dtype, W=W, direct_map=case.direct_map, **kw)
        v.set_cache(case.ngram_key_off, case.ngram_key_ids, case.ngram_target_ids)
        return v

    def set_cache(self, key_off, key_ids, target_ids):
        if self.cache is not None:
            ot.ot_ngram_cache_destroy(self.cache)
        self.cache = ot.ot_ngram_cache_build(self.ctx, key_off, key_ids, target_ids)

    def close(self):
        if self.cache is not None:
            ot.ot_ngram_cache_destroy(self.cache)
            self.cache = None
        if self.ctx is not None:
            ot.ot_verify_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ------------------------------------------------------------------ batches
    def upload(self, case) -> dict:
        """Device copies of one batch's inputs and fresh output buffers."""
        dev = self.device
        i32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(dev)
        inp = {
            "B": case.B, "M": case.M, "K": case.K, "step": case.step, "seed": case.seed,
            "row_off_host": np.ascontiguousarray(case.row_off, dtype=np.int32),
            "row_off": i32(case.row_off),
            "hidden": None if case.hidden is None else _to_device(case.hidden, case.dtype, dev),
            "target_logits": None if case.target_logits is None else _to_device(case.target_logits, "f32", dev),
            "draft_logits": _to_device(case.draft_logits, case.dtype, dev),
            "draft_ids": i32(case.draft_ids),
            "temperature": torch.from_numpy(np.ascontiguousarray(case.temperature, dtype=np.float32)).to(dev),
            "draft_temperature": None if case.draft_temperature is None else
            torch.from_numpy(np.ascontiguousarray(case.draft_temperature, dtype=np.float32)).to(dev),
            "seq_id": torch.from_numpy(np.ascontiguousarray(case.seq_id, dtype=np.uint64).view(np.int64)).to(dev),
        }
        inp["out"] = self.alloc_outputs(case.B, case.M)
        return inp

    def alloc_outputs(self, B: int, M: int) -> dict:
        dev = self.device
        out = {n: torch.full((max(B, 1),), -7, dtype=torch.int32, device=dev) for n in ot.OUT_INT_B}
        out.update({n: torch.full((max(M, 1),), -7, dtype=torch.int32, device=dev) for n in ot.OUT_INT_M})
        out.update({n: torch.full((max(M, 1),), -7.0, dtype=torch.float32, device=dev) for n in ot.OUT_F32_M})
        return out

    def step(self, inp: dict, *, from_logits: bool = False, use_cache: bool = True, step: Optional[int] = None):
        """Enqueues one ot_verify_step on the context's stream (asynchronous)."""
        sin = ot.make_step_in(B=inp["B"], step=inp["step"] if step is None else step, row_off=inp["row_off"],
                              row_off_host=inp["row_off_host"], hidden=inp["hidden"], draft_logits=inp["draft_logits"],
                              draft_ids=inp["draft_ids"], temperature=inp["temperature"],
                              draft_temperature=inp["draft_temperature"], seq_id=inp["seq_id"], seed=inp["seed"])
        sout = ot.make_step_out(inp["out"])
        cache = self.cache if use_cache else None
        if from_logits:
            ot.ot_verify_step_from_logits(self.ctx, cache, sin, inp["target_logits"], sout)
        else:
            ot.ot_verify_step(self.ctx, cache, sin, sout)

    def distill_loss(self, inp: dict, *, from_logits: bool = False, lam: float = 0.2, lambda_mode: int = ot.OT_LAMBDA_FIXED,
                     ngram_term: int = ot.OT_NGRAM_TERM_NLL, accepted_only: bool = False, with_qprime: bool = False,
                     sync: bool = True) -> Optional[dict]:
        """Enqueues ot_distill_loss after a step on `inp`; with sync, waits and returns its outputs as numpy arrays."""
        dev = self.device
        M = max(inp["M"], 1)
        key = ("loss_buffers", M, with_qprime)
        buf = inp.get(key)
        if buf is None:
            buf = {"kind": torch.full((M,), -7, dtype=torch.int32, device=dev),
                   "totals": torch.full((5,), -7.0, dtype=torch.float64, device=dev)}
            buf.update({n: torch.full((M,), -7.0, dtype=torch.float64, device=dev) for n in ("kl", "nll", "weight")})
            if with_qprime:
                buf["qprime"] = torch.full((M, self.V_t), -7.0, dtype=torch.float32, device=dev)
            inp[key] = buf
        sin = ot.make_step_in(B=inp["B"], step=inp["step"], row_off=inp["row_off"], row_off_host=inp["row_off_host"],
                              hidden=inp["hidden"], draft_logits=inp["draft_logits"], draft_ids=inp["draft_ids"],
                              temperature=inp["temperature"], draft_temperature=inp["draft_temperature"],
                              seq_id=inp["seq_id"], seed=inp["seed"])
        ot.ot_distill_loss(self.ctx, sin, ot.make_step_out(inp["out"]), inp["target_logits"] if from_logits else None,
                           lam=lam, lambda_mode=lambda_mode, ngram_term=ngram_term, accepted_only=accepted_only, buffers=buf)
        if not sync:
            return None
        self.synchronize()
        res = {n: t.cpu().numpy()[:inp["M"]] for n, t in buf.items() if n != "totals"}
        totals = buf["totals"].cpu().numpy()
        res.update(loss_dm=float(totals[0]), loss_ngram=float(totals[1]), n_dm=int(totals[2]), n_ngram_tokens=int(totals[3]),
                   loss=float(totals[4]))
        return res

    def synchronize(self):
        if self.stream is not None:
            self.stream.synchronize()
        else:
            torch.cuda.synchronize(self.device)

    def results(self, inp: dict) -> dict:
        """Synchronises and returns the outputs as numpy arrays trimmed to [B] / [M]."""
        self.synchronize()
        B, M = inp["B"], inp["M"]
        res = {}
        for n, t in inp["out"].items():
            a = t.cpu().numpy()
            res[n] = a[:B] if n in ot.OUT_INT_B else a[:M]
        return res

    def workspace(self, M: int, K: int, with_logits: bool = False) -> dict:
        """Row statistics (and optionally the logits) the last step left in the library's workspace."""
        self.synchronize()
        v = ot.ot_verify_workspace(self.ctx)
        ws = {
            "row_max": read_device(v.row_max, M, np.float32),
            "row_sumexp": read_device(v.row_sumexp, M, np.float64),
            "row_argmax": read_device(v.row_argmax, M, np.int32),
            "draft_row_max": read_device(v.draft_row_max, K, np.float32),
            "draft_row_sumexp": read_device(v.draft_row_sumexp, K, np.float64),
            "draft_row_argmax": read_device(v.draft_row_argmax, K, np.int32),
        }
        if with_logits:
            ws["logits"] = read_device(v.logits, M * int(v.ld_logits), np.float32).reshape(M, int(v.ld_logits))
        return ws

    def run_case(self, case, **kw) -> dict:
        inp = self.upload(case)
        self.step(inp, from_logits=case.hidden is None, **kw)
        return self.results(inp)
