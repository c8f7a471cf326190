"""Seeded synthetic workloads shaped like the paper's verification inputs.

The paper evaluates a Llama-68M drafter (draft vocabulary 32000) against
Vicuna-7B / Qwen2-7B / Llama3-8B targets (vocabularies 32000 / 152064 / 128256,
Appendix table of model latency and vocabulary statistics) with draft lengths of
3-5 tokens, n-gram caches of a few thousand to a few tens of thousands of
entries whose usage frequency is long-tailed (Appendix, n-gram distribution
figure).  None of those models, tokenizers or datasets is available here, so
every input is drawn from a seeded ``numpy.random.Generator(PCG64)`` with those
*shapes* only.

Nothing in this file is part of the verification method: it draws tensors,
rounds them to the storage dtype, builds vocabulary maps / cache entries and
picks drafted ids.  The softmax used to *pick drafted ids* stands in for the
drafter's own sampling (Algorithm 1, draft loop), which is outside the
verification step.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

__all__ = [
    "VerifyCase",
    "CaseSpec",
    "make_case",
    "baseline_spec",
    "baseline_case",
    "f32_to_bf16_bits",
    "bf16_bits_to_f32",
]


# --------------------------------------------------------------------------- dtype helpers
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 values to bfloat16 (round-to-nearest-even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns to float32 exactly."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------- containers
@dataclass
class CaseSpec:
    """Recipe for one synthetic verification batch."""

    name: str
    dtype: str                      # "bf16" or "f32": storage type of hidden, W and draft logits
    d: int
    V_t: int
    V_d: int
    k: Sequence[int]                # drafted tokens per sequence (ragged allowed)
    temperature: Sequence[float]    # per sequence; 0 means greedy
    n_direct: int = 0               # number of direct draft<->target pairs (ignored when identity_map)
    identity_map: bool = False      # V_d == V_t identity map ...
    permute_frac: float = 0.0       # ... with this fraction of ids permuted among themselves
    n_ngram: int = 0                # n-gram cache entries
    ngram_len: Tuple[int, int] = (2, 3)   # inclusive range of key lengths
    zipf_a: float = 0.0             # >0: key component ids follow a truncated Zipf(a); 0: uniform
    plant_cover: float = 0.0        # target fraction of draft positions covered by planted cache keys
    max_ngram_len: int = 0          # capacity handed to the library (0: ngram_len[1], at least 2)
    draft_temperature: Optional[Sequence[float]] = None
    data_seed: int = 0
    philox_seed: int = 0
    step: int = 0
    align: float = 0.0              # probability that a mapped position is made "agreeable" (see make_case)
    logits_only: bool = False       # draw target logits directly instead of hidden states and W
    sigma_h: float = 1.0
    sigma_w: float = 0.02
    sigma_q: float = 2.0


@dataclass
class VerifyCase:
    """One batch of inputs, bit-identical for the CPU oracle and the HIP path.

    Floating-point tensors are float32 arrays when ``dtype == "f32"`` and uint16
    arrays of bfloat16 bit patterns when ``dtype == "bf16"``.
    """

    spec: CaseSpec
    name: str
    dtype: str
    d: int
    V_t: int
    V_d: int
    B: int
    k: np.ndarray                   # [B] int32
    row_off: np.ndarray             # [B+1] int32; sequence b owns rows row_off[b]..row_off[b+1]-1 (k_b+1 rows)
    hidden: Optional[np.ndarray]    # [M, d]
    W: Optional[np.ndarray]         # [d, V_t]
    target_logits: Optional[np.ndarray]  # [M, V_t] float32, only for logits_only cases
    draft_logits: np.ndarray        # [K, V_d]; sequence b's rows start at row_off[b] - b
    draft_ids: np.ndarray           # [K] int32
    direct_map: np.ndarray          # [V_d] int32, target id or -1
    ngram_key_off: np.ndarray       # [E+1] int32
    ngram_key_ids: np.ndarray       # [sum len] int32
    ngram_target_ids: np.ndarray    # [E] int32
    max_ngram_len: int
    temperature: np.ndarray         # [B] float32
    draft_temperature: Optional[np.ndarray]
    seed: int                       # Philox key (uint64)
    seq_id: np.ndarray              # [B] uint64
    step: int
    planted: List[List[Tuple[int, int]]] = field(default_factory=list)  # per sequence (start, len) of planted keys

    @property
    def M(self) -> int:
        return int(self.row_off[-1])

    @property
    def K(self) -> int:
        return int(self.k.sum())


# --------------------------------------------------------------------------- building blocks
def _store(x32: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "f32":
        return np.ascontiguousarray(x32, dtype=np.float32)
    if dtype == "bf16":
        return f32_to_bf16_bits(x32)
    raise ValueError(f"unknown dtype {dtype!r}")


def _values(stored: np.ndarray, dtype: str) -> np.ndarray:
    return stored if dtype == "f32" else bf16_bits_to_f32(stored)


def _normal(rng: np.random.Generator, shape, sigma: float, dtype: str, slab_rows: int = 256) -> np.ndarray:
    """N(0, sigma^2) in float32, rounded to the storage dtype, drawn in row slabs to bound memory."""
    rows = shape[0]
    out = np.empty(shape, dtype=np.float32 if dtype == "f32" else np.uint16)
    for r0 in range(0, rows, slab_rows):
        r1 = min(rows, r0 + slab_rows)
        blk = rng.standard_normal((r1 - r0,) + tuple(shape[1:]), dtype=np.float32)
        blk *= np.float32(sigma)
        out[r0:r1] = _store(blk, dtype)
    return out


def _direct_map(rng, spec: CaseSpec) -> np.ndarray:
    dmap = np.full(spec.V_d, -1, dtype=np.int32)
    if spec.identity_map:
        assert spec.V_d == spec.V_t
        dmap[:] = np.arange(spec.V_d, dtype=np.int32)
        n_perm = int(round(spec.permute_frac * spec.V_d))
        if n_perm >= 2:
            ids = rng.choice(spec.V_d, size=n_perm, replace=False)
            dmap[ids] = ids[rng.permutation(n_perm)].astype(np.int32)
        return dmap
    n = spec.n_direct
    assert n <= spec.V_d and n <= spec.V_t
    src = rng.choice(spec.V_d, size=n, replace=False)
    dst = rng.choice(spec.V_t, size=n, replace=False)
    dmap[src] = dst.astype(np.int32)
    return dmap


def _zipf_sampler(rng, V_d: int, a: float):
    """Returns draw(n) -> ids with P(rank r) ~ r^-a over a fixed random rank->id permutation."""
    if a <= 0.0:
        return lambda n: rng.integers(0, V_d, size=n)
    w = np.arange(1, V_d + 1, dtype=np.float64) ** (-a)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    rank_to_id = rng.permutation(V_d)

    def draw(n):
        r = np.searchsorted(cdf, rng.random(n), side="right")
        return rank_to_id[np.minimum(r, V_d - 1)]

    return draw


def _ngram_cache(rng, spec: CaseSpec, dmap: np.ndarray):
    """Entries (key of 2..L draft ids -> one target id outside the direct image), keys unique."""
    E = spec.n_ngram
    if E == 0:
        return np.zeros(1, np.int32), np.zeros(0, np.int32), np.zeros(0, np.int32)
    lo, hi = spec.ngram_len
    used = np.zeros(spec.V_t, dtype=bool)
    used[dmap[dmap >= 0]] = True
    free = np.flatnonzero(~used)
    assert free.size >= E, "not enough unshared target ids for the n-gram entries"
    targets = free[rng.choice(free.size, size=E, replace=False)].astype(np.int32)
    draw = _zipf_sampler(rng, spec.V_d, spec.zipf_a)
    keys, seen = [], set()
    while len(keys) < E:
        need = E - len(keys)
        lens = rng.integers(lo, hi + 1, size=need)
        ids = draw(int(lens.sum()))
        p = 0
        for L in lens:
            key = tuple(int(v) for v in ids[p:p + L])
            p += L
            if key not in seen:
                seen.add(key)
                keys.append(key)
    key_off = np.zeros(E + 1, dtype=np.int32)
    key_off[1:] = np.cumsum([len(kk) for kk in keys])
    key_ids = np.fromiter((v for kk in keys for v in kk), dtype=np.int32, count=int(key_off[-1]))
    return key_off, key_ids, targets


def _pick_from_logits(rng, row64: np.ndarray, T: float) -> int:
    """Stand-in for the drafter's sampling d ~ q(.) at temperature T (argmax when T == 0)."""
    if T <= 0.0:
        return int(np.argmax(row64))
    z = row64 / T
    z = z - z.max()
    e = np.exp(z)
    c = np.cumsum(e)
    return int(min(np.searchsorted(c, rng.random() * c[-1], side="right"), row64.size - 1))


# --------------------------------------------------------------------------- main entry
def make_case(spec: CaseSpec) -> VerifyCase:
    """Draw one batch according to ``spec``.

    Draw order (fixed, so a spec always yields the same bits): direct map, cache,
    draft logits, drafted ids (walking each sequence; a position starts a planted
    cache key with the probability that gives ``plant_cover``), then W and hidden
    states (or target logits when ``logits_only``).

    ``align`` > 0 makes some mapped positions "agreeable": the drafted id gets a
    raised draft logit before it is sampled, and the hidden row of that mapped
    position is set to a scaled copy of the LM-head column of the token the
    proposal maps to (or, for ``logits_only``, that logit is raised), so that
    p/q' lands in a mid range and acceptance runs of several tokens, rejections
    deep in the window and bonus tokens all occur.  The BASELINE configurations
    use align = 0.
    """
    root = np.random.SeedSequence(spec.data_seed)
    s_map, s_cache, s_q, s_ids, s_w, s_h = (np.random.Generator(np.random.PCG64(s)) for s in root.spawn(6))

    k = np.asarray(spec.k, dtype=np.int32)
    B = int(k.size)
    assert np.all(k >= 0)
    row_off = np.zeros(B + 1, dtype=np.int32)
    row_off[1:] = np.cumsum(k + 1)
    M, K = int(row_off[-1]), int(k.sum())
    temperature = np.asarray(spec.temperature, dtype=np.float32)
    assert temperature.size == B
    dtemp = None if spec.draft_temperature is None else np.asarray(spec.draft_temperature, dtype=np.float32)

    dmap = _direct_map(s_map, spec)
    key_off, key_ids, tgt_ids = _ngram_cache(s_cache, spec, dmap)
    E = int(tgt_ids.size)
    max_L = spec.max_ngram_len or max(2, spec.ngram_len[1] if E else 2)

    # ---- draft logits, with optional bumps for agreeable positions
    q_store = _normal(s_q, (max(K, 1), spec.V_d), spec.sigma_q, spec.dtype)[:K]
    q_val = _values(q_store, spec.dtype).astype(np.float32)

    # ---- drafted ids
    by_len = {}
    for e in range(E):
        by_len.setdefault(int(key_off[e + 1] - key_off[e]), []).append(e)
    lens_sorted = sorted(by_len)
    if E and spec.plant_cover > 0.0:
        mean_L = float(np.mean(np.diff(key_off)))
        c = spec.plant_cover
        rho = c / (mean_L * (1.0 - c) + c)
    else:
        rho = 0.0
    log_norm_q = np.log(spec.V_d) + 0.5 * spec.sigma_q ** 2  # log of the expected softmax normaliser

    draft_ids = np.zeros(K, dtype=np.int32)
    planted: List[List[Tuple[int, int]]] = []
    agree: List[Tuple[int, int]] = []   # (global row, target id) of agreeable mapped positions
    for b in range(B):
        kb = int(k[b])
        base = int(row_off[b]) - b
        Td = float(dtemp[b]) if dtemp is not None else float(temperature[b])
        s, j, plist = 0, 0, []
        while s < kb:
            fit = [L for L in lens_sorted if L <= kb - s]
            if fit and s_ids.random() < rho:
                counts = np.array([len(by_len[L]) for L in fit], dtype=np.float64)
                L = fit[int(s_ids.choice(len(fit), p=counts / counts.sum()))]
                e = by_len[L][int(s_ids.integers(0, len(by_len[L])))]
                draft_ids[base + s: base + s + L] = key_ids[key_off[e]: key_off[e] + L]
                plist.append((s, L))
                if spec.align > 0.0 and s_ids.random() < spec.align:
                    agree.append((int(row_off[b]) + j, int(tgt_ids[e])))
                s += L
            else:
                want_agree = spec.align > 0.0 and s_ids.random() < spec.align
                if want_agree:
                    c_id = int(s_ids.integers(0, spec.V_d))
                    bump = np.float32(log_norm_q + s_ids.uniform(-2.0, 2.0))
                    q_val[base + s, c_id] = np.float32(q_val[base + s, c_id]) + bump
                    q_store[base + s] = _store(q_val[base + s], spec.dtype)
                    q_val[base + s] = _values(q_store[base + s], spec.dtype)
                d_id = _pick_from_logits(s_ids, q_val[base + s].astype(np.float64), Td)
                draft_ids[base + s] = d_id
                if want_agree and dmap[d_id] >= 0:
                    agree.append((int(row_off[b]) + j, int(dmap[d_id])))
                s += 1
            j += 1
        planted.append(plist)

    # ---- target side
    hidden = W = Z = None
    if spec.logits_only:
        sigma_z = spec.sigma_w * np.sqrt(spec.d) * spec.sigma_h
        Z = _normal(s_h, (max(M, 1), spec.V_t), sigma_z, "f32")[:M]
        log_norm_p = np.log(spec.V_t) + 0.5 * sigma_z ** 2
        for row, t in agree:
            Z[row, t] = np.float32(log_norm_p + s_h.uniform(-2.0, 3.0))
    else:
        W = _normal(s_w, (spec.d, spec.V_t), spec.sigma_w, spec.dtype)
        h32 = s_h.standard_normal((max(M, 1), spec.d), dtype=np.float32)[:M] * np.float32(spec.sigma_h)
        log_norm_p = np.log(spec.V_t) + 0.5 * (spec.sigma_w ** 2) * spec.d
        for row, t in agree:
            w_t = _values(W[:, t], spec.dtype).astype(np.float64)
            z_star = log_norm_p + s_h.uniform(-2.0, 3.0)
            beta = z_star / float(w_t @ w_t)
            h32[row] = (beta * w_t + 0.3 * s_h.standard_normal(spec.d)).astype(np.float32)
        hidden = _store(h32, spec.dtype)

    seq_id = np.arange(B, dtype=np.uint64)
    return VerifyCase(
        spec=spec, name=spec.name, dtype=spec.dtype, d=spec.d, V_t=spec.V_t, V_d=spec.V_d, B=B, k=k,
        row_off=row_off, hidden=hidden, W=W, target_logits=Z, draft_logits=q_store, draft_ids=draft_ids,
        direct_map=dmap, ngram_key_off=key_off, ngram_key_ids=key_ids, ngram_target_ids=tgt_ids,
        max_ngram_len=int(max_L), temperature=temperature, draft_temperature=dtemp,
        seed=int(spec.philox_seed), seq_id=seq_id, step=int(spec.step), planted=planted,
    )


# --------------------------------------------------------------------------- the five BASELINE configurations
def baseline_spec(i: int, *, greedy: bool = False, scale: Optional[dict] = None) -> CaseSpec:
    """Spec of BASELINE configuration ``i`` (1..5).

    ``greedy`` selects the temperature-0 run of configuration 2.  ``scale`` may
    override fields (e.g. ``{"d": 128, "V_t": 4096}``) to get a same-structure
    case small enough for CPU-only tests.
    """
    if i == 1:
        s = CaseSpec(name="cfg1_tiny_f32", dtype="f32", d=256, V_t=1024, V_d=512, k=[4], temperature=[1.0],
                     n_direct=400, n_ngram=64, ngram_len=(2, 3), zipf_a=0.0, plant_cover=0.0,
                     data_seed=1000, philox_seed=0)
    elif i == 2:
        T = 0.0 if greedy else 1.0
        s = CaseSpec(name="cfg2_vicuna7b" + ("_greedy" if greedy else ""), dtype="bf16", d=4096, V_t=32000,
                     V_d=32000, k=[5], temperature=[T], identity_map=True, permute_frac=0.02,
                     data_seed=1001, philox_seed=1)
    elif i == 3:
        s = CaseSpec(name="cfg3_qwen2_7b", dtype="bf16", d=3584, V_t=152064, V_d=32000, k=[5],
                     temperature=[1.0], n_direct=28000, n_ngram=20000, ngram_len=(2, 4), zipf_a=1.1,
                     plant_cover=0.30, data_seed=10002, philox_seed=2)
    elif i == 4:
        s = CaseSpec(name="cfg4_llama3_8b_b16", dtype="bf16", d=4096, V_t=128256, V_d=32000, k=[8] * 16,
                     temperature=[0.7] * 16, n_direct=30000, n_ngram=50000, ngram_len=(2, 5), zipf_a=1.1,
                     plant_cover=0.30, data_seed=1003, philox_seed=3)
    elif i == 5:
        rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([1004, 77])))
        kk = rng.integers(1, 11, size=64).tolist()
        tt = np.where(rng.random(64) < 0.5, 0.0, 1.0).tolist()
        s = CaseSpec(name="cfg5_adaptive_ragged_b64", dtype="bf16", d=3584, V_t=152064, V_d=32000, k=kk,
                     temperature=tt, n_direct=28000, n_ngram=100000, ngram_len=(2, 6), zipf_a=1.05,
                     plant_cover=0.30, data_seed=1004, philox_seed=4)
    else:
        raise ValueError("configuration index must be 1..5")
    if scale:
        for key, val in scale.items():
            setattr(s, key, val)
        s.name += "_scaled"
    return s


def baseline_case(i: int, **kw) -> VerifyCase:
    return make_case(baseline_spec(i, **kw))
