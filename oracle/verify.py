"""CPU oracle of the target-side verification step of cross-vocabulary speculative decoding.

TEST INFRASTRUCTURE ONLY: plain NumPy float64, slow and obvious.  Imported by
tests/, by __graft_entry__.smoke() and by bench.py's cpu_baseline leg; it shares
no code with the HIP path and the product never calls it.

What it computes (OmniDraft, Methodology): for every sequence of a batch,

  1. target logits z_j = h_j . W for the k+1 verified rows (Algorithm 1, the
     parallel target pass over the mapped tokens) and the
     target distribution p_j = softmax(z_j / T)              (Notation paragraph);
  2. the draft distribution q_i = softmax(zq_i / T_d) at each drafted position;
  3. the translation of the drafted ids d_0..d_{k-1} into target-vocabulary
     tokens t_0..t_{m-1} with probabilities q'(t_j): a direct id map on the
     shared vocabulary, and n-gram cache entries that merge several consecutive
     draft tokens into one target token whose probability is the product of the
     sub-token probabilities            (Section "Cross-vocabulary N-gram Cache", Eq. 1);
  4. rejection sampling with ratios min(1, p(t_j)/q'(t_j))          (Algorithm 1);
  5. the final token: from norm(max(0, p - q')) at the first rejected position,
     with q' extended to the whole target vocabulary by Eq. 2, or a free token
     from p when every mapped token was accepted                    (Algorithm 1).

Readings taken where the paper is silent (each mirrored by the HIP path):
  * scan is left to right, greedy, longest cache match first, n-gram beats the
    direct map, no partial match at the end of the window;
  * a drafted id with neither a cache hit nor a direct image ends the proposal
    ("unmappable"): the final token is then drawn from the residual built from
    that position's draft distribution, which keeps direct-map-only decoding
    exactly lossless;
  * q' is not renormalised after mapping; target ids without a direct pre-image
    get q' = 0;
  * Eq. 2's "otherwise" branch uses the draft distribution at the first
    sub-token's position, and its two overrides apply only for the n-gram
    matched at the rejected position itself; the n-gram case wins if both
    overrides name the same target id;
  * u in [0,1), accept iff u < ratio; q' = 0 gives ratio 1 if p > 0 else 0;
  * temperature 0 is the greedy limit: accept iff t_j is the (lowest-index)
    argmax of z_j, emit the argmax at the first mismatch, no uniforms used;
  * the final token is drawn by inverse CDF over ascending token id with one
    24-bit uniform; a residual of total mass 0 falls back to p (flagged);
  * duplicate cache keys: the last entry wins.

Pins (tests/test_oracle_*.py, all `-m "not gpu"`): library softmax/matmul special
cases, the span patterns of Fig. 1 and of the Appendix table of n-gram inference
examples, an independent naive matcher, the invariants of speculative sampling
(q = p accepts everything, residual sums to one, T = 0 is an argmax match, Eq. 2
conserves mass), exact enumeration of the emitted-token law on tiny vocabularies
(equals p for direct maps), Monte Carlo against that law, and Philox known-answer
vectors.  No function here is "parity unpinned".
"""
from __future__ import annotations

from typing import Dict, Optional, Tuple

import numpy as np

from .philox import uniforms

FLAG_UNMAPPABLE = 1   # a drafted id had no cache hit and no direct image; proposal cut there
FLAG_RESID_ZERO = 2   # residual had zero mass; final token drawn from p instead
FLAG_BAD_ID = 4       # a drafted id was outside [0, V_d); the sequence emits nothing


# --------------------------------------------------------------------------- input widening
def widen(x: np.ndarray, dtype: str) -> np.ndarray:
    """Stored tensor (float32, or uint16 bfloat16 bit patterns) -> float64, exactly."""
    if dtype == "f32":
        return np.asarray(x, dtype=np.float32).astype(np.float64)
    if dtype == "bf16":
        return (np.asarray(x, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    raise ValueError(dtype)


# --------------------------------------------------------------------------- step 1: LM head
def lm_head_logits(hidden: np.ndarray, W: np.ndarray, dtype: str, slab: int = 8192) -> np.ndarray:
    """z = H . W in float64; W is walked in column slabs only to bound memory (no other blocking)."""
    H = widen(hidden, dtype)
    V_t = W.shape[1]
    Z = np.empty((H.shape[0], V_t), dtype=np.float64)
    for c0 in range(0, V_t, slab):
        c1 = min(V_t, c0 + slab)
        Z[:, c0:c1] = H @ widen(W[:, c0:c1], dtype)
    return Z


# --------------------------------------------------------------------------- steps 1-2: distributions
def distribution(z: np.ndarray, T: float) -> np.ndarray:
    """softmax(z / T) for T > 0; one-hot at the lowest-index argmax for T == 0."""
    z = np.asarray(z, dtype=np.float64)
    if T <= 0.0:
        p = np.zeros_like(z)
        p[int(np.argmax(z))] = 1.0
        return p
    a = (z - z.max()) / T
    e = np.exp(a)
    return e / e.sum()


# --------------------------------------------------------------------------- step 3: translation (Eq. 1)
def build_cache(key_off, key_ids, target_ids) -> Dict[Tuple[int, ...], int]:
    """The n-gram cache C = {(t_i, [d_j])} as a dict keyed by the draft-id tuple; last duplicate wins."""
    cache: Dict[Tuple[int, ...], int] = {}
    for e in range(len(target_ids)):
        cache[tuple(int(v) for v in key_ids[key_off[e]:key_off[e + 1]])] = int(target_ids[e])
    return cache


def map_merge(d, dmap, cache, max_ngram_len: int):
    """Scan d_0..d_{k-1}; returns (tokens t_j, spans (s_j, L_j), unmappable, s_end)."""
    k = len(d)
    tokens, spans = [], []
    s = 0
    unmappable = False
    while s < k:
        hit = None
        for L in range(min(max_ngram_len, k - s), 1, -1):
            t = cache.get(tuple(int(v) for v in d[s:s + L]))
            if t is not None:
                hit = (t, L)
                break
        if hit is not None:
            tokens.append(hit[0])
            spans.append((s, hit[1]))
            s += hit[1]
        elif dmap[d[s]] >= 0:
            tokens.append(int(dmap[d[s]]))
            spans.append((s, 1))
            s += 1
        else:
            unmappable = True
            break
    return tokens, spans, unmappable, s


def qprime_pointwise(q_rows, d, span) -> float:
    """Eq. 1: q'(t_j) = q(d) for a direct token, the product of sub-token probabilities for an n-gram."""
    s, L = span
    prod = 1.0
    for l in range(L):
        prod *= q_rows[s + l][int(d[s + l])]
    return float(prod)


def inverse_map(dmap, V_t: int) -> np.ndarray:
    """tmap[t] = the draft id whose direct image is t, or -1 (the direct map is a bijection on the shared part)."""
    dmap = np.asarray(dmap)
    tmap = np.full(V_t, -1, dtype=np.int64)
    src = np.flatnonzero(dmap >= 0)
    tmap[dmap[src]] = src
    return tmap


def qprime_full(q_s: np.ndarray, dmap, tmap: np.ndarray, ngram=None) -> np.ndarray:
    """Eq. 2: q' over the whole target vocabulary, from the draft distribution q_s at draft position s.

    ngram = (t, pi, d1): the n-gram matched at this position maps to target id t with product pi, and its
    first sub-token is d1.  Then q'(t) = pi and, if d1 has a direct image, q'(dmap[d1]) = q_s(d1) - pi.
    """
    qp = np.where(tmap >= 0, q_s[np.maximum(tmap, 0)], 0.0)
    if ngram is not None:
        t, pi, d1 = ngram
        if dmap[d1] >= 0:
            qp[int(dmap[d1])] = q_s[int(d1)] - pi
        qp[int(t)] = pi
    return qp


# --------------------------------------------------------------------------- steps 4-5
def residual(p: np.ndarray, qp: np.ndarray) -> np.ndarray:
    """Unnormalised residual max(0, p - q') (Notation paragraph)."""
    return np.maximum(0.0, p - qp)


def sample_inverse_cdf(r: np.ndarray, u: float):
    """Token = min{v : c_v > u * c_last}, c = running sum of r in ascending id.

    Returns (v, margin, (prev, next)): margin is the distance of u * c_last to the nearer edge of v's cell as a
    fraction of the total mass; prev / next are the nearest ids below / above v with r > 0 (-1 if none).  The
    last two are diagnostics for comparisons against lower-precision implementations.
    """
    c = np.cumsum(r)
    total = c[-1]
    x = u * total
    v = int(np.searchsorted(c, x, side="right"))
    if v >= r.size:
        v = int(np.flatnonzero(r > 0)[-1])
    below = c[v - 1] if v > 0 else 0.0
    margin = min(x - below, c[v] - x) / total
    support = np.flatnonzero(r > 0)
    at = int(np.searchsorted(support, v))
    prev_id = int(support[at - 1]) if at > 0 else -1
    next_id = int(support[at + 1]) if at + 1 < support.size else -1
    return v, float(margin), (prev_id, next_id)


def verify_step(*, row_off, draft_ids, draft_logits, direct_map, V_t: int, cache: Optional[dict],
                max_ngram_len: int, temperature, draft_temperature=None, seed: int, seq_id, step: int,
                dtype: str, hidden=None, W=None, target_logits=None, return_logits: bool = False) -> dict:
    """One verification step for a ragged batch.  Either (hidden, W) or float32 target_logits is given."""
    row_off = np.asarray(row_off, dtype=np.int64)
    B = row_off.size - 1
    M = int(row_off[-1])
    cache = cache or {}
    dmap = np.asarray(direct_map, dtype=np.int64)
    V_d = dmap.size
    tmap = inverse_map(dmap, V_t)
    if target_logits is not None:
        Z = np.asarray(target_logits, dtype=np.float32).astype(np.float64)
    else:
        Z = lm_head_logits(hidden, W, dtype)
    Zq = widen(draft_logits, dtype)

    out = {
        "n_mapped": np.zeros(B, np.int32), "n_accept": np.zeros(B, np.int32),
        "n_accept_draft": np.zeros(B, np.int32), "n_emit": np.zeros(B, np.int32),
        "hits_proposed": np.zeros(B, np.int32), "hits_accepted": np.zeros(B, np.int32),
        "flags": np.zeros(B, np.int32),
        "out_tokens": np.full(M, -1, np.int32), "mapped_ids": np.full(M, -1, np.int32),
        "span_start": np.full(M, -1, np.int32), "span_len": np.zeros(M, np.int32),
        "p_tok": np.zeros(M, np.float64), "q_tok": np.zeros(M, np.float64), "ratio": np.zeros(M, np.float64),
        # diagnostics (not part of the library's outputs)
        "u_margin": np.full(M, np.inf), "cdf_margin": np.full(B, np.inf), "top2_gap": np.full(M, np.inf),
        "row_max": Z.max(axis=1) if M else np.zeros(0), "row_argmax": Z.argmax(axis=1) if M else np.zeros(0, np.int64),
        "row_sumexp": np.zeros(M), "final_row": np.full(B, -1, np.int32),
        "cdf_neighbors": np.full((B, 2), -1, np.int64),
        "used_keys": [],          # draft-id tuples of the cache entries the translation used, in batch order
    }
    if return_logits:
        out["logits"] = Z

    for b in range(B):
        r0 = int(row_off[b])
        k = int(row_off[b + 1]) - r0 - 1
        q0 = r0 - b
        d = np.asarray(draft_ids[q0:q0 + k], dtype=np.int64)
        T = float(temperature[b])
        Td = T if draft_temperature is None else float(draft_temperature[b])
        for j in range(k + 1):
            zz = Z[r0 + j]
            if T > 0:
                out["row_sumexp"][r0 + j] = np.exp((zz - zz.max()) / T).sum()
            top2 = np.partition(zz, -2)[-2:]
            out["top2_gap"][r0 + j] = top2[1] - top2[0]

        if np.any(d < 0) or np.any(d >= V_d):
            out["flags"][b] |= FLAG_BAD_ID
            continue

        q_rows = [distribution(Zq[q0 + i], Td) for i in range(k)]
        tokens, spans, unmappable, s_end = map_merge(d, dmap, cache, max_ngram_len)
        m = len(tokens)
        out["n_mapped"][b] = m
        if unmappable:
            out["flags"][b] |= FLAG_UNMAPPABLE
        qprime = [qprime_pointwise(q_rows, d, sp) for sp in spans]
        for j in range(m):
            out["mapped_ids"][r0 + j] = tokens[j]
            out["span_start"][r0 + j], out["span_len"][r0 + j] = spans[j]
            out["q_tok"][r0 + j] = qprime[j]
        out["hits_proposed"][b] = sum(1 for sp in spans if sp[1] > 1)
        out["used_keys"] += [tuple(int(v) for v in d[sp[0]:sp[0] + sp[1]]) for sp in spans if sp[1] > 1]

        # ---- rejection sampling, Algorithm 1: accept t_j with probability min(1, p(t_j)/q'(t_j))
        accepted = np.zeros(m, dtype=bool)
        for j in range(m):
            p_j = distribution(Z[r0 + j], T)
            pt = float(p_j[tokens[j]])
            out["p_tok"][r0 + j] = pt
            if T > 0:
                if qprime[j] > 0.0:
                    ratio = min(1.0, pt / qprime[j])
                else:
                    ratio = 1.0 if pt > 0.0 else 0.0
                u, _ = uniforms(seed, seq_id[b], step, j)
                accepted[j] = u < ratio
                out["u_margin"][r0 + j] = abs(u - ratio)
            else:
                ratio = 1.0 if pt > 0.0 else 0.0
                accepted[j] = pt > 0.0
            out["ratio"][r0 + j] = ratio
        n = m if accepted.all() else int(np.argmin(accepted))
        out["u_margin"][r0 + n + 1:r0 + k + 1] = np.inf      # positions after the first rejection are never tested
        out["n_accept"][b] = n
        out["n_accept_draft"][b] = sum(spans[j][1] for j in range(n))
        out["hits_accepted"][b] = sum(1 for j in range(n) if spans[j][1] > 1)
        out["out_tokens"][r0:r0 + n] = tokens[:n]
        out["n_emit"][b] = n + 1
        out["final_row"][b] = r0 + n

        # ---- final token at row n
        p_n = distribution(Z[r0 + n], T)
        if T <= 0:
            out["out_tokens"][r0 + n] = int(np.argmax(p_n))
            continue
        if n == m and not unmappable:
            r = p_n                                       # free token ~ p (Algorithm 1, n == m branch)
        else:
            s = spans[n][0] if n < m else s_end
            ngram = None
            if n < m and spans[n][1] > 1:
                ngram = (tokens[n], qprime[n], int(d[s]))
            r = residual(p_n, qprime_full(q_rows[s], dmap, tmap, ngram))
            if r.sum() <= 0.0:
                out["flags"][b] |= FLAG_RESID_ZERO
                r = p_n
        _, u2 = uniforms(seed, seq_id[b], step, n)
        v, margin, neighbors = sample_inverse_cdf(r, u2)
        out["out_tokens"][r0 + n] = v
        out["cdf_margin"][b] = margin
        out["cdf_neighbors"][b] = neighbors
    return out


def verify_case(case, **kw) -> dict:
    """Convenience: run verify_step on a workloads.VerifyCase."""
    cache = build_cache(case.ngram_key_off, case.ngram_key_ids, case.ngram_target_ids)
    return verify_step(row_off=case.row_off, draft_ids=case.draft_ids, draft_logits=case.draft_logits,
                       direct_map=case.direct_map, V_t=case.V_t, cache=cache, max_ngram_len=case.max_ngram_len,
                       temperature=case.temperature, draft_temperature=case.draft_temperature, seed=case.seed,
                       seq_id=case.seq_id, step=case.step, dtype=case.dtype, hidden=case.hidden, W=case.W,
                       target_logits=case.target_logits, **kw)
