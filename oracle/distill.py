"""CPU oracle of the forward value of the hybrid cross-vocabulary distillation loss.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py): plain NumPy float64, no shared code with the HIP path.

What the paper fixes (Section "Cross-vocabulary Distillation", the loss equation):

    L = L_DM + lambda * L_N-gram
      = E_{d_i ~ q} [ D_KL(q' || p)(t_i | x) * I_DM(d_i)  -  lambda * log q(d_i | x) * I_N-gram(d_i) ]

  * on a drafted token that translates through the direct map, the reverse KL between q', the draft distribution
    lifted into the target vocabulary (Eq. 2), and the target distribution p at that position;
  * on drafted tokens that are sub-tokens of an n-gram, the negative log-likelihood under the draft model;
  * lambda is a constant (0.2 in the experiments) or the verified target probability p(t_i) of the n-gram;
  * the n-gram term may instead be the approximate KL D_KL(q' || p) with Eq. 2's two overrides (the n-gram's
    target id gets the product of sub-token probabilities, the direct image of its first sub-token the rest).

Readings taken where the paper is silent (mirrored by the library):
  * p and q are the step's own distributions (same temperatures as the verification); a sequence whose target or
    draft temperature is 0 (one-hot distributions, KL undefined) contributes nothing;
  * q' is not renormalised (as in verification); the KL sum runs over the ids with q'(v) > 0:
    sum_v q'(v) * (ln q'(v) - ln p(v));
  * the tokens considered are those the translation scan reached (an unmappable id ends it);
  * I_N-gram selects every sub-token of a proposed n-gram; with `n_accept` given only the n-grams the target
    accepted count (the paper speaks of n-grams "accepted by the target during inference");
  * the expectation is the mean over the drafted tokens considered: loss = (sum of KL terms + sum of weighted
    n-gram terms) / (number of direct tokens + number of n-gram sub-tokens); the sums and counts are returned too.
"""
from __future__ import annotations

from typing import Optional

import numpy as np

from .verify import distribution, inverse_map, lm_head_logits, map_merge, qprime_full, widen

KIND_NONE, KIND_DIRECT, KIND_NGRAM = 0, 1, 2


def reverse_kl(qp: np.ndarray, p: np.ndarray) -> float:
    """sum over {v : q'(v) > 0} of q'(v) (ln q'(v) - ln p(v)); q' need not sum to one."""
    live = qp > 0.0
    return float(np.sum(qp[live] * (np.log(qp[live]) - np.log(p[live]))))


def hybrid_loss(*, row_off, draft_ids, draft_logits, direct_map, V_t: int, cache: Optional[dict], max_ngram_len: int,
                temperature, draft_temperature=None, dtype: str, hidden=None, W=None, target_logits=None,
                lam: float = 0.2, lambda_mode: str = "fixed", ngram_term: str = "nll", n_accept=None) -> dict:
    """Forward values of the loss for one ragged batch (arguments as oracle.verify.verify_step).

    lambda_mode: "fixed" (weight lam) or "target_prob" (weight p(t_i)); ngram_term: "nll" or "approx_kl".
    Per-row outputs are indexed like the verification outputs: entry row_off[b] + j is mapped token j of sequence b.
    """
    assert lambda_mode in ("fixed", "target_prob") and ngram_term in ("nll", "approx_kl")
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
        "kind": np.zeros(M, np.int32), "kl": np.zeros(M), "nll": np.zeros(M), "weight": np.zeros(M),
        "loss_dm": 0.0, "loss_ngram": 0.0, "n_dm": 0, "n_ngram_tokens": 0, "loss": 0.0,
    }
    for b in range(B):
        r0 = int(row_off[b])
        k = int(row_off[b + 1]) - r0 - 1
        q0 = r0 - b
        d = np.asarray(draft_ids[q0:q0 + k], dtype=np.int64)
        T = float(temperature[b])
        Td = T if draft_temperature is None else float(draft_temperature[b])
        if T <= 0.0 or Td <= 0.0 or np.any(d < 0) or np.any(d >= V_d):
            continue
        q_rows = [distribution(Zq[q0 + i], Td) for i in range(k)]
        tokens, spans, _, _ = map_merge(d, dmap, cache, max_ngram_len)
        for j, (t, (s, L)) in enumerate(zip(tokens, spans)):
            p_j = distribution(Z[r0 + j], T)
            if L == 1:
                out["kind"][r0 + j] = KIND_DIRECT
                out["kl"][r0 + j] = reverse_kl(qprime_full(q_rows[s], dmap, tmap, None), p_j)
                out["loss_dm"] += out["kl"][r0 + j]
                out["n_dm"] += 1
                continue
            if n_accept is not None and j >= int(n_accept[b]):
                continue
            out["kind"][r0 + j] = KIND_NGRAM
            logq = [float(np.log(q_rows[s + l][int(d[s + l])])) for l in range(L)]
            out["nll"][r0 + j] = -sum(logq)
            w = lam if lambda_mode == "fixed" else float(p_j[t])
            out["weight"][r0 + j] = w
            if ngram_term == "nll":
                term = out["nll"][r0 + j]
            else:
                pi = float(np.prod([q_rows[s + l][int(d[s + l])] for l in range(L)]))
                out["kl"][r0 + j] = reverse_kl(qprime_full(q_rows[s], dmap, tmap, (t, pi, int(d[s]))), p_j)
                term = out["kl"][r0 + j]
            out["loss_ngram"] += w * term
            out["n_ngram_tokens"] += L
    n = out["n_dm"] + out["n_ngram_tokens"]
    out["loss"] = (out["loss_dm"] + out["loss_ngram"]) / max(1, n)
    return out


def hybrid_loss_case(case, **kw) -> dict:
    """Convenience: run hybrid_loss on a workloads.VerifyCase."""
    from .verify import build_cache
    cache = build_cache(case.ngram_key_off, case.ngram_key_ids, case.ngram_target_ids)
    return hybrid_loss(row_off=case.row_off, draft_ids=case.draft_ids, draft_logits=case.draft_logits,
                       direct_map=case.direct_map, V_t=case.V_t, cache=cache, max_ngram_len=case.max_ngram_len,
                       temperature=case.temperature, draft_temperature=case.draft_temperature, dtype=case.dtype,
                       hidden=case.hidden, W=case.W, target_logits=case.target_logits, **kw)
