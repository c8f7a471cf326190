"""CPU oracle of the adaptive-drafting stop rule and of the acceptance head's loss value.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py): plain NumPy float64, no shared code with the HIP path.

What the paper fixes (Section "Online Adaptive Drafting", the three-line equation after it, and the appendix on
online adaptive drafting training):
  * a head f_phi maps the embedding e_i of proposed token i to a logit; P(y_i accepted | y_<i accepted) =
    sigmoid(f_phi(e_i));
  * P(some y_i', i' <= i, rejected) = 1 - prod_{i' <= i} sigmoid(f_phi(e_i')); drafting exits once it exceeds gamma;
  * the head is trained with a weighted binary cross-entropy against the labels min(1, p(y_i) / q(y_i)).

Readings taken where the paper is silent (mirrored by the library):
  * the head itself (its layers) belongs to the drafter and is not modelled: its logits are the input;
  * the rule is evaluated after every proposed token, so the proposal keeps the token that tipped the product over
    gamma: n_keep = min{i >= 1 : 1 - prod_{i' <= i} sigmoid > gamma}, or all k tokens if that never happens;
  * "weighted": one weight on the accept side and one on the reject side of the cross-entropy (SpecDec++, which
    the paper adopts, up-weights rejections):
        bce_i = -( w_accept * l_i * ln sigmoid(a_i) + w_reject * (1 - l_i) * ln(1 - sigmoid(a_i)) );
    the value is the mean over the labelled positions, and the sum and the count are returned beside it.
"""
from __future__ import annotations

import numpy as np


def sigmoid(a: np.ndarray) -> np.ndarray:
    return 1.0 / (1.0 + np.exp(-np.asarray(a, dtype=np.float64)))


def stop_rule(*, row_off, head_logits, gamma: float, n_valid=None) -> dict:
    """Per row (entry row_off[b] + i is proposed token i of sequence b): p_accept, p_any_reject; per sequence n_keep.

    n_valid[b] (default k_b): only the first n_valid[b] tokens of sequence b exist for the rule.
    """
    row_off = np.asarray(row_off, dtype=np.int64)
    B = row_off.size - 1
    M = int(row_off[-1])
    a = np.asarray(head_logits, dtype=np.float32).astype(np.float64)
    out = {"p_accept": np.zeros(M), "p_any_reject": np.zeros(M), "n_keep": np.zeros(B, np.int32),
           "stop_margin": np.full(B, np.inf)}
    g = float(np.float32(gamma))
    for b in range(B):
        r0 = int(row_off[b])
        k = int(row_off[b + 1]) - r0 - 1
        n = k if n_valid is None else min(k, int(n_valid[b]))
        keep = n
        alive = 1.0                                  # probability that every token so far is accepted
        for i in range(n):
            s = float(sigmoid(a[r0 + i]))
            alive *= s
            out["p_accept"][r0 + i] = s
            out["p_any_reject"][r0 + i] = 1.0 - alive
            out["stop_margin"][b] = min(out["stop_margin"][b], abs((1.0 - alive) - g))
            if keep == n and 1.0 - alive > g:
                keep = i + 1
        out["n_keep"][b] = keep
    return out


def weighted_bce(*, row_off, head_logits, labels, w_accept: float = 1.0, w_reject: float = 1.0, n_valid=None) -> dict:
    """Weighted binary cross-entropy of the head's logits against acceptance-ratio labels in [0, 1]."""
    row_off = np.asarray(row_off, dtype=np.int64)
    B = row_off.size - 1
    a = np.asarray(head_logits, dtype=np.float32).astype(np.float64)
    l = np.asarray(labels, dtype=np.float32).astype(np.float64)
    total, count = 0.0, 0
    for b in range(B):
        r0 = int(row_off[b])
        k = int(row_off[b + 1]) - r0 - 1
        n = k if n_valid is None else min(k, int(n_valid[b]))
        for i in range(n):
            x = a[r0 + i]
            # ln sigmoid(x) = -ln(1 + e^-x) and ln(1 - sigmoid(x)) = -ln(1 + e^x), written so that neither overflows
            ln_s = -(np.log1p(np.exp(-abs(x))) + max(-x, 0.0))
            ln_1ms = -(np.log1p(np.exp(-abs(x))) + max(x, 0.0))
            total += -(w_accept * l[r0 + i] * ln_s + w_reject * (1.0 - l[r0 + i]) * ln_1ms)
            count += 1
    return {"sum": total, "count": count, "mean": total / max(1, count)}
