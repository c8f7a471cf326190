"""Pins for the oracle of the adaptive-drafting stop rule and the acceptance head's weighted BCE."""
import math

import numpy as np
import pytest
import scipy.special

from oracle import adaptive as oa


def test_stop_rule_closed_forms():
    # logit 0 everywhere: sigmoid = 1/2, so P(some rejection among the first i) = 1 - 2^-i
    out = oa.stop_rule(row_off=[0, 7], head_logits=np.zeros(7), gamma=0.8)
    assert out["p_accept"][:6].tolist() == [0.5] * 6
    assert out["p_any_reject"][:6].tolist() == [1 - 0.5 ** i for i in range(1, 7)]
    assert out["n_keep"].tolist() == [3]             # 0.5, 0.75, 0.875 > 0.8: the third token tips it and is kept
    assert oa.stop_rule(row_off=[0, 7], head_logits=np.zeros(7), gamma=0.3)["n_keep"].tolist() == [1]
    # a confident head never stops; a threshold of 1 can never be exceeded
    assert oa.stop_rule(row_off=[0, 7], head_logits=np.full(7, 30.0), gamma=0.3)["n_keep"].tolist() == [6]
    assert oa.stop_rule(row_off=[0, 7], head_logits=np.full(7, -3.0), gamma=1.0)["n_keep"].tolist() == [6]
    # strict inequality: 1 - 1/2 is not > 1/2
    assert oa.stop_rule(row_off=[0, 3], head_logits=np.zeros(3), gamma=0.5)["n_keep"].tolist() == [2]


def test_stop_rule_against_library_sigmoid_and_cumprod():
    rng = np.random.default_rng(7)
    k = [5, 0, 9, 1, 12]
    row_off = np.concatenate([[0], np.cumsum(np.array(k) + 1)])
    a = rng.standard_normal(row_off[-1]).astype(np.float32) * 2 + 1
    out = oa.stop_rule(row_off=row_off, head_logits=a, gamma=0.6)
    for b, kb in enumerate(k):
        r0 = row_off[b]
        s = scipy.special.expit(a[r0:r0 + kb].astype(np.float64))
        np.testing.assert_allclose(out["p_accept"][r0:r0 + kb], s, rtol=1e-15)
        rej = 1.0 - np.cumprod(s)
        np.testing.assert_allclose(out["p_any_reject"][r0:r0 + kb], rej, rtol=1e-14, atol=1e-16)
        assert np.all(np.diff(out["p_any_reject"][r0:r0 + kb]) >= 0)          # more tokens, more chances to fail
        over = np.flatnonzero(rej > np.float32(0.6))
        assert out["n_keep"][b] == (over[0] + 1 if over.size else kb)
        assert out["p_accept"][r0 + kb] == 0.0                                # the bonus row carries nothing
    # n_valid shortens the window
    short = oa.stop_rule(row_off=row_off, head_logits=a, gamma=0.999999, n_valid=[2, 0, 3, 1, 4])
    assert short["n_keep"].tolist() == [2, 0, 3, 1, 4]


def test_weighted_bce_against_library_log_sigmoid():
    rng = np.random.default_rng(8)
    k = [4, 6, 0, 3]
    row_off = np.concatenate([[0], np.cumsum(np.array(k) + 1)])
    a = (rng.standard_normal(row_off[-1]) * 4).astype(np.float32)
    l = rng.uniform(0, 1, row_off[-1]).astype(np.float32)
    l[1], l[2] = 1.0, 0.0
    got = oa.weighted_bce(row_off=row_off, head_logits=a, labels=l, w_accept=1.0, w_reject=6.0)
    want, n = 0.0, 0
    for b, kb in enumerate(k):
        for i in range(kb):
            x, y = float(a[row_off[b] + i]), float(l[row_off[b] + i])
            want += -(y * scipy.special.log_expit(x) + 6.0 * (1 - y) * scipy.special.log_expit(-x))
            n += 1
    assert got["count"] == n == 13
    assert got["sum"] == pytest.approx(want, rel=1e-13)
    assert got["mean"] == pytest.approx(want / n, rel=1e-13)


def test_weighted_bce_closed_forms_and_extremes():
    # logit 0: both sides cost ln 2 whatever the label, so the weights add up
    one = oa.weighted_bce(row_off=[0, 4], head_logits=np.zeros(4), labels=[0.25, 1.0, 0.0, 0.5], w_accept=2.0, w_reject=3.0)
    assert one["sum"] == pytest.approx(math.log(2) * (2 * 0.25 + 3 * 0.75 + 2 * 1 + 3 * 1), rel=1e-14)
    # a perfect confident head costs (almost) nothing, a confidently wrong one about |logit| per token; no overflow
    good = oa.weighted_bce(row_off=[0, 3], head_logits=[80.0, -80.0, 0.0], labels=[1.0, 0.0, 0.0])
    assert 0.0 <= good["sum"] < 1e-30
    bad = oa.weighted_bce(row_off=[0, 3], head_logits=[-80.0, 80.0, 0.0], labels=[1.0, 0.0, 0.0])
    assert bad["sum"] == pytest.approx(160.0, rel=1e-12)
    # minimiser: for a soft label l the unweighted cost is smallest at sigmoid(a) = l
    l = 0.3
    grid = np.linspace(-3, 3, 601).astype(np.float32)
    costs = [oa.weighted_bce(row_off=[0, 2], head_logits=[x, 0.0], labels=[l, 0.0])["sum"] for x in grid]
    assert abs(scipy.special.expit(float(grid[int(np.argmin(costs))])) - l) < 0.003
