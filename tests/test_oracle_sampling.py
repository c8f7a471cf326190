"""Pins for the oracle's acceptance rule, residual and final-token draw.

The invariants are those of speculative sampling (Leviathan et al.; Chen et al., cited by the paper's
Notation paragraph): the emitted tokens follow the target distribution p whenever q' is a proper
sub-distribution obtained through a one-to-one map.  With an n-gram in play Eq. 2 is only approximately
lossless, so there the exactly enumerated law of the algorithm is what the Monte Carlo run is held to.
"""
import itertools
from collections import defaultdict

import numpy as np
import pytest
import scipy.stats

from oracle import philox
from oracle import verify as ov
from workloads import CaseSpec, make_case


# --------------------------------------------------------------------------- exact law by enumeration
def exact_law(Z, Zq, T, dmap, cache, max_len, V_t):
    """Exact probability of every emitted token tuple: sum over all draft tuples, u integrated analytically."""
    k = Zq.shape[0]
    V_d = Zq.shape[1]
    p = [ov.distribution(Z[j], T) for j in range(k + 1)]
    q = [ov.distribution(Zq[i], T) for i in range(k)]
    tmap = ov.inverse_map(dmap, V_t)
    law = defaultdict(float)

    def spread(prefix, weight, r):
        tot = r.sum()
        for v in np.flatnonzero(r > 0):
            law[prefix + (int(v),)] += weight * r[v] / tot

    for tup in itertools.product(range(V_d), repeat=k):
        w = float(np.prod([q[i][tup[i]] for i in range(k)]))
        if w == 0.0:
            continue
        tokens, spans, unm, s_end = ov.map_merge(tup, dmap, cache, max_len)
        reach = w
        for j, (t, sp) in enumerate(zip(tokens, spans)):
            qp = ov.qprime_pointwise(q, tup, sp)
            ratio = min(1.0, p[j][t] / qp) if qp > 0 else (1.0 if p[j][t] > 0 else 0.0)
            if ratio < 1.0:
                ng = (t, qp, tup[sp[0]]) if sp[1] > 1 else None
                r = ov.residual(p[j], ov.qprime_full(q[sp[0]], dmap, tmap, ng))
                spread(tuple(tokens[:j]), reach * (1.0 - ratio), r if r.sum() > 0 else p[j])
            reach *= ratio
        m = len(tokens)
        if unm:
            r = ov.residual(p[m], ov.qprime_full(q[s_end], dmap, tmap))
            spread(tuple(tokens), reach, r if r.sum() > 0 else p[m])
        else:
            spread(tuple(tokens), reach, p[m])
    return dict(law)


def _tiny(seed, V_d, V_t, k, n_direct, bijective=False):
    rng = np.random.default_rng(seed)
    Z = rng.standard_normal((k + 1, V_t)).astype(np.float32) * 1.5
    Zq = rng.standard_normal((k, V_d)).astype(np.float32) * 1.5
    dmap = np.full(V_d, -1)
    if bijective:
        dmap[:] = rng.permutation(V_t)[:V_d]
    else:
        src = rng.choice(V_d, n_direct, replace=False)
        dmap[src] = rng.choice(V_t, n_direct, replace=False)
    return Z, Zq, dmap


def _marginal(law, pos, V_t):
    out = np.zeros(V_t)
    for tup, pr in law.items():
        if len(tup) > pos:
            out[tup[pos]] += pr
    return out


@pytest.mark.parametrize("T", [1.0, 0.6])
@pytest.mark.parametrize("bijective", [True, False])
def test_direct_map_is_exactly_lossless(T, bijective):
    """First token ~ p_0; given it was an accepted draft, the next ~ p_1; the free token ~ p_2."""
    V_d, V_t, k = (6, 6, 2) if bijective else (6, 8, 2)
    Z, Zq, dmap = _tiny(11, V_d, V_t, k, n_direct=4, bijective=bijective)
    law = exact_law(Z, Zq, T, dmap, {}, 4, V_t)
    assert sum(law.values()) == pytest.approx(1.0, abs=1e-12)
    p = [ov.distribution(Z[j], T) for j in range(k + 1)]
    np.testing.assert_allclose(_marginal(law, 0, V_t), p[0], atol=1e-12)
    for pos in (1, 2):
        marg = _marginal(law, pos, V_t)
        np.testing.assert_allclose(marg / marg.sum(), p[pos], atol=1e-12)


def test_ngram_law_is_only_approximately_p():
    """With a 2-gram in the cache the emitted law stays a distribution but deviates slightly from p (Eq. 2 text)."""
    V_d, V_t, k = 5, 7, 2
    Z, Zq, dmap = _tiny(12, V_d, V_t, k, n_direct=4)
    free = [t for t in range(V_t) if t not in set(dmap[dmap >= 0].tolist())]
    cache = {(1, 2): free[0], (3, 0): free[1]}
    law = exact_law(Z, Zq, 1.0, dmap, cache, 4, V_t)
    assert sum(law.values()) == pytest.approx(1.0, abs=1e-12)
    p0 = ov.distribution(Z[0], 1.0)
    dev = np.abs(_marginal(law, 0, V_t) - p0).max()
    assert 1e-6 < dev < 0.2


# --------------------------------------------------------------------------- Monte Carlo of verify_step vs the exact law
def _monte_carlo(Z, Zq, T, dmap, cache, max_len, V_t, n_draws, seed):
    rng = np.random.default_rng(seed)
    k, V_d = Zq.shape
    q = [ov.distribution(Zq[i], T) for i in range(k)]
    counts = defaultdict(int)
    ids = np.stack([rng.choice(V_d, size=n_draws, p=q[i]) for i in range(k)], axis=1)
    for it in range(n_draws):
        o = ov.verify_step(row_off=[0, k + 1], draft_ids=ids[it], draft_logits=Zq, direct_map=dmap, V_t=V_t,
                           cache=cache, max_ngram_len=max_len, temperature=[T], seed=99, seq_id=[5], step=it,
                           dtype="f32", target_logits=Z)
        counts[tuple(int(t) for t in o["out_tokens"][:o["n_emit"][0]])] += 1
    return counts


def _chi2_pvalue(counts, law, n):
    keys = sorted(law, key=lambda t: -law[t])
    assert set(counts) <= set(law), "the step emitted a tuple the exact law gives probability zero"
    exp, obs, acc_e, acc_o = [], [], 0.0, 0
    for t in keys:                                   # pool the tail so every cell expects >= 8
        acc_e += law[t] * n
        acc_o += counts.get(t, 0)
        if acc_e >= 8:
            exp.append(acc_e), obs.append(acc_o)
            acc_e, acc_o = 0.0, 0
    if acc_e > 0:
        exp[-1] += acc_e
        obs[-1] += acc_o
    exp, obs = np.array(exp), np.array(obs)
    stat = ((obs - exp) ** 2 / exp).sum()
    return scipy.stats.chi2.sf(stat, len(exp) - 1)


@pytest.mark.parametrize("scenario", ["bijective", "partial", "ngram"])
def test_monte_carlo_matches_exact_law(scenario):
    n = 40_000
    if scenario == "bijective":
        V_d, V_t, k = 5, 5, 2
        Z, Zq, dmap = _tiny(21, V_d, V_t, k, 0, bijective=True)
        cache = {}
    elif scenario == "partial":
        V_d, V_t, k = 5, 7, 2
        Z, Zq, dmap = _tiny(22, V_d, V_t, k, n_direct=3)
        cache = {}
    else:
        V_d, V_t, k = 4, 7, 3
        Z, Zq, dmap = _tiny(23, V_d, V_t, k, n_direct=3)
        free = [t for t in range(V_t) if t not in set(dmap[dmap >= 0].tolist())]
        cache = {(0, 1): free[0], (2, 2, 3): free[1], (1, 3): free[2]}
    law = exact_law(Z, Zq, 0.9, dmap, cache, 4, V_t)
    counts = _monte_carlo(Z, Zq, 0.9, dmap, cache, 4, V_t, n, seed=7)
    assert _chi2_pvalue(counts, law, n) > 1e-3
    # a deliberately wrong law (target rows swapped) must be rejected by the same statistic: the test has power
    wrong = exact_law(Z[::-1].copy(), Zq, 0.9, dmap, cache, 4, V_t)
    if set(counts) <= set(wrong):
        assert _chi2_pvalue(counts, wrong, n) < 1e-6


# --------------------------------------------------------------------------- invariants on verify_step
def _step(Z, Zq, ids, dmap, T, cache=None, Td=None, step=0, k_list=None, seed=3):
    k_list = k_list or [len(ids)]
    row_off = np.concatenate([[0], np.cumsum(np.array(k_list) + 1)])
    B = len(k_list)
    return ov.verify_step(row_off=row_off, draft_ids=np.asarray(ids), draft_logits=Zq, direct_map=dmap,
                          V_t=Z.shape[1], cache=cache, max_ngram_len=4, temperature=[T] * B if np.isscalar(T) else T,
                          draft_temperature=Td, seed=seed, seq_id=np.arange(B), step=step, dtype="f32",
                          target_logits=Z)


def test_q_equals_p_accepts_everything_then_free_token():
    rng = np.random.default_rng(31)
    V, k = 50, 6
    Z = rng.standard_normal((k + 1, V)).astype(np.float32) * 2
    Zq = Z[:k].copy()                                   # drafter == target, identity map
    for step in range(50):
        ids = rng.integers(0, V, size=k)
        o = _step(Z, Zq, ids, np.arange(V), 1.0, step=step)
        assert o["n_accept"][0] == k and o["n_emit"][0] == k + 1 and o["flags"][0] == 0
        assert np.all(o["ratio"][:k] == 1.0)
        assert o["out_tokens"][:k].tolist() == ids.tolist()
        assert 0 <= o["out_tokens"][k] < V


def test_free_token_follows_p_by_inverse_cdf():
    """k = 0: the only output is a draw from p_0; the draw is the inverse CDF at the second Philox word."""
    rng = np.random.default_rng(32)
    V = 9
    Z = rng.standard_normal((1, V)).astype(np.float32)
    p = ov.distribution(Z[0].astype(np.float64), 1.0)
    edges = np.concatenate([[0.0], np.cumsum(p)])
    for step in range(200):
        o = _step(Z, np.zeros((0, 4), np.float32), [], np.arange(4), 1.0, step=step)
        _, u2 = philox.uniforms(3, 0, step, 0)
        v = int(o["out_tokens"][0])
        assert o["n_emit"][0] == 1 and edges[v] <= u2 * edges[-1] < edges[v + 1]


def test_residual_properties():
    rng = np.random.default_rng(33)
    p = rng.dirichlet(np.ones(30))
    qp = rng.dirichlet(np.ones(30)) * 0.8
    r = ov.residual(p, qp)
    assert np.all(r[qp >= p] == 0) and np.all(r >= 0)
    assert (r / r.sum()).sum() == pytest.approx(1.0, abs=1e-14)
    # total mass of the residual is 1 - sum(min(p, q')) + (1 - 1) ... i.e. sum(p) - sum(min(p, q'))
    assert r.sum() == pytest.approx(1.0 - np.minimum(p, qp).sum(), abs=1e-14)


def test_inverse_cdf_picks_the_right_cell_and_skips_zero_mass():
    r = np.array([0.0, 0.2, 0.0, 0.0, 0.5, 0.3, 0.0])
    for u, want in [(0.0, 1), (0.1999, 1), (0.2, 4), (0.6999, 4), (0.7, 5), (0.999999, 5)]:
        assert ov.sample_inverse_cdf(r, u)[0] == want
    v, margin, nb = ov.sample_inverse_cdf(r, 0.45)
    assert v == 4 and margin == pytest.approx(0.25) and nb == (1, 5)


def test_temperature_zero_is_argmax_match():
    rng = np.random.default_rng(34)
    V, k = 40, 5
    Z = rng.standard_normal((k + 1, V)).astype(np.float32)
    am = Z.argmax(axis=1)
    dmap = rng.permutation(V)
    inv = np.argsort(dmap)
    Zq = rng.standard_normal((k, V)).astype(np.float32)
    for n_good in range(k + 1):
        ids = inv[am[:k]].copy()                        # drafts whose images are the target argmaxes
        if n_good < k:
            ids[n_good] = inv[(am[n_good] + 1) % V]     # first mismatch at n_good
        o = _step(Z, Zq, ids, dmap, 0.0)
        assert o["n_accept"][0] == n_good and o["n_emit"][0] == n_good + 1
        assert o["out_tokens"][:n_good + 1].tolist() == am[:n_good + 1].tolist()
        assert np.all(np.isinf(o["u_margin"]))          # no uniforms consumed


def test_low_temperature_tends_to_greedy():
    rng = np.random.default_rng(35)
    V, k = 30, 3
    Z = rng.standard_normal((k + 1, V)).astype(np.float32) * 3
    Zq = rng.standard_normal((k, V)).astype(np.float32) * 3
    ids = Zq.argmax(axis=1)
    a = _step(Z, Zq, ids, np.arange(V), 0.0)
    b = _step(Z, Zq, ids, np.arange(V), 1e-3)
    assert a["out_tokens"].tolist() == b["out_tokens"].tolist() and a["n_accept"][0] == b["n_accept"][0]


def test_unmappable_first_token_draws_from_residual_of_that_position():
    rng = np.random.default_rng(36)
    V_d, V_t = 6, 8
    Z = rng.standard_normal((3, V_t)).astype(np.float32)
    Zq = rng.standard_normal((2, V_d)).astype(np.float32)
    dmap = np.array([0, 1, 2, -1, 4, 5])
    o = _step(Z, Zq, [3, 1], dmap, 1.0)
    assert o["n_mapped"][0] == 0 and o["n_accept"][0] == 0 and o["n_emit"][0] == 1
    assert o["flags"][0] == ov.FLAG_UNMAPPABLE
    p0 = ov.distribution(Z[0], 1.0)
    q0 = ov.distribution(Zq[0], 1.0)
    r = ov.residual(p0, ov.qprime_full(q0, dmap, ov.inverse_map(dmap, V_t)))
    _, u2 = philox.uniforms(3, 0, 0, 0)
    assert o["out_tokens"][0] == ov.sample_inverse_cdf(r, u2)[0]


def test_zero_residual_falls_back_to_p_and_is_flagged():
    """In exact arithmetic a residual of zero mass cannot occur; with underflow it can: p and q' both collapse
    to the same one-hot while the drafted id (probability 0 under q) has no image, which forces the residual path."""
    V_d, V_t = 4, 5
    Z = np.zeros((2, V_t), np.float32)
    Z[0, 1] = 2000.0                                    # p_0 is exactly one-hot at target id 1
    Zq = np.zeros((1, V_d), np.float32)
    Zq[0, 2] = 2000.0                                   # q_0 is exactly one-hot at draft id 2 ...
    dmap = np.array([0, -1, 1, 3])                      # ... whose image is target id 1; draft id 1 has no image
    o = _step(Z, Zq, [1], dmap, 1.0)
    assert o["n_mapped"][0] == 0 and o["flags"][0] == (ov.FLAG_UNMAPPABLE | ov.FLAG_RESID_ZERO)
    assert o["n_emit"][0] == 1 and o["out_tokens"][0] == 1          # drawn from p, which is one-hot


def test_bad_draft_id_emits_nothing():
    Z = np.zeros((3, 5), np.float32)
    Zq = np.zeros((2, 4), np.float32)
    for bad in (-1, 4, 1000):
        o = _step(Z, Zq, [1, bad], np.arange(4), 1.0)
        assert o["flags"][0] == ov.FLAG_BAD_ID and o["n_emit"][0] == 0 and np.all(o["out_tokens"] == -1)


def test_ragged_batch_rows_and_streams_are_independent():
    """A sequence's result does not depend on its neighbours, only on its own seq_id stream."""
    spec = CaseSpec(name="ragged", dtype="f32", d=16, V_t=300, V_d=120, k=[3, 0, 5, 1], temperature=[1.0, 0.8, 0.0, 1.0],
                    n_direct=90, n_ngram=40, ngram_len=(2, 3), plant_cover=0.4, align=0.6, data_seed=5, philox_seed=9,
                    logits_only=True)
    c = make_case(spec)
    full = ov.verify_case(c)
    cache = ov.build_cache(c.ngram_key_off, c.ngram_key_ids, c.ngram_target_ids)
    for b in range(c.B):
        r0, r1 = int(c.row_off[b]), int(c.row_off[b + 1])
        q0 = r0 - b
        one = ov.verify_step(row_off=[0, r1 - r0], draft_ids=c.draft_ids[q0:q0 + c.k[b]],
                             draft_logits=c.draft_logits[q0:q0 + c.k[b]], direct_map=c.direct_map, V_t=c.V_t,
                             cache=cache, max_ngram_len=c.max_ngram_len, temperature=c.temperature[b:b + 1],
                             seed=c.seed, seq_id=c.seq_id[b:b + 1], step=c.step, dtype="f32",
                             target_logits=c.target_logits[r0:r1])
        assert one["out_tokens"].tolist() == full["out_tokens"][r0:r1].tolist()
        for key in ("n_mapped", "n_accept", "n_accept_draft", "n_emit", "hits_proposed", "hits_accepted", "flags"):
            assert one[key][0] == full[key][b]
    assert full["n_emit"].min() >= 1


def test_counts_are_consistent_on_an_agreeable_batch():
    spec = CaseSpec(name="agree", dtype="f32", d=16, V_t=500, V_d=200, k=[6] * 40, temperature=[1.0] * 40,
                    n_direct=150, n_ngram=60, ngram_len=(2, 4), plant_cover=0.4, align=0.85, data_seed=6,
                    philox_seed=10, logits_only=True)
    c = make_case(spec)
    o = ov.verify_case(c)
    assert o["n_accept"].max() >= 3 and (o["n_accept"] == o["n_mapped"]).any() and o["hits_accepted"].sum() > 0
    for b in range(c.B):
        r0 = int(c.row_off[b])
        n, m = int(o["n_accept"][b]), int(o["n_mapped"][b])
        assert 0 <= n <= m <= c.k[b] and o["n_emit"][b] == n + 1
        L = o["span_len"][r0:r0 + m]
        assert o["n_accept_draft"][b] == L[:n].sum()
        assert o["hits_proposed"][b] == (L > 1).sum() and o["hits_accepted"][b] == (L[:n] > 1).sum()
        assert np.all(o["out_tokens"][r0:r0 + n] == o["mapped_ids"][r0:r0 + n])
        assert np.all(o["out_tokens"][r0 + n + 1:r0 + c.k[b] + 1] == -1)
        starts = o["span_start"][r0:r0 + m]
        assert np.array_equal(starts, np.concatenate([[0], np.cumsum(L)[:-1]])[:m])
        # q' of an n-gram is the product of its sub-token probabilities (Eq. 1), ratio = min(1, p/q')
        np.testing.assert_allclose(o["ratio"][r0:r0 + m],
                                   np.minimum(1.0, o["p_tok"][r0:r0 + m] / o["q_tok"][r0:r0 + m]), rtol=1e-12)
