"""Pins for the oracle of the hybrid distillation loss (forward values)."""
import math
import os

import numpy as np
import pytest
import scipy.special
import scipy.stats

from oracle import distill as od
from oracle import verify as ov
from workloads import CaseSpec, make_case

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _gold():
    vals = {}
    with open(os.path.join(GOLD, "hybrid_loss_worked_example.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            key, rest = line.split(None, 1)
            vals[key] = rest.split()
    return vals


def _worked_inputs():
    g = _gold()
    dmap = np.array([int(x) for x in g["dmap"]])
    cache = {(int(g["cache"][0]), int(g["cache"][1])): int(g["cache"][3])}
    q0 = np.array([float(x) for x in g["q0"]])
    q1 = np.array([float(x) for x in g["q1"]])
    p = np.array([float(x) for x in g["p"]])
    # logits = ln(probability) at temperature 1 reproduce the distributions exactly (up to rounding)
    draft_logits = np.log(np.stack([q0, q1, q0])).astype(np.float64)
    target_logits = np.tile(np.log(p), (5, 1))
    return g, dict(row_off=[0, 3, 5], draft_ids=[1, 2, 0], draft_logits=draft_logits, direct_map=dmap, V_t=5, cache=cache,
                   max_ngram_len=4, temperature=[1.0, 1.0], dtype="f64", target_logits=target_logits)


@pytest.fixture(autouse=True)
def _f64_logits(monkeypatch):
    # the worked example feeds float64 draft logits straight through (the production dtypes round ln(0.3) etc.);
    # the target logits are rounded to float32 as at the library's interface, which the example tolerates (1e-7)
    real_widen = ov.widen
    monkeypatch.setattr(od, "widen", lambda x, dtype: np.asarray(x, np.float64) if dtype == "f64" else real_widen(x, dtype))


def test_worked_example():
    g, kw = _worked_inputs()
    out = od.hybrid_loss(**kw, lam=0.2)
    assert out["kind"].tolist() == [od.KIND_NGRAM, 0, 0, od.KIND_DIRECT, 0]
    assert out["nll"][0] == pytest.approx(float(g["nll_A"][0]), rel=1e-12)
    assert out["kl"][3] == pytest.approx(float(g["kl_B"][0]), rel=1e-6)
    assert (out["n_dm"], out["n_ngram_tokens"]) == (1, 2)
    assert out["loss"] == pytest.approx(float(g["loss_fixed"][0]), rel=1e-6)
    dyn = od.hybrid_loss(**kw, lambda_mode="target_prob")
    assert dyn["weight"][0] == pytest.approx(float(g["weight_A"][0]), rel=1e-6)
    assert dyn["loss_ngram"] == pytest.approx(float(g["weight_A"][0]) * float(g["nll_A"][0]), rel=1e-6)
    akl = od.hybrid_loss(**kw, ngram_term="approx_kl", lam=1.0)
    assert akl["kl"][0] == pytest.approx(float(g["approxkl_A"][0]), rel=1e-6)
    assert akl["loss_ngram"] == pytest.approx(float(g["approxkl_A"][0]), rel=1e-6)


def _case(seed, **over):
    kw = dict(name="distill", dtype="f32", d=16, V_t=300, V_d=120, k=[5, 3, 6, 0, 4], temperature=[1.0, 0.7, 1.3, 1.0, 1.0],
              n_direct=90, n_ngram=60, ngram_len=(2, 3), plant_cover=0.5, data_seed=seed, philox_seed=1, logits_only=True)
    kw.update(over)
    return make_case(CaseSpec(**kw))


def test_identical_models_give_zero_kl():
    """V_d == V_t, identity map, draft logits == target logits at the same temperature: q' = p, so every KL is 0."""
    rng = np.random.default_rng(3)
    V, k = 50, 4
    Z = rng.standard_normal((k + 1, V)).astype(np.float32)
    out = od.hybrid_loss(row_off=[0, k + 1], draft_ids=rng.integers(0, V, k), draft_logits=Z[:k], direct_map=np.arange(V), V_t=V,
                         cache={}, max_ngram_len=4, temperature=[0.8], dtype="f32", target_logits=Z)
    assert out["n_dm"] == k and out["n_ngram_tokens"] == 0
    assert np.all(np.abs(out["kl"]) < 1e-14) and abs(out["loss"]) < 1e-14


def test_bijective_map_kl_is_the_library_relative_entropy_and_nonnegative():
    rng = np.random.default_rng(4)
    V, k = 40, 6
    perm = rng.permutation(V)                                 # draft id dd <-> target id perm[dd]
    Z = rng.standard_normal((k + 1, V)).astype(np.float32) * 2
    Zq = rng.standard_normal((k, V)).astype(np.float32) * 2
    d = rng.integers(0, V, k)
    out = od.hybrid_loss(row_off=[0, k + 1], draft_ids=d, draft_logits=Zq, direct_map=perm, V_t=V, cache={}, max_ngram_len=4,
                         temperature=[1.0], draft_temperature=[0.6], dtype="f32", target_logits=Z)
    for j in range(k):
        q = scipy.special.softmax(Zq[j].astype(np.float64) / 0.6)
        p = scipy.special.softmax(Z[j].astype(np.float64))
        lifted = np.zeros(V)
        lifted[perm] = q                                      # forward scatter, the definition of the lifted distribution
        assert out["kl"][j] == pytest.approx(scipy.stats.entropy(lifted, p), rel=1e-10)
        assert out["kl"][j] >= 0.0


def test_partial_map_is_not_renormalised():
    """With mass s = sum q' < 1: sum q' ln(q'/p) = s * KL(q'/s || p) + s ln s (may be negative)."""
    case = _case(11, n_ngram=0)
    out = od.hybrid_loss_case(case)
    Zq = case.draft_logits.astype(np.float64)
    checked = 0
    for b in range(case.B):
        r0, q0 = case.row_off[b], case.row_off[b] - b
        for j in range(case.row_off[b + 1] - r0 - 1):
            if out["kind"][r0 + j] != od.KIND_DIRECT:
                continue
            q = scipy.special.softmax(Zq[q0 + j] / case.temperature[b])
            p = scipy.special.softmax(case.target_logits[r0 + j].astype(np.float64) / case.temperature[b])
            lifted = np.zeros(case.V_t)
            for dd in range(case.V_d):
                if case.direct_map[dd] >= 0:
                    lifted[case.direct_map[dd]] += q[dd]
            s = lifted.sum()
            assert s < 1.0
            assert out["kl"][r0 + j] == pytest.approx(s * scipy.stats.entropy(lifted / s, p) + s * math.log(s), rel=1e-9, abs=1e-12)
            checked += 1
    assert checked >= 5


def test_ngram_nll_is_the_library_log_softmax_and_uniform_closed_form():
    case = _case(12)
    out = od.hybrid_loss_case(case)
    ref = ov.verify_case(case)
    Zq = case.draft_logits.astype(np.float64)
    seen = 0
    for b in range(case.B):
        r0, q0 = case.row_off[b], case.row_off[b] - b
        for j in range(ref["n_mapped"][b]):
            s, L = ref["span_start"][r0 + j], ref["span_len"][r0 + j]
            if L < 2:
                assert out["kind"][r0 + j] == od.KIND_DIRECT and out["nll"][r0 + j] == 0.0
                continue
            want = -sum(scipy.special.log_softmax(Zq[q0 + s + l] / case.temperature[b])[case.draft_ids[q0 + s + l]] for l in range(L))
            assert out["kind"][r0 + j] == od.KIND_NGRAM
            assert out["nll"][r0 + j] == pytest.approx(want, rel=1e-12)
            assert out["weight"][r0 + j] == 0.2
            seen += 1
    assert seen >= 3
    assert out["n_dm"] + out["n_ngram_tokens"] == sum(int(ref["span_len"][r].sum()) for r in [slice(None)])
    # uniform draft model: every sub-token costs ln V_d
    V_d = 64
    flat = od.hybrid_loss(row_off=[0, 4], draft_ids=[5, 6, 7], draft_logits=np.zeros((3, V_d), np.float32), direct_map=np.arange(V_d),
                          V_t=V_d + 1, cache={(5, 6, 7): V_d}, max_ngram_len=4, temperature=[1.0], dtype="f32",
                          target_logits=np.zeros((4, V_d + 1), np.float32))
    assert flat["nll"][0] == pytest.approx(3 * math.log(V_d), rel=1e-14)
    assert flat["loss"] == pytest.approx(0.2 * 3 * math.log(V_d) / 3, rel=1e-14)


def test_dynamic_lambda_is_the_verified_target_probability():
    case = _case(13, n_direct=120, plant_cover=0.7, k=[6, 6, 6, 6, 6])
    dyn = od.hybrid_loss_case(case, lambda_mode="target_prob")
    ref = ov.verify_case(case)
    ng = dyn["kind"] == od.KIND_NGRAM
    assert ng.sum() >= 3
    np.testing.assert_allclose(dyn["weight"][ng], ref["p_tok"][ng], rtol=1e-12)
    assert dyn["loss_ngram"] == pytest.approx(float(np.sum(ref["p_tok"][ng] * dyn["nll"][ng])), rel=1e-12)


def test_approximate_kl_by_brute_force_scatter():
    """Eq. 2 built the other way round (loop over draft ids, scatter forward, then the two overrides), tiny vocabularies."""
    case = _case(14, V_t=60, V_d=25, n_direct=18, n_ngram=30, plant_cover=0.7, k=[4, 4, 4, 4], temperature=[1.0, 0.7, 1.3, 1.0])
    out = od.hybrid_loss_case(case, ngram_term="approx_kl", lam=1.0)
    ref = ov.verify_case(case)
    Zq = case.draft_logits.astype(np.float64)
    seen = 0
    for b in range(case.B):
        r0, q0 = case.row_off[b], case.row_off[b] - b
        T = case.temperature[b]
        for j in range(ref["n_mapped"][b]):
            s, L = ref["span_start"][r0 + j], ref["span_len"][r0 + j]
            if L < 2:
                continue
            qs = [scipy.special.softmax(Zq[q0 + s + l] / T) for l in range(L)]
            ids = [int(case.draft_ids[q0 + s + l]) for l in range(L)]
            pi = math.prod(qs[l][ids[l]] for l in range(L))
            qp = [0.0] * case.V_t
            for dd in range(case.V_d):
                if case.direct_map[dd] >= 0:
                    qp[case.direct_map[dd]] = qs[0][dd]
            if case.direct_map[ids[0]] >= 0:
                qp[case.direct_map[ids[0]]] = qs[0][ids[0]] - pi
            qp[ref["mapped_ids"][r0 + j]] = pi
            p = scipy.special.softmax(case.target_logits[r0 + j].astype(np.float64) / T)
            want = sum(qp[v] * math.log(qp[v] / p[v]) for v in range(case.V_t) if qp[v] > 0.0)
            assert out["kl"][r0 + j] == pytest.approx(want, rel=1e-9, abs=1e-13)
            seen += 1
    assert seen >= 2


def test_masks_accepted_only_and_greedy_sequences_are_skipped():
    case = _case(15)
    ref = ov.verify_case(case)
    everything = od.hybrid_loss_case(case)
    accepted = od.hybrid_loss_case(case, n_accept=ref["n_accept"])
    assert accepted["n_dm"] == everything["n_dm"]                       # the direct-mapping term ignores acceptance
    for b in range(case.B):
        r0 = case.row_off[b]
        for j in range(ref["n_mapped"][b]):
            if ref["span_len"][r0 + j] >= 2:
                assert accepted["kind"][r0 + j] == (od.KIND_NGRAM if j < ref["n_accept"][b] else od.KIND_NONE)
    greedy = _case(15, temperature=[1.0, 0.0, 1.3, 1.0, 1.0])
    out = od.hybrid_loss_case(greedy)
    r0, r1 = greedy.row_off[1], greedy.row_off[2]
    assert not out["kind"][r0:r1].any() and out["kind"].any()
    assert not out["kl"][r0:r1].any() and not out["nll"][r0:r1].any()
