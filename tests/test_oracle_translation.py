"""Pins for the oracle's LM head, distributions, translation scan (Eq. 1) and full mapping (Eq. 2)."""
import os

import numpy as np
import pytest
import scipy.special
from hypothesis import given, settings, strategies as st

from oracle import verify as ov
from workloads import f32_to_bf16_bits

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# --------------------------------------------------------------------------- LM head and softmax
def test_lm_head_brute_force_and_orientation():
    rng = np.random.default_rng(5)
    d, V, M = 7, 7, 3                        # square on purpose: a transposed W would not raise, only mis-compute
    H = rng.integers(-8, 9, size=(M, d)).astype(np.float32)
    W = rng.integers(-8, 9, size=(d, V)).astype(np.float32)
    want = np.zeros((M, V))
    for i in range(M):
        for v in range(V):
            for c in range(d):
                want[i, v] += float(H[i, c]) * float(W[c, v])
    assert np.array_equal(ov.lm_head_logits(H, W, "f32"), want)
    # small integers are exact in bfloat16, so the bf16 route must give the very same numbers
    assert np.array_equal(ov.lm_head_logits(f32_to_bf16_bits(H), f32_to_bf16_bits(W), "bf16"), want)
    # slab boundaries do not change anything
    assert np.array_equal(ov.lm_head_logits(H, W, "f32", slab=3), want)


def test_lm_head_closed_forms():
    d, V = 16, 40
    W = np.zeros((d, V), np.float32)
    W[np.arange(V) % d, np.arange(V)] = 1.0           # column v selects hidden component v % d
    H = np.arange(2 * d, dtype=np.float32).reshape(2, d)
    Z = ov.lm_head_logits(H, W, "f32")
    assert np.array_equal(Z, H[:, np.arange(V) % d].astype(np.float64))
    ones = np.ones((1, d), np.float32)
    W2 = np.random.default_rng(0).standard_normal((d, V)).astype(np.float32)
    np.testing.assert_allclose(ov.lm_head_logits(ones, W2, "f32")[0], W2.astype(np.float64).sum(axis=0), rtol=1e-14)


def test_widen_bf16_exact():
    vals = np.array([1.0, -2.5, 0.00390625, 3.0e38, -1.0e-30, 0.0], np.float32)
    bits = f32_to_bf16_bits(vals)
    w = ov.widen(bits, "bf16")
    assert w.dtype == np.float64
    # widening then re-rounding gives the same bits, and values sit within half a bf16 ulp of the source
    assert np.array_equal(f32_to_bf16_bits(w.astype(np.float32)), bits)
    np.testing.assert_allclose(w, vals.astype(np.float64), rtol=2.0 ** -8)
    assert ov.widen(np.array([0x3F80, 0xC020], np.uint16), "bf16").tolist() == [1.0, -2.5]


@pytest.mark.parametrize("T", [1.0, 0.7, 0.01, 3.0])
def test_distribution_matches_library_softmax(T):
    z = np.random.default_rng(1).standard_normal(1000) * 3.0
    np.testing.assert_allclose(ov.distribution(z, T), scipy.special.softmax(z / T), rtol=1e-12, atol=0)
    assert abs(ov.distribution(z, T).sum() - 1.0) < 1e-12


def test_distribution_temperature_zero_is_lowest_index_argmax():
    z = np.array([0.5, 2.0, -1.0, 2.0, 1.0])
    assert ov.distribution(z, 0.0).tolist() == [0, 1, 0, 0, 0]
    # and it is the T -> 0 limit of the softmax when the maximum is unique
    z2 = np.array([0.5, 2.0, -1.0, 1.9, 1.0])
    np.testing.assert_allclose(ov.distribution(z2, 1e-4), ov.distribution(z2, 0.0), atol=1e-12)


# --------------------------------------------------------------------------- scan patterns from the paper
def _patterns():
    with open(os.path.join(GOLD, "span_patterns.txt")) as f:
        return [tuple(int(x) for x in ln.split()) for ln in f if ln.strip() and not ln.startswith("#")]


@pytest.mark.parametrize("pattern", _patterns())
def test_scan_reproduces_paper_span_patterns(pattern):
    k = sum(pattern)
    d = [100 + i for i in range(k)]                 # made-up draft ids
    dmap = np.full(200, -1)
    dmap[100:100 + k] = np.arange(k) + 10           # every single token also has a direct image
    cache, s = {}, 0
    want_tokens = []
    for L in pattern:
        if L > 1:
            cache[tuple(d[s:s + L])] = 50 + s
            want_tokens.append(50 + s)
        else:
            want_tokens.append(10 + s)
        s += L
    tokens, spans, unmappable, s_end = ov.map_merge(d, dmap, cache, 4)
    assert [sp[1] for sp in spans] == list(pattern)
    assert [sp[0] for sp in spans] == list(np.cumsum((0,) + pattern[:-1]))
    assert tokens == want_tokens and not unmappable and s_end == k


def test_ngram_beats_direct_map_and_longest_wins():
    dmap = np.arange(10)
    cache = {(1, 2): 20, (1, 2, 3): 30, (2, 3): 40}
    tokens, spans, _, _ = ov.map_merge([1, 2, 3, 4], dmap, cache, 4)
    assert tokens == [30, 4] and spans == [(0, 3), (3, 1)]
    # with the window capped at 2 the shorter key is used, then scanning resumes after it (no overlap)
    tokens, spans, _, _ = ov.map_merge([1, 2, 3, 4], dmap, cache, 2)
    assert tokens == [20, 3, 4] and spans == [(0, 2), (2, 1), (3, 1)]
    # a key cut by the end of the window never matches partially
    tokens, spans, _, _ = ov.map_merge([0, 1, 2], dmap, {(1, 2, 3): 30}, 4)
    assert tokens == [0, 1, 2]


def test_empty_cache_is_the_direct_map():
    rng = np.random.default_rng(2)
    dmap = rng.permutation(50)
    d = rng.integers(0, 50, size=9)
    tokens, spans, unmappable, s_end = ov.map_merge(d, dmap, {}, 8)
    assert tokens == dmap[d].tolist() and spans == [(i, 1) for i in range(9)] and not unmappable and s_end == 9


def test_unmappable_token_cuts_the_proposal():
    dmap = np.array([0, 1, -1, 3])
    tokens, spans, unmappable, s_end = ov.map_merge([1, 2, 3], dmap, {}, 4)
    assert tokens == [1] and unmappable and s_end == 1
    # ... unless an n-gram covers it
    tokens, spans, unmappable, s_end = ov.map_merge([1, 2, 3], dmap, {(2, 3): 9}, 4)
    assert tokens == [1, 9] and not unmappable and s_end == 3


def test_duplicate_cache_keys_last_wins():
    c = ov.build_cache([0, 2, 4, 7], [5, 6, 5, 6, 1, 2, 3], [11, 22, 33])
    assert c == {(5, 6): 22, (1, 2, 3): 33}


def _naive_scan(d, dmap, entries, max_len):
    """Independent matcher: linear search over the entry list at every position, keep the longest."""
    out, s = [], 0
    while s < len(d):
        best = None
        for key, t in entries:                       # later entries override earlier equal keys
            L = len(key)
            if L <= max_len and s + L <= len(d) and all(d[s + i] == key[i] for i in range(L)):
                if best is None or L >= best[1]:
                    best = (t, L)
        if best is None:
            if dmap[d[s]] < 0:
                return out, True
            best = (int(dmap[d[s]]), 1)
        out.append((best[0], s, best[1]))
        s += best[1]
    return out, False


@settings(max_examples=400, deadline=None)
@given(st.data())
def test_scan_agrees_with_naive_matcher(data):
    V = data.draw(st.integers(2, 5))
    k = data.draw(st.integers(0, 8))
    d = data.draw(st.lists(st.integers(0, V - 1), min_size=k, max_size=k))
    dmap = np.array(data.draw(st.lists(st.integers(-1, 6), min_size=V, max_size=V)))
    n_e = data.draw(st.integers(0, 6))
    entries = []
    for e in range(n_e):
        L = data.draw(st.integers(2, 4))
        entries.append((tuple(data.draw(st.lists(st.integers(0, V - 1), min_size=L, max_size=L))), 100 + e))
    max_len = data.draw(st.integers(2, 4))
    key_off = np.cumsum([0] + [len(kk) for kk, _ in entries])
    key_ids = [v for kk, _ in entries for v in kk]
    cache = ov.build_cache(key_off, key_ids, [t for _, t in entries])
    tokens, spans, unmappable, _ = ov.map_merge(d, dmap, cache, max_len)
    want, want_unm = _naive_scan(d, dmap, entries, max_len)
    assert [(t, s, L) for t, (s, L) in zip(tokens, spans)] == want and unmappable == want_unm


# --------------------------------------------------------------------------- Eq. 1 / Eq. 2 worked example
def _gold_example():
    rows = {}
    with open(os.path.join(GOLD, "eq2_worked_example.txt")) as f:
        for ln in f:
            if ln.strip() and not ln.startswith("#"):
                key, *vals = ln.split()
                rows[key] = vals
    return rows


def test_eq1_eq2_worked_example():
    g = _gold_example()
    dmap = np.array([int(x) for x in g["dmap"]])
    cv = g["cache"]
    cache = {tuple(int(x) for x in cv[:cv.index("->")]): int(cv[-1])}
    q_rows = [np.array([float(x) for x in g["q0"]]), np.array([float(x) for x in g["q1"]])]
    d = [int(x) for x in g["drafted"]]
    p = np.array([float(x) for x in g["p"]])
    tokens, spans, unm, _ = ov.map_merge(d, dmap, cache, 4)
    assert tokens == [int(g["mapped"][0])] and spans == [tuple(int(x) for x in g["span"])] and not unm
    pi = ov.qprime_pointwise(q_rows, d, spans[0])
    assert pi == pytest.approx(float(g["qprime"][0]), rel=1e-15)
    assert min(1.0, p[tokens[0]] / pi) == pytest.approx(float(g["ratio"][0]), rel=1e-15)
    tmap = ov.inverse_map(dmap, p.size)
    qfull = ov.qprime_full(q_rows[0], dmap, tmap, (tokens[0], pi, d[0]))
    np.testing.assert_allclose(qfull, [float(x) for x in g["qfull"]], rtol=0, atol=1e-15)
    r = ov.residual(p, qfull)
    np.testing.assert_allclose(r, [float(x) for x in g["resid"]], rtol=0, atol=1e-15)
    np.testing.assert_allclose(r / r.sum(), [float(x) for x in g["residnorm"]], rtol=1e-14, atol=0)


def test_eq2_without_ngram_is_the_scatter_through_the_direct_map():
    rng = np.random.default_rng(3)
    V_d, V_t = 12, 20
    dmap = np.full(V_d, -1)
    src = rng.choice(V_d, 8, replace=False)
    dmap[src] = rng.choice(V_t, 8, replace=False)
    q = rng.dirichlet(np.ones(V_d))
    qp = ov.qprime_full(q, dmap, ov.inverse_map(dmap, V_t))
    want = np.zeros(V_t)
    for dd in range(V_d):
        if dmap[dd] >= 0:
            want[dmap[dd]] = q[dd]
    assert np.array_equal(qp, want)
    assert qp.sum() == pytest.approx(q[dmap >= 0].sum(), rel=1e-15)


@settings(max_examples=200, deadline=None)
@given(st.integers(0, 10_000))
def test_eq2_invariants(seed):
    """Mass is conserved by the two overrides, the prefix term is never negative, only two ids change."""
    rng = np.random.default_rng(seed)
    V_d, V_t = 10, 16
    dmap = np.full(V_d, -1)
    n_dir = int(rng.integers(1, 9))
    src = rng.choice(V_d, n_dir, replace=False)
    dst = rng.choice(12, n_dir, replace=False)               # direct images live in 0..11
    dmap[src] = dst
    tmap = ov.inverse_map(dmap, V_t)
    L = int(rng.integers(2, 5))
    q_rows = [rng.dirichlet(np.ones(V_d) * 0.5) for _ in range(L)]
    d = rng.integers(0, V_d, size=L)
    t_ng = int(rng.integers(12, V_t))                        # n-gram target outside the direct image
    pi = ov.qprime_pointwise(q_rows, d, (0, L))
    plain = ov.qprime_full(q_rows[0], dmap, tmap)
    full = ov.qprime_full(q_rows[0], dmap, tmap, (t_ng, pi, int(d[0])))
    assert full.min() >= 0.0                                  # q(d_1) - prod >= 0
    changed = set(np.flatnonzero(full != plain).tolist())
    allowed = {t_ng} | ({int(dmap[d[0]])} if dmap[d[0]] >= 0 else set())
    assert changed <= allowed
    assert full[t_ng] == pi
    if dmap[d[0]] >= 0:
        assert full.sum() == pytest.approx(plain.sum(), rel=1e-13)          # the overrides cancel
        assert full[dmap[d[0]]] == pytest.approx(q_rows[0][d[0]] - pi, rel=1e-13)
    else:
        assert full.sum() == pytest.approx(plain.sum() + pi, rel=1e-13)
    # pi -> 0 recovers the plain scatter
    tiny = ov.qprime_full(q_rows[0], dmap, tmap, (t_ng, 0.0, int(d[0])))
    assert np.array_equal(tiny, plain)


def test_eq2_ngram_case_wins_over_prefix_case_on_the_same_id():
    dmap = np.array([3, 1, -1])
    q = np.array([0.6, 0.3, 0.1])
    full = ov.qprime_full(q, dmap, ov.inverse_map(dmap, 5), (3, 0.12, 0))   # n-gram target == dmap[d_1]
    assert full[3] == 0.12 and full[1] == 0.3
