"""HIP path vs CPU oracle, through the C ABI, on seeded synthetic batches.  All tests need a real MI355X."""
import numpy as np
import pytest

from workloads import CaseSpec, baseline_case, baseline_spec, make_case

pytestmark = pytest.mark.gpu


def _imports():
    from oracle import verify as ov
    from paper_2507_02659_amd import binding as ot
    from paper_2507_02659_amd.runner import Verifier
    import parity
    return ov, ot, Verifier, parity


def _say(msg):
    print(msg, flush=True)


def _band_budget(B):
    """Sequences that may sit in a tolerance band.  The bands are 1e-5 (ratio) and 1e-6 of the mass per cell edge (CDF)
    wide, and a GPU decision differs from the oracle's only when rounding of about 1e-7 (fp32-accumulated logits) or
    1e-12 (given logits) carries it across: well under 1e-2 per sequence."""
    return max(1, int(np.ceil(1e-2 * B)))


def _run_and_compare(case, *, expect_exact_fraction=0.0, max_divergent=None):
    """One step through the library against the oracle.  A bf16 batch with hidden states runs twice: with the draft
    side hosted by the LM-head launch (where that kernel supports the shape) and with every stage as its own launch;
    the estimate that picks between the two in production would send every small test shape down the second path."""
    ov, ot, Verifier, parity = _imports()
    _say(f"case {case.name}: B={case.B} M={case.M} K={case.K} d={case.d} V_t={case.V_t} V_d={case.V_d} {case.dtype}")
    ref = ov.verify_case(case)
    both = case.hidden is not None and case.dtype == "bf16"
    gpu = rep = None
    for policy in ((ot.OT_DRAFT_SIDE_SEPARATE, ot.OT_DRAFT_SIDE_IN_LM_HEAD) if both else (ot.OT_DRAFT_SIDE_AUTO,)):
        v = Verifier.for_case(case, draft_side=policy)
        try:
            gpu = v.run_case(case)
        finally:
            v.close()
        rep = parity.compare(case, gpu, ref, logits_from_gpu=case.hidden is not None)
        _say(f"  draft_side={policy}: " + rep.summary())
        assert not rep.failures, "\n".join(rep.failures[:10])
        budget = _band_budget(case.B) if max_divergent is None else max_divergent
        assert rep.divergent <= budget, rep.summary()
        assert rep.exact >= expect_exact_fraction * rep.sequences
    return gpu, ref, rep


# --------------------------------------------------------------------------- LM head (MFMA) against float64
@pytest.mark.parametrize("M,d,V_t", [(1, 256, 1024), (5, 320, 1000), (16, 256, 4100), (17, 512, 2048), (48, 128, 777),
                                     (100, 384, 3000), (144, 256, 2304), (150, 256, 1500), (300, 136, 1111),
                                     (257, 192, 2000), (512, 256, 5000), (640, 64, 300)])
def test_lm_head_logits_bf16(M, d, V_t):
    ov, ot, Verifier, parity = _imports()
    k = M - 1 if M - 1 <= 63 else None
    if k is not None:
        ks = [k]
    else:                                   # several sequences so that no k exceeds the cap
        ks, left = [], M
        while left > 0:
            take = min(left, 50)
            ks.append(take - 1)
            left -= take
    spec = CaseSpec(name=f"gemm_{M}x{d}x{V_t}", dtype="bf16", d=d, V_t=V_t, V_d=64, k=ks, temperature=[1.0] * len(ks),
                    n_direct=32, data_seed=M * 7 + d, philox_seed=1)
    case = make_case(spec)
    assert case.M == M
    _say(f"gemm case M={M} d={d} V_t={V_t}")
    v = Verifier.for_case(case)
    try:
        inp = v.upload(case)
        v.step(inp)
        ws = v.workspace(case.M, case.K, with_logits=True)
    finally:
        v.close()
    Z = ov.lm_head_logits(case.hidden, case.W, "bf16")
    np.testing.assert_allclose(ws["logits"], Z, rtol=1e-5, atol=2e-5)


def test_lm_head_logits_f32_config1():
    ov, ot, Verifier, parity = _imports()
    case = baseline_case(1)
    v = Verifier.for_case(case)
    try:
        inp = v.upload(case)
        v.step(inp)
        ws = v.workspace(case.M, case.K, with_logits=True)
    finally:
        v.close()
    Z = ov.lm_head_logits(case.hidden, case.W, "f32")
    np.testing.assert_allclose(ws["logits"], Z, rtol=1e-5, atol=2e-6)


# --------------------------------------------------------------------------- softmax statistics
@pytest.mark.parametrize("dtype,V_t,V_d", [("f32", 1024, 512), ("bf16", 9000, 5003), ("bf16", 4097, 4096), ("f32", 12289, 777)])
def test_softmax_statistics(dtype, V_t, V_d):
    """Row max / argmax exact, sum of exponentials to 2e-6, for target rows (fp32) and draft rows (storage dtype)."""
    ov, ot, Verifier, parity = _imports()
    spec = CaseSpec(name=f"stats_{dtype}_{V_t}_{V_d}", dtype=dtype, d=32, V_t=V_t, V_d=V_d, k=[3, 0, 7, 1],
                    temperature=[1.0, 0.5, 0.0, 2.0], draft_temperature=[0.8, 1.0, 1.0, 0.0], n_direct=min(V_d, V_t) // 2,
                    data_seed=V_t + V_d, philox_seed=2, logits_only=True)
    case = make_case(spec)
    v = Verifier.for_case(case)
    try:
        inp = v.upload(case)
        v.step(inp, from_logits=True)
        ws = v.workspace(case.M, case.K)
    finally:
        v.close()
    Z = case.target_logits.astype(np.float64)
    Zq = ov.widen(case.draft_logits, dtype)
    assert np.array_equal(ws["row_max"].astype(np.float64), Z.max(axis=1))
    assert np.array_equal(ws["row_argmax"], Z.argmax(axis=1))
    assert np.array_equal(ws["draft_row_max"].astype(np.float64), Zq.max(axis=1))
    assert np.array_equal(ws["draft_row_argmax"], Zq.argmax(axis=1))
    for b in range(case.B):
        r0, r1 = case.row_off[b], case.row_off[b + 1]
        T = float(case.temperature[b]) or 1.0
        Td = float(case.draft_temperature[b]) or 1.0
        want = np.exp((Z[r0:r1] - Z[r0:r1].max(axis=1, keepdims=True)) / T).sum(axis=1)
        np.testing.assert_allclose(ws["row_sumexp"][r0:r1], want, rtol=2e-6)
        q0, q1 = r0 - b, r1 - b - 1
        wantq = np.exp((Zq[q0:q1] - Zq[q0:q1].max(axis=1, keepdims=True)) / Td).sum(axis=1)
        np.testing.assert_allclose(ws["draft_row_sumexp"][q0:q1], wantq, rtol=2e-6)


@pytest.mark.parametrize("ks,V_t,V_d", [([7, 3, 0, 9], 6000, 5003),      # 24 workgroups, 19 rows: 5 rows in two pieces
                                        ([5, 5, 6], 12800, 4096),         # 50 workgroups, 16 rows: three pieces a row
                                        ([5, 5, 6], 10240, 1111),         # 40 workgroups, 16 rows: 8 rows in three, 8 in two
                                        ([8, 8], 4100, 1000),             # 17 workgroups, 16 rows: one row in two
                                        ([30, 25, 1, 10], 1500, 24),      # 6 workgroups, 66 rows: whole rows in turn
                                        ([40, 20], 2304, 40000)])         # long rows: more than one batch per wavefront
def test_draft_row_statistics_from_lm_head_launch(ks, V_t, V_d):
    """The LM-head launch that hosts the draft side shares the draft rows out over its multiplying workgroups, in pieces
    of a row where there are more workgroups than rows; the launch that follows merges the pieces.  Row maximum and
    argmax exact, sum of exponentials to 2e-6, for every way the rows can be shared out (bf16 rows, aligned or not)."""
    ov, ot, Verifier, parity = _imports()
    temps = [[1.0, 0.5, 0.0, 2.0][i % 4] for i in range(len(ks))]
    dtemps = [[0.8, 1.0, 1.3, 0.0][i % 4] for i in range(len(ks))]
    spec = CaseSpec(name=f"pieces_{len(ks)}_{V_t}_{V_d}", dtype="bf16", d=64, V_t=V_t, V_d=V_d, k=ks, temperature=temps,
                    draft_temperature=dtemps, n_direct=min(V_d, V_t) // 2, data_seed=V_t + V_d, philox_seed=4)
    case = make_case(spec)
    assert case.M > 16                               # the wide kernel
    v = Verifier.for_case(case, draft_side=ot.OT_DRAFT_SIDE_IN_LM_HEAD)
    try:
        inp = v.upload(case)
        v.step(inp)
        ws = v.workspace(case.M, case.K)
    finally:
        v.close()
    Zq = ov.widen(case.draft_logits, "bf16")
    assert np.array_equal(ws["draft_row_max"].astype(np.float64), Zq.max(axis=1))
    assert np.array_equal(ws["draft_row_argmax"], Zq.argmax(axis=1))
    for b in range(case.B):
        q0, q1 = case.row_off[b] - b, case.row_off[b + 1] - b - 1
        Td = float(case.draft_temperature[b]) or 1.0
        wantq = np.exp((Zq[q0:q1] - Zq[q0:q1].max(axis=1, keepdims=True)) / Td).sum(axis=1)
        np.testing.assert_allclose(ws["draft_row_sumexp"][q0:q1], wantq, rtol=2e-6)


@pytest.mark.parametrize("M,d,V_t", [(20, 256, 1000), (60, 128, 2304), (96, 192, 777), (144, 256, 4100), (300, 136, 1111)])
def test_row_statistics_from_lm_head_epilogue(M, d, V_t):
    """From 17 rows on the LM-head kernel emits the softmax partials itself (no second pass over the logits).

    The oracle's logits are float64 and the kernel's fp32-accumulated, so the maximum is compared to 2e-5, the argmax
    must be a column whose oracle logit is within that band of the oracle's maximum, and the sum of exponentials
    (temperatures 1, 0.5, 2 and greedy rows) to 1e-4."""
    ov, ot, Verifier, parity = _imports()
    ks, left = [], M
    while left > 0:
        take = min(left, 40)
        ks.append(take - 1)
        left -= take
    temps = [[1.0, 0.5, 0.0, 2.0][i % 4] for i in range(len(ks))]
    spec = CaseSpec(name=f"fused_{M}x{d}x{V_t}", dtype="bf16", d=d, V_t=V_t, V_d=64, k=ks, temperature=temps,
                    n_direct=32, data_seed=M * 11 + V_t, philox_seed=1)
    case = make_case(spec)
    assert case.M == M
    _say(f"fused statistics case M={M} d={d} V_t={V_t}")
    v = Verifier.for_case(case, draft_side=ot.OT_DRAFT_SIDE_IN_LM_HEAD)
    try:
        inp = v.upload(case)
        v.step(inp)
        ws = v.workspace(case.M, case.K)
    finally:
        v.close()
    Z = ov.lm_head_logits(case.hidden, case.W, "bf16")
    zmax = Z.max(axis=1)
    np.testing.assert_allclose(ws["row_max"], zmax, rtol=0, atol=2e-5)
    arg = ws["row_argmax"].astype(np.int64)
    assert arg.min() >= 0 and arg.max() < V_t
    assert np.all(Z[np.arange(M), arg] >= zmax - 4e-5)
    for b in range(case.B):
        r0, r1 = case.row_off[b], case.row_off[b + 1]
        T = float(case.temperature[b]) or 1.0
        want = np.exp((Z[r0:r1] - Z[r0:r1].max(axis=1, keepdims=True)) / T).sum(axis=1)
        np.testing.assert_allclose(ws["row_sumexp"][r0:r1], want, rtol=1e-4)


# --------------------------------------------------------------------------- the five BASELINE configurations, full size
@pytest.mark.parametrize("i,greedy", [(1, False), (2, False), (2, True), (3, False), (4, False), (5, False)])
def test_baseline_configuration(i, greedy):
    case = make_case(baseline_spec(i, greedy=greedy))
    gpu, ref, rep = _run_and_compare(case)
    assert np.all(gpu["n_emit"] == gpu["n_accept"] + 1)
    if i in (3, 4, 5):
        assert gpu["hits_proposed"].sum() > 0          # planted cache keys were found by the hash probe


@pytest.mark.parametrize("i", [3, 4, 5])
def test_baseline_configuration_logits_and_row_statistics_elementwise(i):
    """Full-size LM head (d = 3584 / 4096, V_t = 128256 / 152064, every M-block height the configurations use): every
    logit against the float64 product, and the row statistics the launch leaves behind against those of the float64
    logits.  The kernel adds d/32 MFMA partial products in fp32: a running sum of magnitude up to ~2 is rounded to
    2^-24 relative at each of the d/32 additions, a random walk of about sqrt(d/32) * 1.2e-7 = 1.3e-6 at d = 4096
    (standard deviation); over the 18 to 65 million logits of these cases the largest deviation reaches five to six
    of those, so the absolute bound is 1.5e-7 * sqrt(d) (seven standard deviations), next to 1e-5 relative."""
    ov, ot, Verifier, parity = _imports()
    case = make_case(baseline_spec(i))
    _say(f"full-size logits, configuration {i}: M={case.M} d={case.d} V_t={case.V_t}")
    v = Verifier.for_case(case, draft_side=ot.OT_DRAFT_SIDE_IN_LM_HEAD)
    try:
        inp = v.upload(case)
        v.step(inp)
        ws = v.workspace(case.M, case.K, with_logits=True)
    finally:
        v.close()
    Z = ov.lm_head_logits(case.hidden, case.W, "bf16")
    atol = 1.5e-7 * np.sqrt(case.d)
    np.testing.assert_allclose(ws["logits"], Z, rtol=1e-5, atol=atol)
    zmax = Z.max(axis=1)
    np.testing.assert_allclose(ws["row_max"], zmax, rtol=0, atol=2 * atol)
    arg = ws["row_argmax"].astype(np.int64)
    assert arg.min() >= 0 and arg.max() < case.V_t
    assert np.all(Z[np.arange(case.M), arg] >= zmax - 4 * atol)
    for b in range(case.B):
        r0, r1 = case.row_off[b], case.row_off[b + 1]
        T = float(case.temperature[b]) or 1.0
        want = np.exp((Z[r0:r1] - Z[r0:r1].max(axis=1, keepdims=True)) / T).sum(axis=1)
        np.testing.assert_allclose(ws["row_sumexp"][r0:r1], want, rtol=1e-4)
    # the draft rows' statistics (computed next to the LM head) against the widened draft logits
    Zq = ov.widen(case.draft_logits, "bf16")
    assert np.array_equal(ws["draft_row_max"].astype(np.float64), Zq.max(axis=1))
    assert np.array_equal(ws["draft_row_argmax"], Zq.argmax(axis=1))
    for b in range(case.B):
        q0, q1 = case.row_off[b] - b, case.row_off[b + 1] - b - 1
        Td = float(case.temperature[b] if case.draft_temperature is None else case.draft_temperature[b]) or 1.0
        wantq = np.exp((Zq[q0:q1] - Zq[q0:q1].max(axis=1, keepdims=True)) / Td).sum(axis=1)
        np.testing.assert_allclose(ws["draft_row_sumexp"][q0:q1], wantq, rtol=2e-6)


# --------------------------------------------------------------------------- acceptance chains, bonus tokens, deep rejections
@pytest.mark.parametrize("dtype,logits_only,seed", [("bf16", False, 1), ("bf16", True, 2), ("f32", False, 3), ("f32", True, 4)])
def test_agreeable_batches(dtype, logits_only, seed):
    spec = CaseSpec(name=f"agree_{dtype}_{int(logits_only)}", dtype=dtype, d=256, V_t=9000, V_d=3000,
                    k=[6, 3, 8, 1, 0, 5, 7, 2] * 8, temperature=[1.0, 0.7, 0.0, 1.3] * 16, n_direct=2200, n_ngram=900,
                    ngram_len=(2, 5), zipf_a=1.1, plant_cover=0.35, align=0.8, data_seed=50 + seed, philox_seed=seed,
                    logits_only=logits_only)
    case = make_case(spec)
    gpu, ref, rep = _run_and_compare(case)
    assert ref["n_accept"].max() >= 3 and ref["hits_accepted"].sum() > 0
    assert (ref["n_accept"] == ref["n_mapped"]).sum() > 0            # free-token branch exercised
    assert (ref["flags"] & 1).sum() > 0                              # unmappable branch exercised


def test_many_steps_monte_carlo_agreement():
    """Same batch, 300 Philox steps: every step must reproduce the oracle's draws."""
    ov, ot, Verifier, parity = _imports()
    spec = CaseSpec(name="steps", dtype="bf16", d=64, V_t=3000, V_d=1200, k=[4, 6, 2, 5, 3, 6, 1, 4], temperature=[1.0] * 8,
                    n_direct=900, n_ngram=300, ngram_len=(2, 4), plant_cover=0.3, align=0.7, data_seed=77, philox_seed=5,
                    logits_only=True)
    case = make_case(spec)
    cache = ov.build_cache(case.ngram_key_off, case.ngram_key_ids, case.ngram_target_ids)
    total = parity.Report()
    v = Verifier.for_case(case)
    try:
        inp = v.upload(case)
        for step in range(300):
            v.step(inp, from_logits=True, step=step)
            gpu = v.results(inp)
            case.step = step
            ref = ov.verify_case(case)
            total.merge(parity.compare(case, gpu, ref, logits_from_gpu=False))
    finally:
        v.close()
    _say("  " + total.summary())
    assert not total.failures, "\n".join(total.failures[:10])
    assert total.divergent <= _band_budget(total.sequences)   # 2400 sequence-steps


# --------------------------------------------------------------------------- edge cases
def test_ragged_maximum_k_and_empty_sequences():
    spec = CaseSpec(name="edge_k", dtype="bf16", d=128, V_t=5000, V_d=2000, k=[63, 0, 1, 63, 0], temperature=[1.0, 1.0, 0.0, 0.9, 0.0],
                    n_direct=1500, n_ngram=500, ngram_len=(2, 8), plant_cover=0.4, align=0.9, data_seed=88, philox_seed=6)
    _run_and_compare(make_case(spec))


def test_more_sequences_than_the_lm_head_stages():
    """Above 255 sequences the LM-head epilogue emits no statistics and the separate pass over the logits runs."""
    spec = CaseSpec(name="edge_many_seqs", dtype="bf16", d=64, V_t=1300, V_d=600, k=[1, 0, 2] * 90, temperature=[1.0, 0.0, 0.7] * 90,
                    n_direct=400, n_ngram=100, ngram_len=(2, 3), plant_cover=0.3, align=0.8, data_seed=90, philox_seed=8)
    _run_and_compare(make_case(spec))


@pytest.mark.parametrize("M,B", [(16, 2), (17, 2), (33, 3), (96, 6), (97, 6), (144, 9), (145, 9), (160, 10), (176, 11), (177, 11), (288, 12), (289, 12),
                                 (300, 255), (300, 256), (320, 20), (352, 16), (433, 20)])
def test_row_count_boundaries_end_to_end(M, B):
    """Whole steps from hidden states at the row counts where the LM head changes kernel, M-block size or the number of
    M-blocks, and at the sequence count where its epilogue stops emitting the row statistics."""
    ks = [M // B - 1] * B
    for i in range(M - sum(k + 1 for k in ks)):
        ks[i] += 1
    temps = [[1.0, 0.6, 0.0, 1.4][i % 4] for i in range(B)]
    spec = CaseSpec(name=f"rows_{M}_{B}", dtype="bf16", d=64, V_t=1111, V_d=500, k=ks, temperature=temps, n_direct=400,
                    n_ngram=150, ngram_len=(2, 4), plant_cover=0.4, align=0.8, data_seed=1000 + M + B, philox_seed=9)
    case = make_case(spec)
    assert case.M == M and case.B == B
    _run_and_compare(case)


@pytest.mark.parametrize("seed", range(24))
def test_random_shapes_end_to_end(seed):
    """Seeded random batch shapes, vocabulary sizes, temperatures, cache settings and dtypes through the whole step."""
    rng = np.random.default_rng(7000 + seed)
    B = int(rng.integers(1, 41))
    kmax = int(rng.choice([3, 8, 20, 63]))
    k = rng.integers(0, kmax + 1, size=B).tolist()
    if seed % 6 == 0:
        k[0] = 63
    V_d = int(rng.integers(100, 3000))
    V_t = int(rng.integers(max(200, V_d // 2), 6000))
    n_direct = int(rng.integers(V_d // 3, min(V_d, V_t - 60) + 1))
    lmax = int(rng.integers(2, 9))
    n_ngram = int(rng.choice([0, 40, min(500, V_t - n_direct - 10)]))
    temps = rng.choice([0.0, 0.5, 1.0, 2.0], size=B, p=[0.15, 0.25, 0.45, 0.15]).tolist()
    draft_t = None if seed % 3 else rng.choice([0.0, 0.7, 1.0], size=B, p=[0.2, 0.4, 0.4]).tolist()
    spec = CaseSpec(name=f"rand_{seed}", dtype=str(rng.choice(["bf16", "f32"])), d=int(rng.integers(4, 21)) * 8, V_t=V_t, V_d=V_d, k=k,
                    temperature=temps, draft_temperature=draft_t, n_direct=n_direct, n_ngram=n_ngram, ngram_len=(2, lmax),
                    plant_cover=float(rng.choice([0.0, 0.3, 0.7])), align=float(rng.choice([0.0, 0.6, 0.9])), data_seed=9000 + seed,
                    philox_seed=seed, logits_only=bool(rng.integers(0, 2)))
    _run_and_compare(make_case(spec))


def test_draft_temperature_variants():
    spec = CaseSpec(name="edge_td", dtype="f32", d=64, V_t=2500, V_d=1000, k=[5] * 12, temperature=[1.0] * 6 + [0.0] * 6,
                    draft_temperature=[0.0, 0.5, 2.0] * 4, n_direct=800, n_ngram=200, ngram_len=(2, 3), plant_cover=0.3,
                    align=0.7, data_seed=89, philox_seed=7, logits_only=True)
    _run_and_compare(make_case(spec))


def test_bad_draft_ids_are_flagged_not_faulted():
    ov, ot, Verifier, parity = _imports()
    spec = CaseSpec(name="edge_bad", dtype="f32", d=32, V_t=600, V_d=300, k=[4, 4, 4, 4], temperature=[1.0] * 4, n_direct=250,
                    data_seed=90, philox_seed=8, logits_only=True)
    case = make_case(spec)
    case.draft_ids[1] = -1
    case.draft_ids[4 + 2] = 300
    case.draft_ids[8 + 3] = 2 ** 31 - 1
    gpu, ref, rep = _run_and_compare(case)
    assert gpu["flags"].tolist()[:3] == [ot.OT_FLAG_BAD_ID] * 3 and gpu["n_emit"].tolist()[:3] == [0, 0, 0]
    assert gpu["n_emit"][3] >= 1


def test_no_cache_and_empty_cache_agree():
    ov, ot, Verifier, parity = _imports()
    spec = CaseSpec(name="edge_nocache", dtype="bf16", d=64, V_t=2000, V_d=2000, k=[5] * 6, temperature=[1.0] * 6,
                    identity_map=True, permute_frac=0.1, align=0.6, data_seed=91, philox_seed=9)
    case = make_case(spec)
    v = Verifier.for_case(case, draft_side=ot.OT_DRAFT_SIDE_IN_LM_HEAD)
    try:
        a = v.run_case(case)                      # empty cache object
        b = v.run_case(case, use_cache=False)     # NULL cache
    finally:
        v.close()
    for name in a:
        assert np.array_equal(a[name], b[name]), name
    ref = ov.verify_case(case)
    rep = parity.compare(case, a, ref, logits_from_gpu=True)
    assert not rep.failures and rep.divergent <= 1


def test_zero_residual_fallback_flag():
    """p and q' collapse to the same one-hot while the drafted id has no image: residual mass 0, draw from p."""
    ov, ot, Verifier, parity = _imports()
    spec = CaseSpec(name="edge_zero_resid", dtype="f32", d=8, V_t=5, V_d=4, k=[1], temperature=[1.0], n_direct=0,
                    data_seed=92, philox_seed=10, logits_only=True)
    case = make_case(spec)
    case.direct_map[:] = [0, -1, 1, 3]
    case.target_logits[:] = 0
    case.target_logits[0, 1] = 2000.0
    case.draft_logits[:] = 0
    case.draft_logits[0, 2] = 2000.0
    case.draft_ids[:] = [1]
    gpu, ref, rep = _run_and_compare(case)
    assert gpu["flags"][0] == (ot.OT_FLAG_UNMAPPABLE | ot.OT_FLAG_RESID_ZERO) and gpu["out_tokens"][0] == 1


def test_eq2_override_on_shared_target_id():
    """An n-gram whose target id also has a direct pre-image: the n-gram case of Eq. 2 wins."""
    ov, ot, Verifier, parity = _imports()
    spec = CaseSpec(name="edge_shared", dtype="f32", d=8, V_t=40, V_d=30, k=[3] * 32, temperature=[1.0] * 32, n_direct=25,
                    data_seed=93, philox_seed=11, logits_only=True, max_ngram_len=3)
    case = make_case(spec)
    mapped = np.flatnonzero(case.direct_map >= 0)
    d1, d2 = int(mapped[0]), int(mapped[1])
    case.ngram_key_off = np.array([0, 2], np.int32)
    case.ngram_key_ids = np.array([d1, d2], np.int32)
    case.ngram_target_ids = np.array([case.direct_map[mapped[2]]], np.int32)     # shared with a direct image
    for b in range(case.B):
        case.draft_ids[3 * b: 3 * b + 2] = [d1, d2]
    # make the n-gram likely to be rejected: its target logit is very low
    case.target_logits[:, case.ngram_target_ids[0]] = -8.0
    gpu, ref, rep = _run_and_compare(case)
    assert ref["hits_proposed"].sum() == case.B and (ref["n_accept"] == 0).sum() > case.B // 2


def test_determinism_bitwise():
    ov, ot, Verifier, parity = _imports()
    case = make_case(baseline_spec(4, scale={"d": 512, "V_t": 20000, "V_d": 8000, "n_direct": 6000, "n_ngram": 3000}))
    v = Verifier.for_case(case, draft_side=ot.OT_DRAFT_SIDE_IN_LM_HEAD)
    try:
        first = v.run_case(case)
        for _ in range(3):
            again = v.run_case(case)
            for name in first:
                assert np.array_equal(first[name], again[name]), name
    finally:
        v.close()
