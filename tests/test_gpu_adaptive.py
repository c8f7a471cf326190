"""Adaptive-drafting stop rule and the acceptance head's loss value: ot_adaptive_drafting against oracle/adaptive.py."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _imports():
    import torch
    from oracle import adaptive as oa
    from paper_2507_02659_amd import binding as ot
    return torch, oa, ot


def _context(ot, torch, max_batch, max_k):
    """The entry point only needs a context for its stream and limits: a tiny fp32 head."""
    W = torch.zeros((8, 16), dtype=torch.float32, device="cuda")
    return ot.ot_verify_init(d=8, V_t=16, V_d=16, max_batch=max_batch, max_k=max_k, dtype=ot.OT_F32, max_ngram_len=2, W=W,
                             direct_map=np.arange(16, dtype=np.int32))


def _run(ot, torch, ctx, row_off, a, labels, n_valid, gamma, w_accept, w_reject):
    dev = "cuda"
    B, M = row_off.size - 1, int(row_off[-1])
    t = lambda x, dt: None if x is None else torch.from_numpy(np.ascontiguousarray(x, dtype=dt)).to(dev)
    buf = {"p_accept": torch.full((max(M, 1),), -7.0, dtype=torch.float32, device=dev),
           "p_any_reject": torch.full((max(M, 1),), -7.0, dtype=torch.float32, device=dev),
           "n_keep": torch.full((max(B, 1),), -7, dtype=torch.int32, device=dev),
           "bce": None if labels is None else torch.full((3,), -7.0, dtype=torch.float64, device=dev)}
    host_off = np.ascontiguousarray(row_off, dtype=np.int32)
    keep_alive = [t(row_off, np.int32), t(a, np.float32), t(labels, np.float32), t(n_valid, np.int32)]
    ot.ot_adaptive_drafting(ctx, B=B, gamma=gamma, w_accept=w_accept, w_reject=w_reject, row_off=keep_alive[0], row_off_host=host_off,
                            head_logits=keep_alive[1], labels=keep_alive[2], n_valid=keep_alive[3], **buf)
    torch.cuda.synchronize()
    return {k: (None if v is None else v.cpu().numpy()) for k, v in buf.items()}


@pytest.mark.parametrize("seed,gamma,with_valid", [(1, 0.3, False), (2, 0.7, True), (3, 0.95, False), (4, 0.0, True)])
def test_stop_rule_and_bce_against_oracle(seed, gamma, with_valid):
    torch, oa, ot = _imports()
    rng = np.random.default_rng(seed)
    k = rng.integers(0, 64, size=300)                     # ragged, empty sequences and the maximum 63 included
    k[:3] = [0, 63, 1]
    row_off = np.concatenate([[0], np.cumsum(k + 1)]).astype(np.int32)
    M = int(row_off[-1])
    a = (rng.standard_normal(M) * 2.0 + 2.0).astype(np.float32)
    a[rng.integers(0, M, 20)] = rng.choice([-60.0, 60.0, 0.0], 20)           # saturated and neutral logits
    labels = np.clip(rng.uniform(-0.2, 1.2, M), 0, 1).astype(np.float32)
    n_valid = rng.integers(0, 70, size=k.size).astype(np.int32) if with_valid else None
    print(f"adaptive case seed={seed} B={k.size} M={M} gamma={gamma}", flush=True)
    ctx = _context(ot, torch, max_batch=300, max_k=63)
    try:
        got = _run(ot, torch, ctx, row_off, a, labels, n_valid, gamma, 1.0, 6.0)
    finally:
        ot.ot_verify_destroy(ctx)
    want = oa.stop_rule(row_off=row_off, head_logits=a, gamma=gamma, n_valid=n_valid)
    np.testing.assert_allclose(got["p_accept"], want["p_accept"], rtol=1e-6, atol=1e-38)
    np.testing.assert_allclose(got["p_any_reject"], want["p_any_reject"], rtol=1e-6, atol=1e-7)
    # the threshold test is taken in binary64 on both sides; only a product within rounding of gamma may flip it
    differ = np.flatnonzero(got["n_keep"] != want["n_keep"])
    assert all(want["stop_margin"][b] < 1e-12 for b in differ), differ
    assert differ.size <= 1
    bce = oa.weighted_bce(row_off=row_off, head_logits=a, labels=labels, w_accept=1.0, w_reject=6.0, n_valid=n_valid)
    assert got["bce"][1] == bce["count"]
    assert got["bce"][0] == pytest.approx(bce["sum"], rel=1e-12)
    assert got["bce"][2] == pytest.approx(bce["mean"], rel=1e-12)


def test_labels_from_a_verification_step_feed_the_loss():
    """The acceptance ratios a verification step outputs are the labels: same-vocabulary batch, ratios -> BCE."""
    torch, oa, ot = _imports()
    from oracle import verify as ov
    from paper_2507_02659_amd.runner import Verifier
    from workloads import CaseSpec, make_case
    spec = CaseSpec(name="adapt_labels", dtype="f32", d=16, V_t=600, V_d=600, k=[5, 7, 3, 6], temperature=[1.0] * 4, n_direct=600,
                    align=0.8, data_seed=21, philox_seed=2, logits_only=True)
    case = make_case(spec)
    ref = ov.verify_case(case)
    rng = np.random.default_rng(5)
    a = rng.standard_normal(case.M).astype(np.float32)
    v = Verifier.for_case(case)
    try:
        inp = v.upload(case)
        v.step(inp, from_logits=True)
        v.synchronize()
        dev = inp["out"]["ratio"].device
        buf = {"p_accept": torch.zeros(case.M, dtype=torch.float32, device=dev), "p_any_reject": torch.zeros(case.M, dtype=torch.float32, device=dev),
               "n_keep": torch.zeros(case.B, dtype=torch.int32, device=dev), "bce": torch.zeros(3, dtype=torch.float64, device=dev)}
        a_dev = torch.from_numpy(a).to(dev)
        ot.ot_adaptive_drafting(v.ctx, B=case.B, gamma=0.7, w_accept=1.0, w_reject=6.0, row_off=inp["row_off"], row_off_host=inp["row_off_host"],
                                head_logits=a_dev, labels=inp["out"]["ratio"], n_valid=inp["out"]["n_mapped"], **buf)
        v.synchronize()
        got = buf["bce"].cpu().numpy()
    finally:
        v.close()
    want = oa.weighted_bce(row_off=case.row_off, head_logits=a, labels=ref["ratio"], w_accept=1.0, w_reject=6.0, n_valid=ref["n_mapped"])
    assert got[1] == want["count"] > 0
    assert got[0] == pytest.approx(want["sum"], rel=1e-5)          # the step's ratios are float32 outputs


def test_adaptive_argument_errors():
    torch, oa, ot = _imports()
    ctx = _context(ot, torch, max_batch=2, max_k=4)
    try:
        row_off = np.array([0, 3, 5], np.int32)
        with pytest.raises(ot.OtError) as e:
            _run(ot, torch, ctx, row_off, np.zeros(5, np.float32), None, None, 1.5, 1.0, 1.0)
        assert e.value.code == ot.OT_ERR_SHAPE and "gamma" in e.value.message
        with pytest.raises(ot.OtError) as e:
            _run(ot, torch, ctx, np.array([0, 8], np.int32), np.zeros(8, np.float32), None, None, 0.5, 1.0, 1.0)
        assert e.value.code == ot.OT_ERR_SHAPE                      # 7 drafted tokens > max_k
        with pytest.raises(ot.OtError) as e:
            _run(ot, torch, ctx, np.array([0, 2, 4, 6], np.int32), np.zeros(6, np.float32), None, None, 0.5, 1.0, 1.0)
        assert e.value.code == ot.OT_ERR_SHAPE                      # 3 sequences > max_batch
        lib = ot.load_library()
        assert lib.ot_adaptive_drafting(ctx, None, None) == ot.OT_ERR_NULL
        got = _run(ot, torch, ctx, row_off, np.zeros(5, np.float32), None, None, 0.6, 1.0, 1.0)   # no labels: no loss asked
        assert got["n_keep"].tolist() == [2, 1] and got["bce"] is None
    finally:
        ot.ot_verify_destroy(ctx)
