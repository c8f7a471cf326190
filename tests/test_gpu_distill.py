"""Forward values of the hybrid distillation loss: ot_distill_loss against oracle/distill.py, through the C ABI."""
import numpy as np
import pytest

from workloads import CaseSpec, baseline_case, make_case

pytestmark = pytest.mark.gpu

MODES = [("fixed", "nll", False), ("target_prob", "nll", False), ("fixed", "approx_kl", False), ("target_prob", "approx_kl", True),
         ("fixed", "nll", True)]


def _imports():
    from oracle import distill as od
    from oracle import verify as ov
    from paper_2507_02659_amd import binding as ot
    from paper_2507_02659_amd.runner import Verifier
    return od, ov, ot, Verifier


def _say(msg):
    print(msg, flush=True)


def _compare(case, *, rtol, atol, with_qprime=False, modes=MODES):
    """Runs a verification step and then every loss mode on the GPU, and the same through the oracle."""
    od, ov, ot, Verifier = _imports()
    from_logits = case.hidden is None
    _say(f"loss case {case.name}: B={case.B} M={case.M} V_t={case.V_t} V_d={case.V_d} {case.dtype} from_logits={from_logits}")
    ref = ov.verify_case(case)
    v = Verifier.for_case(case, draft_side=ot.OT_DRAFT_SIDE_IN_LM_HEAD)     # the row statistics the loss reads come from the LM-head launch where it supports the shape
    try:
        inp = v.upload(case)
        v.step(inp, from_logits=from_logits)
        gpu_step = v.results(inp)
        # the translation is integer work and must agree exactly; acceptance is compared where it is used below
        for name in ("n_mapped", "mapped_ids", "span_start", "span_len"):
            assert np.array_equal(gpu_step[name], ref[name]), name
        for lambda_mode, ngram_term, accepted_only in modes:
            if accepted_only and not np.array_equal(gpu_step["n_accept"], ref["n_accept"]):
                _say("  acceptance differs inside its rounding band: accepted-only mode not compared")
                continue
            want = od.hybrid_loss_case(case, lam=0.2, lambda_mode=lambda_mode, ngram_term=ngram_term,
                                       n_accept=ref["n_accept"] if accepted_only else None)
            got = v.distill_loss(inp, from_logits=from_logits, lam=0.2,
                                 lambda_mode=ot.OT_LAMBDA_TARGET_PROB if lambda_mode == "target_prob" else ot.OT_LAMBDA_FIXED,
                                 ngram_term=ot.OT_NGRAM_TERM_APPROX_KL if ngram_term == "approx_kl" else ot.OT_NGRAM_TERM_NLL,
                                 accepted_only=accepted_only, with_qprime=with_qprime)
            tag = f"{lambda_mode}/{ngram_term}/accepted_only={accepted_only}"
            assert np.array_equal(got["kind"], want["kind"]), tag
            np.testing.assert_allclose(got["nll"], want["nll"], rtol=rtol, atol=atol, err_msg=tag)
            np.testing.assert_allclose(got["kl"], want["kl"], rtol=rtol, atol=atol, err_msg=tag)
            # lambda = p(t_i) leaves the library as the step's float32 p_tok
            np.testing.assert_allclose(got["weight"], want["weight"], rtol=max(rtol, 2e-7), atol=0, err_msg=tag)
            assert (got["n_dm"], got["n_ngram_tokens"]) == (want["n_dm"], want["n_ngram_tokens"]), tag
            for name in ("loss_dm", "loss_ngram", "loss"):
                assert got[name] == pytest.approx(want[name], rel=10 * rtol, abs=10 * atol), (tag, name)
            _say(f"  {tag}: loss {got['loss']:.9g} (oracle {want['loss']:.9g}), {want['n_dm']} direct tokens, {want['n_ngram_tokens']} n-gram sub-tokens")
            if with_qprime:
                _check_qprime(case, ref, want, got["qprime"], ov)
    finally:
        v.close()


def _check_qprime(case, ref, want, qprime, ov):
    """Every exported row against Eq. 2 written out by the oracle (rows without a term are zero)."""
    tmap = ov.inverse_map(case.direct_map, case.V_t)
    Zq = ov.widen(case.draft_logits, case.dtype)
    for b in range(case.B):
        r0, q0 = case.row_off[b], case.row_off[b] - b
        Td = float(case.temperature[b] if case.draft_temperature is None else case.draft_temperature[b])
        for j in range(case.row_off[b + 1] - r0):
            row = r0 + j
            if want["kind"][row] == 0:
                assert not qprime[row].any()
                continue
            s, L = ref["span_start"][row], ref["span_len"][row]
            q_s = ov.distribution(Zq[q0 + s], Td)
            ngram = None
            if L > 1:
                ngram = (int(ref["mapped_ids"][row]), float(ref["q_tok"][row]), int(case.draft_ids[q0 + s]))
            np.testing.assert_allclose(qprime[row], ov.qprime_full(q_s, case.direct_map, tmap, ngram), rtol=3e-6, atol=1e-30)


@pytest.mark.parametrize("dtype,seed", [("f32", 31), ("bf16", 32), ("f32", 33)])
def test_loss_from_logits_all_modes(dtype, seed):
    spec = CaseSpec(name=f"loss_{dtype}_{seed}", dtype=dtype, d=32, V_t=5000, V_d=2100, k=[6, 0, 9, 3, 1, 7, 5, 4],
                    temperature=[1.0, 1.0, 0.7, 0.0, 1.5, 1.0, 0.9, 1.0],
                    draft_temperature=None if seed != 33 else [0.8, 1.0, 1.0, 1.0, 0.0, 1.2, 1.0, 0.6],
                    n_direct=1700, n_ngram=400, ngram_len=(2, 5), plant_cover=0.5, align=0.8, data_seed=seed, philox_seed=3,
                    logits_only=True)
    # every q'(v) carries the 1e-7 relative error of the kernels' fast exponential and the KL terms have both signs,
    # so the error of a KL value scales with sum |q' (ln q' - ln p)| (a few units), not with the value itself
    _compare(make_case(spec), rtol=2e-6, atol=1e-6, with_qprime=True)


def test_loss_after_the_lm_head_several_tiles_and_ragged_tail():
    """Hidden states through the MFMA LM head (fp32 accumulation against the oracle's float64 logits)."""
    spec = CaseSpec(name="loss_gemm", dtype="bf16", d=128, V_t=9001, V_d=3000, k=[8, 5, 0, 10, 7, 3, 9, 6, 2, 8], temperature=[1.0] * 5 + [0.7] * 5,
                    n_direct=2500, n_ngram=600, ngram_len=(2, 6), plant_cover=0.5, align=0.8, data_seed=41, philox_seed=4)
    _compare(make_case(spec), rtol=1e-4, atol=1e-5)


def test_loss_baseline_configuration_4_full_size():
    case = baseline_case(4)
    _compare(case, rtol=1e-4, atol=1e-5, modes=[("fixed", "nll", False), ("target_prob", "approx_kl", False)])


def test_loss_argument_errors():
    od, ov, ot, Verifier = _imports()
    import ctypes as C
    spec = CaseSpec(name="loss_err", dtype="f32", d=16, V_t=300, V_d=120, k=[2, 1], temperature=[1.0, 1.0], n_direct=90,
                    data_seed=5, philox_seed=1, logits_only=True)
    case = make_case(spec)
    v = Verifier.for_case(case)
    try:
        inp = v.upload(case)
        v.step(inp, from_logits=True)
        with pytest.raises(ot.OtError) as e:
            v.distill_loss(inp, from_logits=True, lambda_mode=7)
        assert e.value.code == ot.OT_ERR_SHAPE and "lambda_mode" in e.value.message
        with pytest.raises(ot.OtError) as e:
            v.distill_loss(inp, from_logits=True, ngram_term=-1)
        assert e.value.code == ot.OT_ERR_SHAPE
        lib = ot.load_library()
        assert lib.ot_distill_loss(v.ctx, None, None, None, None, None) == ot.OT_ERR_NULL
        cfg = ot.ot_loss_config(0.2, 0, 0, 0)
        sin = ot.make_step_in(B=inp["B"], step=0, row_off=inp["row_off"], row_off_host=inp["row_off_host"], hidden=None,
                              draft_logits=inp["draft_logits"], draft_ids=inp["draft_ids"], temperature=inp["temperature"],
                              draft_temperature=None, seq_id=inp["seq_id"], seed=0)
        sout = ot.make_step_out(inp["out"])
        empty = ot.ot_loss_out()
        assert lib.ot_distill_loss(v.ctx, C.byref(sin), C.byref(sout), None, C.byref(cfg), C.byref(empty)) == ot.OT_ERR_NULL
        assert "required" in ot.ot_last_error()
        v.synchronize()
    finally:
        v.close()
