"""ot_adaptive_drafting_static (no context, no allocation, scratch inside the library) against ot_adaptive_drafting.

Two calls in a row on the same GPU, the second with a smaller batch: the shared scratch keeps the first call's
contents, so the second call shows that nothing stale is read.  Both entry points run the same kernels, so every
output must be bit-identical.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _buffers(torch, B, M, with_bce):
    dev = "cuda"
    return {"p_accept": torch.full((max(M, 1),), -7.0, dtype=torch.float32, device=dev),
            "p_any_reject": torch.full((max(M, 1),), -7.0, dtype=torch.float32, device=dev),
            "n_keep": torch.full((max(B, 1),), -7, dtype=torch.int32, device=dev),
            "bce": torch.full((3,), -7.0, dtype=torch.float64, device=dev) if with_bce else None}


def _case(seed, B):
    rng = np.random.default_rng(seed)
    k = rng.integers(0, 64, size=B)
    k[:2] = [63, 0]
    row_off = np.concatenate([[0], np.cumsum(k + 1)]).astype(np.int32)
    M = int(row_off[-1])
    a = (rng.standard_normal(M) * 2.0 + 1.5).astype(np.float32)
    labels = np.clip(rng.uniform(-0.2, 1.2, M), 0, 1).astype(np.float32)
    n_valid = rng.integers(0, 70, size=B).astype(np.int32)
    return row_off, a, labels, n_valid


def test_static_entry_point_matches_the_context_one_twice_in_a_row():
    import torch
    from oracle import adaptive as oa
    from paper_2507_02659_amd import binding as ot

    dev = "cuda"
    W = torch.zeros((8, 16), dtype=torch.float32, device=dev)
    ctx = ot.ot_verify_init(d=8, V_t=16, V_d=16, max_batch=700, max_k=63, dtype=ot.OT_F32, max_ngram_len=2, W=W,
                            direct_map=np.arange(16, dtype=np.int32))
    try:
        for call, (seed, B, gamma) in enumerate([(11, 700, 0.4), (12, 37, 0.7)]):      # the second call is smaller
            row_off, a, labels, n_valid = _case(seed, B)
            M = int(row_off[-1])
            print(f"no-alloc call {call}: B={B} M={M} gamma={gamma}", flush=True)
            t = lambda x, dt: torch.from_numpy(np.ascontiguousarray(x, dtype=dt)).to(dev)
            d_off, d_a, d_l, d_n = t(row_off, np.int32), t(a, np.float32), t(labels, np.float32), t(n_valid, np.int32)
            want, got = _buffers(torch, B, M, True), _buffers(torch, B, M, True)
            common = dict(B=B, gamma=gamma, w_accept=1.0, w_reject=4.0, row_off=d_off, row_off_host=row_off, head_logits=d_a,
                          labels=d_l, n_valid=d_n)
            ot.ot_adaptive_drafting(ctx, **common, **want)
            torch.cuda.synchronize()
            ot.ot_adaptive_drafting_static(**common, **got, stream=torch.cuda.current_stream().cuda_stream)
            torch.cuda.synchronize()
            for name in want:
                assert np.array_equal(want[name].cpu().numpy(), got[name].cpu().numpy()), name
            # and both agree with the oracle's loss value (the stop rule has its own parity tests)
            ref = oa.weighted_bce(row_off=row_off, head_logits=a, labels=labels, n_valid=n_valid, w_accept=1.0, w_reject=4.0)
            np.testing.assert_allclose(got["bce"].cpu().numpy()[2], ref["mean"], rtol=1e-12)
    finally:
        ot.ot_verify_destroy(ctx)


def test_static_entry_point_rejects_what_does_not_fit():
    import torch
    from paper_2507_02659_amd import binding as ot

    B = ot.OT_STATIC_MAX_BATCH + 1
    row_off = np.arange(B + 1, dtype=np.int32)
    buf = _buffers(torch, B, B, False)
    d_off = torch.from_numpy(row_off).to("cuda")
    d_a = torch.zeros(B, dtype=torch.float32, device="cuda")
    with pytest.raises(ot.OtError) as err:
        ot.ot_adaptive_drafting_static(B=B, gamma=0.5, row_off=d_off, row_off_host=row_off, head_logits=d_a, **buf)
    assert err.value.code == ot.OT_ERR_SHAPE and "OT_STATIC_MAX_BATCH" in err.value.message
    torch.cuda.synchronize()
    assert np.all(buf["n_keep"].cpu().numpy() == -7)       # nothing was launched
