"""The C ABI: exported symbols match the header, and every error code can be forced from the host."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "otverify.h")


def _declared():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ot_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    from paper_2507_02659_amd import binding as ot
    lib = ot.load_library()
    names = _declared()
    assert set(names) == set(ot.EXPORTS), (names, ot.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None
    assert "gfx950" in ot.ot_version()


def test_struct_layouts_match_the_header():
    """Field order of the ctypes mirrors follows the header's struct definitions."""
    from paper_2507_02659_amd import binding as ot
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)

    def fields(struct):
        body = re.search(r"typedef struct %s \{(.*?)\} %s;" % (struct, struct), text, flags=re.S).group(1)
        out = []
        for decl in body.split(";"):
            decl = decl.strip()
            if not decl:
                continue
            names = re.sub(r"^(const\s+)?\w+\s*\**", "", decl)
            out += [n.strip().lstrip("*") for n in names.split(",")]
        return out

    for cls in (ot.ot_verify_config, ot.ot_step_in, ot.ot_step_out, ot.ot_workspace_view, ot.ot_loss_config, ot.ot_loss_out,
                ot.ot_adapt_in, ot.ot_adapt_out):
        assert [f[0] for f in cls._fields_] == fields(cls.__name__), cls.__name__
    assert C.sizeof(ot.ot_verify_config) == 8 * 4 + 3 * 8
    assert C.sizeof(ot.ot_step_in) == 8 + 8 * 8 + 8
    assert C.sizeof(ot.ot_step_out) == 14 * 8
    assert C.sizeof(ot.ot_loss_config) == 16 and C.sizeof(ot.ot_loss_out) == 6 * 8
    assert C.sizeof(ot.ot_adapt_in) == 24 + 5 * 8 and C.sizeof(ot.ot_adapt_out) == 4 * 8


def test_init_argument_errors_need_no_gpu():
    """Validation precedes every HIP call, so these run on a machine without a GPU."""
    from paper_2507_02659_amd import binding as ot
    good = dict(d=64, V_t=100, V_d=50, max_batch=2, max_k=4, dtype=ot.OT_BF16, max_ngram_len=3,
                W=0x1000, direct_map=np.full(50, -1, np.int32))

    def code(**kw):
        with pytest.raises(ot.OtError) as e:
            ot.ot_verify_init(**dict(good, **kw))
        assert e.value.message and ot.ot_last_error() == e.value.message
        return e.value.code

    assert code(W=None) == ot.OT_ERR_NULL
    assert code(direct_map=None) == ot.OT_ERR_NULL
    assert code(dtype=7) == ot.OT_ERR_DTYPE
    assert code(d=0) == ot.OT_ERR_SHAPE
    assert code(d=60) == ot.OT_ERR_SHAPE                 # bf16 rows must be 16-byte multiples
    assert code(V_t=-1) == ot.OT_ERR_SHAPE
    assert code(max_batch=0) == ot.OT_ERR_SHAPE
    assert code(max_k=64) == ot.OT_ERR_SHAPE
    assert code(max_ngram_len=1) == ot.OT_ERR_SHAPE
    assert code(max_ngram_len=9) == ot.OT_ERR_SHAPE
    assert code(draft_side=3) == ot.OT_ERR_SHAPE and code(draft_side=-1) == ot.OT_ERR_SHAPE
    dm = np.full(50, -1, np.int32)
    dm[3] = 100
    assert code(direct_map=dm) == ot.OT_ERR_MAP          # out of range
    dm[3] = -2
    assert code(direct_map=dm) == ot.OT_ERR_MAP
    dm[3], dm[9] = 7, 7
    assert code(direct_map=dm) == ot.OT_ERR_MAP          # not one-to-one
    lib = ot.load_library()
    assert lib.ot_verify_init(None, None) == ot.OT_ERR_NULL
    assert lib.ot_ngram_cache_build(None, 0, None, None, None, None) == ot.OT_ERR_NULL
    assert lib.ot_verify_step(None, None, None, None) == ot.OT_ERR_NULL
    assert lib.ot_verify_workspace(None, None) == ot.OT_ERR_NULL
    assert lib.ot_verify_profile(None, 1) == ot.OT_ERR_NULL
    lib.ot_verify_destroy(None)
    lib.ot_ngram_cache_destroy(None)


def test_missing_library_fails_loudly(monkeypatch):
    from paper_2507_02659_amd import binding as ot
    monkeypatch.setattr(ot, "_lib", None)
    monkeypatch.setattr(ot, "LIB_PATH", "/nonexistent/libotverify.so")
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        ot.load_library()


@pytest.mark.gpu
def test_step_and_cache_errors():
    import torch
    from paper_2507_02659_amd import binding as ot
    from paper_2507_02659_amd.runner import Verifier
    from workloads import CaseSpec, make_case
    spec = CaseSpec(name="abi", dtype="bf16", d=64, V_t=500, V_d=300, k=[3, 2], temperature=[1.0, 1.0], n_direct=200,
                    n_ngram=20, ngram_len=(2, 3), data_seed=1, philox_seed=1)
    case = make_case(spec)
    v = Verifier.for_case(case, max_batch=2, max_k=3)
    other = Verifier.for_case(case, max_batch=2, max_k=3)
    try:
        inp = v.upload(case)

        def step_code(**kw):
            fields = dict(B=inp["B"], step=0, row_off=inp["row_off"], row_off_host=inp["row_off_host"], hidden=inp["hidden"],
                          draft_logits=inp["draft_logits"], draft_ids=inp["draft_ids"], temperature=inp["temperature"],
                          draft_temperature=None, seq_id=inp["seq_id"], seed=0)
            fields.update(kw)
            outs = dict(inp["out"])
            if "drop_out" in fields:
                outs[fields.pop("drop_out")] = None
            cache = fields.pop("cache", v.cache)
            with pytest.raises(ot.OtError) as e:
                ot.ot_verify_step(v.ctx, cache, ot.make_step_in(**fields), ot.make_step_out(outs))
            return e.value.code

        assert step_code(B=3) == ot.OT_ERR_SHAPE
        assert step_code(B=-1) == ot.OT_ERR_SHAPE
        assert step_code(row_off=None) == ot.OT_ERR_NULL
        assert step_code(hidden=None) == ot.OT_ERR_NULL
        assert step_code(draft_ids=None) == ot.OT_ERR_NULL
        assert step_code(temperature=None) == ot.OT_ERR_NULL
        assert step_code(seq_id=None) == ot.OT_ERR_NULL
        assert step_code(drop_out="ratio") == ot.OT_ERR_NULL
        assert step_code(row_off_host=np.array([0, 4, 4], np.int32)) == ot.OT_ERR_SHAPE      # zero rows
        assert step_code(row_off_host=np.array([1, 4, 7], np.int32)) == ot.OT_ERR_SHAPE      # does not start at 0
        assert step_code(row_off_host=np.array([0, 5, 7], np.int32)) == ot.OT_ERR_SHAPE      # k = 4 > max_k
        assert step_code(cache=other.cache) == ot.OT_ERR_CTX_MISMATCH
        with pytest.raises(ot.OtError) as e:
            ot.ot_verify_step_from_logits(v.ctx, v.cache, ot.make_step_in(
                B=2, step=0, row_off=inp["row_off"], row_off_host=inp["row_off_host"], hidden=None,
                draft_logits=inp["draft_logits"], draft_ids=inp["draft_ids"], temperature=inp["temperature"],
                draft_temperature=None, seq_id=inp["seq_id"], seed=0), None, ot.make_step_out(inp["out"]))
        assert e.value.code == ot.OT_ERR_NULL

        def cache_code(key_off, key_ids, targets):
            with pytest.raises(ot.OtError) as e:
                ot.ot_ngram_cache_build(v.ctx, key_off, key_ids, targets)
            return e.value.code

        assert cache_code([0, 1], [5], [7]) == ot.OT_ERR_NGRAM                 # length 1
        assert cache_code([0, 4], [1, 2, 3, 4], [7]) == ot.OT_ERR_NGRAM        # longer than max_ngram_len = 3
        assert cache_code([0, 2], [1, 300], [7]) == ot.OT_ERR_NGRAM            # draft id out of range
        assert cache_code([0, 2], [1, 2], [500]) == ot.OT_ERR_NGRAM            # target id out of range
        # B == 0 is a no-op, an empty cache is fine, and the context still works afterwards
        ot.ot_verify_step(v.ctx, None, ot.make_step_in(B=0, step=0, row_off=None, row_off_host=None, hidden=None,
                                                       draft_logits=None, draft_ids=None, temperature=None,
                                                       draft_temperature=None, seq_id=None, seed=0),
                          ot.make_step_out({}))
        empty = ot.ot_ngram_cache_build(v.ctx, [0], [], [])
        ot.ot_ngram_cache_destroy(empty)
        v.step(inp)
        res = v.results(inp)
        assert np.all(res["n_emit"] >= 1)
        torch.cuda.synchronize()
    finally:
        v.close()
        other.close()
