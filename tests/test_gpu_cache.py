"""Life cycle of the n-gram cache on the device (online insertion, use statistics, LRU / LFU eviction, export)
against the oracle's cache, through the C ABI.  Needs a real MI355X."""
import numpy as np
import pytest

from workloads import CaseSpec, make_case

pytestmark = pytest.mark.gpu


def _csr(items):
    key_off = np.concatenate([[0], np.cumsum([len(k) for k, _ in items])]).astype(np.int32)
    key_ids = np.array([v for k, _ in items for v in k], dtype=np.int32)
    targets = np.array([t for _, t in items], dtype=np.int32)
    return key_off, key_ids, targets


def _export_as_dict(ot, cache):
    ex = ot.ot_ngram_cache_export(cache)
    out = {}
    for e in range(ex["target_ids"].size):
        key = tuple(int(v) for v in ex["key_ids"][ex["key_off"][e]:ex["key_off"][e + 1]])
        out[key] = (int(ex["target_ids"][e]), int(ex["uses"][e]), int(ex["last_used"][e]))
    return out, ex


@pytest.mark.parametrize("policy", ["lru", "lfu", "none"])
def test_online_cache_matches_oracle(policy):
    from oracle import verify as ov
    from oracle.ngram_cache import CacheFull, NgramCache
    from paper_2507_02659_amd import binding as ot
    from paper_2507_02659_amd.runner import Verifier
    import parity

    rng = np.random.default_rng({"lru": 1, "lfu": 2, "none": 3}[policy])
    spec = CaseSpec(name=f"cache_{policy}", dtype="f32", d=16, V_t=900, V_d=300, k=[6] * 8, temperature=[1.0] * 8,
                    n_direct=260, data_seed=11, philox_seed=12, logits_only=True, max_ngram_len=4, align=0.5)
    case = make_case(spec)
    free_targets = np.setdiff1d(np.arange(case.V_t), case.direct_map[case.direct_map >= 0])
    # a pool of candidate pairs over a small alphabet, so that keys recur and windows hit them by construction
    pool = []
    while len(pool) < 150:
        L = int(rng.integers(2, 5))
        key = tuple(int(v) for v in rng.integers(0, 40, size=L))
        if key not in {k for k, _ in pool}:
            pool.append((key, int(rng.choice(free_targets))))
    capacity = 200 if policy == "none" else 40
    code = {"none": ot.OT_EVICT_NONE, "lru": ot.OT_EVICT_LRU, "lfu": ot.OT_EVICT_LFU}[policy]
    ref = NgramCache(capacity, policy)
    v = Verifier.for_case(case)
    cache = ot.ot_ngram_cache_create(v.ctx, capacity, code)
    report = parity.Report()
    try:
        for step in range(40):
            # ---- online insertion: a few pairs, some known keys with a changed target
            picks = [pool[int(i)] for i in rng.integers(0, len(pool), size=int(rng.integers(1, 9)))]
            if step % 7 == 3:
                picks = [(k, int(rng.choice(free_targets))) for k, _ in picks]
            if step == 20:                                  # one large call goes through the bulk path
                picks = [pool[int(i)] for i in rng.permutation(len(pool))[:60]]
            want_evicted = ref.insert(picks)
            got_evicted = ot.ot_ngram_cache_insert(cache, *_csr(picks))
            assert got_evicted == want_evicted, (step, got_evicted, want_evicted)
            assert ot.ot_ngram_cache_size(cache)[0] == len(ref)
            # ---- a step whose windows contain keys that are in the cache right now
            known = list(ref.entries)
            ids = rng.integers(0, case.V_d, size=case.K).astype(np.int32)
            for b in range(case.B):
                key = known[int(rng.integers(0, len(known)))]
                at = 6 * b + int(rng.integers(0, 6 - len(key) + 1))
                ids[at:at + len(key)] = key
            case.draft_ids = ids
            case.step = step
            inp = v.upload(case)
            sin = ot.make_step_in(B=inp["B"], step=step, row_off=inp["row_off"], row_off_host=inp["row_off_host"],
                                  hidden=None, draft_logits=inp["draft_logits"], draft_ids=inp["draft_ids"],
                                  temperature=inp["temperature"], draft_temperature=None, seq_id=inp["seq_id"],
                                  seed=inp["seed"])
            ot.ot_verify_step_from_logits(v.ctx, cache, sin, inp["target_logits"], ot.make_step_out(inp["out"]))
            gpu = v.results(inp)
            o = ov.verify_step(row_off=case.row_off, draft_ids=ids, draft_logits=case.draft_logits,
                               direct_map=case.direct_map, V_t=case.V_t, cache=ref.as_dict(), max_ngram_len=4,
                               temperature=case.temperature, seed=case.seed, seq_id=case.seq_id, step=step,
                               dtype="f32", target_logits=case.target_logits)
            ref.record_step(o["used_keys"])
            report.merge(parity.compare(case, gpu, o, logits_from_gpu=False))
            assert o["hits_proposed"].sum() >= 1
            if step % 5 == 4:
                if step % 10 == 9:
                    # a maintenance call that fails after it has read the device's use log (no room for the entries)
                    # leaves the log in place; the uses in it must not be counted again by the next call
                    tiny = np.zeros(4, np.int32)
                    with pytest.raises(ot.OtError) as e:
                        ot._check(ot.load_library().ot_ngram_cache_export(cache, 0, 0, ot._ptr(tiny), ot._ptr(tiny), ot._ptr(tiny),
                                                                        None, None))
                    assert e.value.code == ot.OT_ERR_SHAPE
                got, _ = _export_as_dict(ot, cache)
                assert got == ref.snapshot(), step
        print("  " + report.summary(), flush=True)
        assert not report.failures, "\n".join(report.failures[:10])
        assert report.divergent <= 2
        got, ex = _export_as_dict(ot, cache)
        assert got == ref.snapshot()
        if policy != "none":
            assert len(ref) == capacity                    # the cache ran full and evicted
        # ---- save / load: an export imported into a fresh cache carries the statistics along, so that both caches go
        # on evicting the same entries; re-inserting it instead keeps the mapping only
        again = ot.ot_ngram_cache_create(v.ctx, capacity, code)
        ot.ot_ngram_cache_import(again, ex["key_off"], ex["key_ids"], ex["target_ids"], ex["uses"], ex["last_used"])
        got2, ex2 = _export_as_dict(ot, again)
        assert got2 == ref.snapshot()
        assert np.array_equal(ex2["key_ids"], ex["key_ids"]) and np.array_equal(ex2["key_off"], ex["key_off"])   # same insertion order
        if policy != "none":
            more = [((90 + i, 91 + i, 92), int(free_targets[i])) for i in range(12)]
            assert ot.ot_ngram_cache_insert(again, *_csr(more)) == ot.ot_ngram_cache_insert(cache, *_csr(more)) == ref.insert(more)
            a_state, b_state = _export_as_dict(ot, again)[0], _export_as_dict(ot, cache)[0]
            assert {k: v[:2] for k, v in a_state.items()} == {k: v[:2] for k, v in b_state.items()} == \
                   {k: v[:2] for k, v in ref.snapshot().items()}       # same survivors (the two clocks may differ)
        ot.ot_ngram_cache_destroy(again)
        plain = ot.ot_ngram_cache_create(v.ctx, max(capacity, len(ref)), code)
        ot.ot_ngram_cache_insert(plain, ex["key_off"], ex["key_ids"], ex["target_ids"])
        assert {k: t for k, (t, _, _) in _export_as_dict(ot, plain)[0].items()} == {k: t for k, (t, _, _) in got.items()}
        ot.ot_ngram_cache_destroy(plain)
        # ---- error paths
        if policy == "none":
            full = ot.ot_ngram_cache_create(v.ctx, 2, ot.OT_EVICT_NONE)
            ot.ot_ngram_cache_insert(full, *_csr([((1, 2), 5)]))
            with pytest.raises(ot.OtError) as e:
                ot.ot_ngram_cache_insert(full, *_csr([((1, 2), 6), ((3, 4), 7), ((5, 6), 8)]))
            assert e.value.code == ot.OT_ERR_SHAPE
            assert _export_as_dict(ot, full)[0] == {(1, 2): (5, 0, 1)}          # the failed call changed nothing
            ot.ot_ngram_cache_destroy(full)
            with pytest.raises(ot.OtError) as e:
                ot.ot_ngram_cache_create(v.ctx, 5, 9)
            assert e.value.code == ot.OT_ERR_SHAPE
            with pytest.raises(ot.OtError) as e:
                ot.ot_ngram_cache_create(v.ctx, -1, ot.OT_EVICT_LRU)
            assert e.value.code == ot.OT_ERR_SHAPE
    finally:
        ot.ot_ngram_cache_destroy(cache)
        v.close()


def test_bulk_build_equals_online_inserts():
    """ot_ngram_cache_build and one-by-one inserts into an empty cache translate identically."""
    from paper_2507_02659_amd import binding as ot
    from paper_2507_02659_amd.runner import Verifier
    spec = CaseSpec(name="cache_build", dtype="bf16", d=64, V_t=4000, V_d=1500, k=[7] * 16, temperature=[1.0] * 16,
                    n_direct=1200, n_ngram=300, ngram_len=(2, 5), plant_cover=0.4, data_seed=21, philox_seed=22,
                    logits_only=True)
    case = make_case(spec)
    v = Verifier.for_case(case)                         # bulk-built cache
    try:
        a = v.run_case(case)
        online = ot.ot_ngram_cache_create(v.ctx, 300, ot.OT_EVICT_LRU)
        for e in range(300):
            ko = case.ngram_key_off
            ot.ot_ngram_cache_insert(online, [0, ko[e + 1] - ko[e]], case.ngram_key_ids[ko[e]:ko[e + 1]],
                                     case.ngram_target_ids[e:e + 1])
        ot.ot_ngram_cache_destroy(v.cache)
        v.cache = online
        b = v.run_case(case)
        for name in a:
            assert np.array_equal(a[name], b[name]), name
        assert a["hits_proposed"].sum() > 0
    finally:
        v.close()


@pytest.mark.parametrize("policy", ["lru", "lfu"])
def test_full_cache_of_100k_entries_evicts_one_entry_per_step(policy):
    """Steady state of a full cache: every step is followed by an insert that evicts.  The library keeps the eviction
    order on the host and moves only the touched slots, so a call costs microseconds whatever the cache holds; the
    state is compared with the oracle's after every tenth step and at the end."""
    import ctypes
    import time
    from oracle import verify as ov
    from oracle.ngram_cache import NgramCache
    from paper_2507_02659_amd import binding as ot
    from paper_2507_02659_amd.runner import Verifier
    import parity

    lib = ot.load_library()
    rng = np.random.default_rng(5 if policy == "lru" else 6)
    capacity = 100_000
    spec = CaseSpec(name=f"cache_big_{policy}", dtype="f32", d=16, V_t=4000, V_d=3000, k=[8] * 8, temperature=[1.0] * 8,
                    n_direct=2500, data_seed=31, philox_seed=32, logits_only=True, max_ngram_len=4, align=0.5)
    case = make_case(spec)
    free_targets = np.setdiff1d(np.arange(case.V_t), case.direct_map[case.direct_map >= 0])
    keys = set()
    while len(keys) < capacity + 64:
        L = int(rng.integers(2, 5))
        keys.add(tuple(int(x) for x in rng.integers(0, case.V_d, size=L)))
    keys = sorted(keys)
    rng.shuffle(keys)
    pairs = [(k, int(rng.choice(free_targets))) for k in keys]
    ref = NgramCache(capacity, policy)
    code = {"lru": ot.OT_EVICT_LRU, "lfu": ot.OT_EVICT_LFU}[policy]
    v = Verifier.for_case(case)
    cache = ot.ot_ngram_cache_create(v.ctx, capacity, code)
    report = parity.Report()
    try:
        ot.ot_ngram_cache_insert(cache, *_csr(pairs[:capacity]))       # fills the cache in one call
        ref.insert(pairs[:capacity])
        assert ot.ot_ngram_cache_size(cache)[0] == capacity
        wall = []
        for step in range(40):
            known = pairs[int(rng.integers(0, capacity - 2000)) + 1000][0] if step else pairs[capacity // 2][0]
            live = [k for k in (known, pairs[capacity - 1 - step][0]) if k in ref.entries]
            ids = rng.integers(0, case.V_d, size=case.K).astype(np.int32)
            for b, key in enumerate(live):
                ids[8 * b:8 * b + len(key)] = key
            case.draft_ids = ids
            inp = v.upload(case)
            sin = ot.make_step_in(B=inp["B"], step=step, row_off=inp["row_off"], row_off_host=inp["row_off_host"], hidden=None,
                                  draft_logits=inp["draft_logits"], draft_ids=inp["draft_ids"], temperature=inp["temperature"],
                                  draft_temperature=None, seq_id=inp["seq_id"], seed=inp["seed"])
            ot.ot_verify_step_from_logits(v.ctx, cache, sin, inp["target_logits"], ot.make_step_out(inp["out"]))
            gpu = v.results(inp)
            o = ov.verify_step(row_off=case.row_off, draft_ids=ids, draft_logits=case.draft_logits, direct_map=case.direct_map,
                               V_t=case.V_t, cache=ref.as_dict(), max_ngram_len=4, temperature=case.temperature, seed=case.seed,
                               seq_id=case.seq_id, step=step, dtype="f32", target_logits=case.target_logits)
            ref.record_step(o["used_keys"])
            report.merge(parity.compare(case, gpu, o, logits_from_gpu=False))
            new = [pairs[capacity + step]]                            # one unseen pair: one eviction
            ko, ki, ti = _csr(new)
            ev = ctypes.c_int32()
            args = (cache, 1, ot._ptr(ko), ot._ptr(ki), ot._ptr(ti), ctypes.byref(ev))
            t0 = time.perf_counter()                                  # the library call alone, arguments marshalled before
            rc = lib.ot_ngram_cache_insert(*args)
            wall.append(time.perf_counter() - t0)
            ot._check(rc)
            assert ev.value == ref.insert(new) == 1
            if step % 10 == 9:
                assert _export_as_dict(ot, cache)[0] == ref.snapshot(), step
        print(f"  insert with one eviction at {capacity} entries: median {1e6 * np.median(wall):.1f} us, "
              f"max {1e6 * max(wall):.1f} us; " + report.summary(), flush=True)
        assert not report.failures, "\n".join(report.failures[:10])
        assert _export_as_dict(ot, cache)[0] == ref.snapshot()
        assert np.median(wall) < 2e-4          # about 45 us on an idle box; a whole-table round trip took milliseconds
    finally:
        ot.ot_ngram_cache_destroy(cache)
        v.close()
