"""Pins for the oracle's n-gram cache life cycle (insertion, use statistics, LRU / LFU eviction)."""
import os
import random
from collections import OrderedDict

import numpy as np
import pytest

from oracle import verify as ov
from oracle.ngram_cache import CacheFull, NgramCache

GOLD = os.path.join(os.path.dirname(__file__), "golden", "cache_eviction_trace.txt")


def _key(letter):
    i = ord(letter) - ord("A")
    return (10 + i, 20 + i)


def _trace():
    events, want = [], {}
    for ln in open(GOLD):
        ln = ln.strip()
        if not ln or ln.startswith("#"):
            continue
        head, *rest = ln.split()
        if head == "insert":
            events.append(("insert", [(_key(x.split(":")[0]), int(x.split(":")[1])) for x in rest]))
        elif head == "use":
            events.append(("use", [_key(x) for x in rest]))
        else:
            want[head] = {_key(x.split(":")[0]): tuple(int(v) for v in x.split(":")[1:]) for x in rest}
    return events, want


@pytest.mark.parametrize("policy", ["lru", "lfu"])
def test_hand_worked_eviction_trace(policy):
    events, want = _trace()
    c = NgramCache(3, policy)
    for kind, arg in events:
        c.insert(arg) if kind == "insert" else c.record_step(arg)
    assert c.snapshot() == want[policy]


def test_without_eviction_it_is_the_plain_dictionary():
    rng = np.random.default_rng(0)
    lens = rng.integers(2, 5, size=300)
    key_off = np.concatenate([[0], np.cumsum(lens)])
    key_ids = rng.integers(0, 6, size=key_off[-1])            # tiny alphabet: many duplicate keys
    targets = rng.integers(0, 1000, size=300)
    items = [(tuple(key_ids[key_off[e]:key_off[e + 1]]), targets[e]) for e in range(300)]
    ref = ov.build_cache(key_off, key_ids, targets)
    one = NgramCache(len(ref), "none")
    one.insert(items)
    assert one.as_dict() == ref
    many = NgramCache(len(ref), "none")
    for it in items:                                          # one call per pair: same final mapping
        many.insert([it])
    assert many.as_dict() == ref


def test_full_cache_without_policy_rejects_the_whole_call():
    c = NgramCache(2, "none")
    c.insert([((1, 2), 5)])
    before = (c.snapshot(), c.clock)
    with pytest.raises(CacheFull):
        c.insert([((1, 2), 6), ((3, 4), 7), ((5, 6), 8)])
    assert (c.snapshot(), c.clock) == before
    c.insert([((1, 2), 6), ((3, 4), 7)])                      # a known key needs no new place
    assert c.as_dict() == {(1, 2): 6, (3, 4): 7}


def test_lru_matches_the_textbook_ordered_dict():
    """One access or one insertion per tick, so recency is a total order: the classic move-to-end LRU."""
    rnd = random.Random(1)
    cap = 8
    c = NgramCache(cap, "lru")
    ref = OrderedDict()
    for _ in range(3000):
        key = (rnd.randrange(0, 5), rnd.randrange(0, 5))
        if key in ref and rnd.random() < 0.6:
            c.record_step([key])
            ref.move_to_end(key)
        else:
            t = rnd.randrange(0, 100)
            c.insert([(key, t)])
            if key not in ref and len(ref) >= cap:
                ref.popitem(last=False)
            ref[key] = t
            ref.move_to_end(key)
        assert c.as_dict() == dict(ref)


def test_lfu_evicts_a_least_used_entry_and_keeps_counts():
    rnd = random.Random(2)
    cap = 6
    c = NgramCache(cap, "lfu")
    uses = {}
    for _ in range(3000):
        key = (rnd.randrange(0, 4), rnd.randrange(0, 5))
        if key in uses and rnd.random() < 0.7:
            times = 2 if rnd.random() < 0.3 else 1
            c.record_step([key] * times)
            uses[key] += times
        else:
            before = dict(uses)
            c.insert([(key, 1)])
            if key not in before:
                gone = set(before) - set(c.entries)
                if len(before) >= cap:
                    assert len(gone) == 1
                    victim = gone.pop()
                    assert before[victim] == min(before.values())      # a least frequently used entry went
                    del uses[victim]
                else:
                    assert not gone
                uses[key] = 0
        assert {k: v[1] for k, v in c.entries.items()} == uses
        assert len(c) <= cap


def test_used_keys_reported_by_the_verification_oracle():
    dmap = np.arange(30)
    cache = {(1, 2): 20, (4, 5, 6): 21}
    Z = np.zeros((7, 40), np.float32)
    Zq = np.zeros((6, 30), np.float32)
    o = ov.verify_step(row_off=[0, 7], draft_ids=[1, 2, 3, 4, 5, 6], draft_logits=Zq, direct_map=dmap, V_t=40,
                       cache=cache, max_ngram_len=3, temperature=[1.0], seed=0, seq_id=[0], step=0, dtype="f32",
                       target_logits=Z)
    assert o["used_keys"] == [(1, 2), (4, 5, 6)] and o["hits_proposed"][0] == 2


@pytest.mark.parametrize("policy", ["none", "lru", "lfu"])
def test_an_insert_call_without_pairs_changes_nothing(policy):
    """There is no event to date: the clock does not tick, no stamp moves."""
    c = NgramCache(4, policy)
    c.insert([((1, 2), 7)])
    c.record_step([(1, 2)])
    before = (c.clock, c.snapshot())
    assert c.insert([]) == 0
    assert (c.clock, c.snapshot()) == before


def test_load_keeps_statistics_and_therefore_the_victims():
    """Hand example: X was used twice, long ago; Y never, recently.  After a save / load LRU still evicts X first and
    LFU still evicts Y first; a plain re-insert would have forgotten both facts."""
    saved = [((1, 2), 10, 2, 5), ((3, 4), 11, 0, 7)]           # (key, target, uses, last_used) in insertion order
    for policy, victim in (("lru", (1, 2)), ("lfu", (3, 4))):
        c = NgramCache(2, policy)
        c.load(saved)
        assert c.clock == 7 and c.snapshot() == {(1, 2): (10, 2, 5), (3, 4): (11, 0, 7)}
        assert c.insert([((5, 6), 12)]) == 1
        assert victim not in c.entries and len(c) == 2
    with pytest.raises(CacheFull):
        NgramCache(1, "lru").load(saved)


@pytest.mark.parametrize("policy", ["lru", "lfu"])
def test_export_then_load_continues_like_the_original(policy):
    rng = random.Random(17)
    pool = [((a, b), 100 + 7 * a + b) for a in range(6) for b in range(6)]
    a = NgramCache(9, policy)
    for _ in range(60):
        a.insert(rng.sample(pool, rng.randint(1, 3)))
        a.record_step(rng.choices(list(a.entries), k=rng.randint(0, 3)))
    b = NgramCache(9, policy)
    b.load(a.export())
    b.clock = a.clock                       # the original may have ticked since its latest stamp
    assert b.snapshot() == a.snapshot()
    for _ in range(60):
        items = rng.sample(pool, rng.randint(1, 3))
        used_from = list(a.entries)
        assert a.insert(items) == b.insert(items)
        used = rng.choices(list(a.entries), k=rng.randint(0, 3))
        a.record_step(used)
        b.record_step(used)
        assert a.snapshot() == b.snapshot() and a.export() == b.export()
