"""The library's host-side n-gram table (plain C++: probing, backward-shift deletion, eviction order, import/export) and
its argument checks, built with AddressSanitizer + UndefinedBehaviorSanitizer and driven with 10^4 random operations
against the oracle's cache.  No GPU involved: this is the host code that otherwise only runs on the GPU machine."""
import os
import subprocess

import numpy as np
import pytest

from oracle.ngram_cache import CacheFull, NgramCache

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2507_02659_amd", "csrc")
POLICY = {"none": 0, "lru": 1, "lfu": 2}


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("host_table") / "host_table_driver")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
           "-Wall", "-Wextra", "-Werror", "-I", CSRC, os.path.join(ROOT, "tests", "host_table_driver.cpp"),
           os.path.join(CSRC, "ngram_table.cpp"), "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    return exe


def _items(lines, items, with_target=True, stats=None):
    for i, it in enumerate(items):
        key = it[0]
        row = [len(key), *key]
        if with_target:
            row.append(it[1])
        if stats is not None:
            row += [it[2], it[3]]
        lines.append(" ".join(str(int(v)) for v in row))


def _parse_dumps(out):
    dumps, cur = [], None
    for ln in out.splitlines():
        if ln.startswith("state"):
            w = ln.split()
            cur = {"clock": int(w[2]), "entries": []}
        elif ln.startswith("entry"):
            left, right = ln[len("entry"):].split("->")
            key = tuple(int(v) for v in left.split())
            w = right.split()
            cur["entries"].append((key, int(w[0]), int(w[2]), int(w[4])))
        elif ln == "end":
            dumps.append(cur)
    return dumps


@pytest.mark.parametrize("policy,capacity", [("lru", 24), ("lfu", 24), ("lru", 1), ("lfu", 3), ("none", 400)])
def test_random_operations_against_the_oracle(driver, policy, capacity):
    rng = np.random.default_rng(capacity * 7 + POLICY[policy])
    ref = NgramCache(capacity, policy)
    lines = [f"init {capacity} {POLICY[policy]} 6"]
    want = []
    n_ops = 2500
    for op in range(n_ops):
        kind = rng.choice(["insert", "step", "step", "roundtrip"], p=[0.55, 0.3, 0.1, 0.05])
        if kind == "insert":
            items = []
            for _ in range(int(rng.integers(0, 6))):
                L = int(rng.integers(2, 7))
                items.append((tuple(int(v) for v in rng.integers(0, 5, size=L)), int(rng.integers(0, 1000))))   # small alphabet: keys recur and collide
            try:
                ref.insert(items)
                ok = True
            except CacheFull:
                ok = False
            lines.append(f"insert {len(items)}")
            _items(lines, items)
        elif kind == "step" and len(ref):
            keys = list(ref.entries)
            used = [keys[int(i)] for i in rng.integers(0, len(keys), size=int(rng.integers(0, 5)))]
            ref.record_step(used)
            lines.append(f"step {len(used)}")
            _items(lines, [(k,) for k in used], with_target=False)
        elif kind == "roundtrip":
            # what the table exports, loaded into a fresh oracle cache, must keep going like the original
            saved = ref.export()
            fresh = NgramCache(capacity, policy)
            fresh.load(saved)
            ref = fresh
            lines.append(f"init {capacity} {POLICY[policy]} 6")
            lines.append(f"import {len(saved)}")
            _items(lines, saved, stats=True)
            lines.append("step 0")
            ref.record_step([])
        if op % 25 == 0 or op == n_ops - 1:
            lines.append("dump")
            want.append((ref.clock, ref.export()))
    r = subprocess.run([driver], input="\n".join(lines) + "\n", capture_output=True, text=True)
    assert r.returncode == 0, (r.stdout[-2000:], r.stderr[-4000:])
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-4000:]
    dumps = _parse_dumps(r.stdout)
    assert len(dumps) == len(want)
    for i, (got, exp) in enumerate(zip(dumps, want)):
        assert got["entries"] == exp[1], f"dump {i}"
        assert got["clock"] == exp[0], f"dump {i}"


def test_row_offset_and_entry_checks(driver):
    script = "\n".join([
        "init 4 0 3",
        "offsets 3 5 0 2 3 9",          # fine: k = 1, 0, 5
        "offsets 3 5 0 2 2 9",          # second sequence owns no row
        "offsets 2 3 0 5 6",            # first sequence drafted 4 > max_k
        "offsets 1 3 1 2",              # does not start at 0
        "insert 1", "1 7 5",            # key too short
        "insert 1", "4 1 2 3 4 5",      # key too long for max_len 3
        "insert 1", "2 1 -2 5",         # negative draft id
        "insert 1", "2 1 2 5",
        "dump"]) + "\n"
    r = subprocess.run([driver], input=script, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    out = r.stdout.splitlines()
    assert out[:4] == ["offsets 0", "offsets 2", "offsets 1", "offsets 1"]
    assert out[4].startswith("rejected") and out[5].startswith("rejected") and out[6].startswith("rejected")
    assert out[7].startswith("evicted 0")
    assert _parse_dumps(r.stdout)[0]["entries"] == [((1, 2), 5, 0, 1)]
