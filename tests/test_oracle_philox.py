"""Pins for the oracle's Philox4x32-10 and its uniform construction."""
import os

import numpy as np

from oracle import philox

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def _vectors():
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            w = [int(x, 16) for x in line.split()]
            yield w[0:4], w[4:6], tuple(w[6:10])


def test_known_answer_vectors():
    n = 0
    for ctr, key, want in _vectors():
        assert philox.philox4x32_10(ctr, key) == want
        n += 1
    assert n == 3


def test_uniform_construction():
    # the counter layout is (position, step, sequence low, sequence high); key = (seed low, seed high)
    seed, seq, step, j = 0x299F31D0A4093822, 0x0370734413198A2E, 0x85A308D3, 0x243F6A88
    u_acc, u_fin = philox.uniforms(seed, seq, step, j)
    assert u_acc == (0xD16CFE09 >> 8) / 2.0 ** 24
    assert u_fin == (0x94FDCCEB >> 8) / 2.0 ** 24
    # exactly representable in binary32
    assert np.float32(u_acc) == u_acc and np.float32(u_fin) == u_fin


def test_uniforms_are_uniform_and_distinct_per_coordinate():
    us = np.array([philox.uniforms(7, s, t, j) for s in range(20) for t in range(20) for j in range(10)])
    assert us.min() >= 0.0 and us.max() < 1.0
    # mean of 4000 U[0,1) draws: sd = 0.0046
    assert abs(us[:, 0].mean() - 0.5) < 0.02 and abs(us[:, 1].mean() - 0.5) < 0.02
    assert abs(np.corrcoef(us[:, 0], us[:, 1])[0, 1]) < 0.06
    assert len({tuple(r) for r in us}) == len(us)
    # each coordinate changes the draw
    base = philox.uniforms(1, 2, 3, 4)
    assert philox.uniforms(2, 2, 3, 4) != base
    assert philox.uniforms(1, 3, 3, 4) != base
    assert philox.uniforms(1, 2, 4, 4) != base
    assert philox.uniforms(1, 2, 3, 5) != base
    assert philox.uniforms(1 + (1 << 32), 2, 3, 4) != base
    assert philox.uniforms(1, 2 + (1 << 32), 3, 4) != base
