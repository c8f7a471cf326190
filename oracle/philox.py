"""Philox4x32-10 counter-based generator, plain Python integers.

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg; the product path never touches this package.

The algorithm is the public one of Salmon, Moraes, Dror and Shaw, "Parallel
random numbers: as easy as 1, 2, 3" (SC'11): ten rounds, each round multiplies
counter words 0 and 2 by two fixed odd constants, keeps the 64-bit products'
high and low halves, mixes the high halves with the other two counter words and
the key, and the key is advanced by two Weyl constants between rounds.  Pinned
by the known-answer vectors in tests/golden/philox4x32_10_kat.txt.

The verification step keys its uniforms on (seed, sequence, step, position):
key = (seed low word, seed high word), counter = (position j, step, sequence id
low word, sequence id high word).  Word 0 of the output decides acceptance at
mapped position j, word 1 drives the final-token draw at row j.  A uniform is
the top 24 bits of a word times 2^-24: exactly representable in binary32 and
binary64, so a GPU and this code compare the very same number.
"""
from __future__ import annotations

_MASK = 0xFFFFFFFF
_MUL0 = 0xD2511F53
_MUL1 = 0xCD9E8D57
_WEYL0 = 0x9E3779B9
_WEYL1 = 0xBB67AE85


def philox4x32_10(counter, key):
    """counter: 4 words, key: 2 words (each 0..2^32-1) -> tuple of 4 output words."""
    c0, c1, c2, c3 = (int(c) & _MASK for c in counter)
    k0, k1 = (int(k) & _MASK for k in key)
    for _ in range(10):
        prod0 = _MUL0 * c0
        prod1 = _MUL1 * c2
        c0, c1, c2, c3 = ((prod1 >> 32) ^ c1 ^ k0) & _MASK, prod1 & _MASK, ((prod0 >> 32) ^ c3 ^ k1) & _MASK, prod0 & _MASK
        k0 = (k0 + _WEYL0) & _MASK
        k1 = (k1 + _WEYL1) & _MASK
    return c0, c1, c2, c3


def uniforms(seed: int, seq_id: int, step: int, j: int):
    """(u_accept, u_final) in [0,1) for mapped position / row j of one sequence."""
    seed = int(seed) & 0xFFFFFFFFFFFFFFFF
    seq_id = int(seq_id) & 0xFFFFFFFFFFFFFFFF
    x = philox4x32_10((j, step, seq_id & _MASK, seq_id >> 32), (seed & _MASK, seed >> 32))
    return (x[0] >> 8) * 2.0 ** -24, (x[1] >> 8) * 2.0 ** -24
