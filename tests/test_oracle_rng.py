"""Pins for the oracle's random stream and its integer exponential clock."""
import math
import os

import numpy as np

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def test_philox_known_answers():
    n = 0
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        w = [int(x, 16) for x in line.split()]
        assert oracle.philox4x32_10(w[0:4], w[4:6]) == w[6:10]
        n += 1
    assert n == 3


def test_stream_keying_layout():
    # counter = (slot>>2, node, batch, epoch<<8 | domain<<4 | layer), key = (seed lo, seed hi)
    seed, epoch, batch, layer, node = 0x0123456789ABCDEF, 77, 5, 2, 4242
    for slot in (0, 1, 2, 3, 4, 9, 1023):
        words = oracle.philox4x32_10([slot >> 2, node, batch, (epoch << 8) | (2 << 4) | layer],
                                     [seed & 0xFFFFFFFF, seed >> 32])
        assert oracle.slot_word(seed, epoch, batch, layer, node, slot) == words[slot & 3]
    for domain, ident in ((0, 17), (1, 99999)):
        w = oracle.philox4x32_10([0, ident, 0, (epoch << 8) | (domain << 4)],
                                 [seed & 0xFFFFFFFF, seed >> 32])
        assert oracle.shuffle_key(seed, epoch, domain, ident) == (w[0] << 32) | w[1]


def test_stream_is_equidistributed():
    words = np.array([oracle.slot_word(7, 1, 0, 0, 3, s) for s in range(40000)], dtype=np.uint64)
    u = words.astype(np.float64) / 2.0 ** 32
    assert abs(u.mean() - 0.5) < 0.01
    assert abs(u.var() - 1.0 / 12.0) < 0.005
    bits = ((words[:, None] >> np.arange(32, dtype=np.uint64)[None, :]) & 1).mean(axis=0)
    assert np.all(np.abs(bits - 0.5) < 0.02)
    # distinct (node, layer, batch, epoch) give different streams
    a = [oracle.slot_word(7, 1, 0, 0, 3, s) for s in range(64)]
    for other in ((7, 1, 0, 0, 4), (7, 1, 0, 1, 3), (7, 1, 1, 0, 3), (7, 2, 0, 0, 3), (8, 1, 0, 0, 3)):
        b = [oracle.slot_word(*other, s) for s in range(64)]
        assert sum(x == y for x, y in zip(a, b)) == 0


def test_exp_clock_matches_log2():
    # E(r) = -log2((2r+1)/2^33) in Q24: compare with the library logarithm
    rng = np.random.default_rng(1)
    rs = list(rng.integers(0, 2 ** 32, size=20000, dtype=np.uint64)) + [0, 1, 2, 3, 2 ** 31 - 1, 2 ** 31, 2 ** 32 - 1]
    worst = 0.0
    for r in rs:
        r = int(r)
        exact = -math.log2((2 * r + 1) / 2.0 ** 33)
        worst = max(worst, abs(oracle.exp_clock_q24(r) / 2.0 ** 24 - exact))
    assert worst < 2.0 ** -22, worst
    assert oracle.exp_clock_q24(0) == 33 << 24
    assert oracle.exp_clock_q24(2 ** 32 - 1) >= 0


def test_exp_clock_is_monotone():
    rng = np.random.default_rng(2)
    rs = np.sort(rng.integers(0, 2 ** 32, size=5000, dtype=np.uint64))
    e = [oracle.exp_clock_q24(int(r)) for r in rs]
    assert all(e[i] >= e[i + 1] for i in range(len(e) - 1))
    # also over a dense run of consecutive words
    e = [oracle.exp_clock_q24(r) for r in range(10 ** 6, 10 ** 6 + 3000)]
    assert all(e[i] >= e[i + 1] for i in range(len(e) - 1))


def test_slot_key_special_cases():
    q = oracle.q_intra
    assert q(0.5) == 32768 and q(1.0) == 65536 and q(0.9) == 58982
    for r in (0, 5, 2 ** 32 - 1):
        assert oracle.slot_key(r, True, q(0.5)) == r == oracle.slot_key(r, False, q(0.5))
        assert oracle.slot_key(r, True, q(1.0)) == r
        assert oracle.slot_key(r, False, q(1.0)) == (1 << 62) + r
        e = oracle.exp_clock_q24(r)
        assert oracle.slot_key(r, True, q(0.9)) == e * (65536 - q(0.9))
        assert oracle.slot_key(r, False, q(0.9)) == e * q(0.9)
