"""Pins for the oracle's Philox4x32-10 and its uniform mapping."""
import os

import numpy as np

import oracle

MASK = 0xFFFFFFFF


def philox_bigint(ctr, key, rounds=10):
    """Independent implementation with Python integers, written from the SC'11 paper:
    each round multiplies counter words 0 and 2 by the two round multipliers, crosses
    the high halves over, xors in the neighbours and the key, then bumps the key by
    the two Weyl constants (golden ratio, sqrt(3) - 1)."""
    c = list(ctr)
    k = list(key)
    for r in range(rounds):
        p0 = 0xD2511F53 * c[0]
        p1 = 0xCD9E8D57 * c[2]
        c = [((p1 >> 32) ^ c[1] ^ k[0]) & MASK, p1 & MASK,
             ((p0 >> 32) ^ c[3] ^ k[1]) & MASK, p0 & MASK]
        k = [(k[0] + 0x9E3779B9) & MASK, (k[1] + 0xBB67AE85) & MASK]
    return c


def test_known_answer_vectors(golden_dir):
    rows = [l.split() for l in open(os.path.join(golden_dir, "philox4x32_10_kat.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        v = [int(x, 16) for x in r]
        assert oracle.philox4x32_10(v[0:4], v[4:6]) == v[6:10]
        assert philox_bigint(v[0:4], v[4:6]) == v[6:10]


def test_matches_bigint_on_random_counters():
    rng = np.random.default_rng(7)
    for _ in range(20000):
        ctr = [int(x) for x in rng.integers(0, 2**32, 4)]
        key = [int(x) for x in rng.integers(0, 2**32, 2)]
        assert oracle.philox4x32_10(ctr, key) == philox_bigint(ctr, key)


def test_bijective_on_a_counter_block():
    # a block cipher in counter mode: distinct counters give distinct 128-bit outputs
    seen = set()
    for i in range(1 << 14):
        out = tuple(oracle.philox4x32_10([i, 3, 0, 0], [42, 0]))
        seen.add(out)
    assert len(seen) == 1 << 14


def test_uniform_mapping():
    # word -> ((word >> 9) + 0.5) / 2^23 with the documented counter layout
    seed, step, row = 0x123456789ABCDEF, (5 << 32) | 77, 9
    for i in (0, 1, 2, 3, 4, 7, 1001, 152063):
        w = philox_bigint([i >> 2, row, step & MASK, step >> 32], [seed & MASK, seed >> 32])
        k = w[i & 3] >> 9
        u = oracle.uniform(seed, step, row, i)
        assert u == (k + 0.5) / 2**23
        assert 2.0**-24 <= u <= 1 - 2.0**-24
        assert float(np.float32(u)) == u  # exact in binary32


def test_uniform_statistics():
    n = 200000
    u = np.array([oracle.uniform(11, 0, 0, i) for i in range(n)])
    hist, _ = np.histogram(u, bins=64, range=(0, 1))
    chi2 = ((hist - n / 64) ** 2 / (n / 64)).sum()
    assert chi2 < 120  # 63 dof, p ~ 1e-5
    assert abs(u.mean() - 0.5) < 4 * (1 / 12**0.5) / n**0.5
    # different step, row or seed changes the stream
    assert oracle.uniform(11, 1, 0, 5) != oracle.uniform(11, 0, 0, 5)
    assert oracle.uniform(11, 0, 1, 5) != oracle.uniform(11, 0, 0, 5)
    assert oracle.uniform(12, 0, 0, 5) != oracle.uniform(11, 0, 0, 5)
