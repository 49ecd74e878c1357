"""Pins for the oracle's Philox4x32-10: published known-answer values, an
independent vectorised uint64 implementation, and uniformity of the 24-bit draw."""
import os

import numpy as np
from scipy import stats

from oracle.philox import philox4x32_10, uniform24


def _philox_np(ctr, key):
    """Independent formulation: numpy uint64 lanes, key schedule precomputed."""
    c = np.array(ctr, dtype=np.uint64)
    ks = [(np.uint64(key[0]) + np.uint64(r) * np.uint64(0x9E3779B9)) % np.uint64(1 << 32) for r in range(10)]
    kt = [(np.uint64(key[1]) + np.uint64(r) * np.uint64(0xBB67AE85)) % np.uint64(1 << 32) for r in range(10)]
    lo32 = np.uint64(0xFFFFFFFF)
    for r in range(10):
        a = np.uint64(0xD2511F53) * c[0]
        b = np.uint64(0xCD9E8D57) * c[2]
        c = np.array([(b >> np.uint64(32)) ^ c[1] ^ ks[r], b & lo32,
                      (a >> np.uint64(32)) ^ c[3] ^ kt[r], a & lo32], dtype=np.uint64)
    return tuple(int(x) for x in c)


def test_known_answers(golden_dir):
    rows = [l.split() for l in open(os.path.join(golden_dir, "philox4x32_10_kat.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        v = [int(x, 16) for x in r]
        assert philox4x32_10(v[0:4], v[4:6]) == tuple(v[6:10])


def test_against_independent_implementation():
    rng = np.random.default_rng(5)
    for _ in range(200):
        ctr = [int(x) for x in rng.integers(0, 1 << 32, 4, dtype=np.uint64)]
        key = [int(x) for x in rng.integers(0, 1 << 32, 2, dtype=np.uint64)]
        assert philox4x32_10(ctr, key) == _philox_np(ctr, key)


def test_uniform24_range_and_uniformity():
    u = np.array([uniform24(12345, p, h, 3) for p in range(4000) for h in range(5)])
    assert u.min() >= 0.0 and u.max() < 1.0
    assert np.all(u * 16777216 == np.floor(u * 16777216))           # exactly 24 bits
    counts, _ = np.histogram(u, bins=20, range=(0, 1))
    assert stats.chisquare(counts).pvalue > 1e-3
    # draws differ by position, head, sequence and seed
    base = uniform24(1, 10, 2, 3)
    assert len({base, uniform24(1, 11, 2, 3), uniform24(1, 10, 3, 3), uniform24(1, 10, 2, 4),
                uniform24(2, 10, 2, 3), uniform24(1 + (1 << 32), 10, 2, 3)}) == 6
