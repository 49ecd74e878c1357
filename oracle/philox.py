"""Philox4x32-10 counter-based generator (Salmon, Moraes, Dror, Shaw, SC'11),
written out with Python integers.  Test infrastructure only.

The method's random draws (resampling with "token probabilities serving as
sampling weights", paper appendix "Independent Sampling"; first candidates
x_{1:D} ~ U(0,V), Alg. 1) are keyed by (seed; position, head, sequence), so a
draw depends on where it is used, not on how many draws preceded it.
"""

_M0 = 0xD2511F53          # multipliers of the two 32x32->64 products
_M1 = 0xCD9E8D57
_W0 = 0x9E3779B9          # Weyl increments of the two key words
_W1 = 0xBB67AE85
_MASK = 0xFFFFFFFF


def philox4x32_10(counter, key):
    """counter: 4 uint32, key: 2 uint32 -> 4 uint32 after ten rounds."""
    c0, c1, c2, c3 = (int(c) & _MASK for c in counter)
    k0, k1 = (int(k) & _MASK for k in key)
    for rnd in range(10):
        if rnd > 0:
            k0 = (k0 + _W0) & _MASK
            k1 = (k1 + _W1) & _MASK
        p0 = _M0 * c0
        p1 = _M1 * c2
        hi0, lo0 = p0 >> 32, p0 & _MASK
        hi1, lo1 = p1 >> 32, p1 & _MASK
        c0, c1, c2, c3 = hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0
    return c0, c1, c2, c3


def uniform24(seed: int, pos: int, head: int, seq_id: int) -> float:
    """Uniform in [0,1) with 24 random bits: counter (pos, head, seq_id, 0),
    key = the two halves of the 64-bit seed, first output word >> 8."""
    out = philox4x32_10((pos, head, seq_id, 0), (seed & _MASK, (seed >> 32) & _MASK))
    return (out[0] >> 8) * (1.0 / 16777216.0)
