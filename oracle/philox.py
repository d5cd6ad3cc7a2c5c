"""Philox4x32-10 counter-based generator (Salmon, Moraes, Dror, Shaw:
"Parallel Random Numbers: As Easy as 1, 2, 3", SC'11, Sec. 3.3).

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

The rollout samples with a temperature (paper Sec. 4.1 "Implementation
Details"); which generator draws the uniform numbers is not part of the
method, so this build fixes one that is a pure function of (key, counter):
ten rounds of
    (hi0, lo0) = M0 * c0      (hi1, lo1) = M1 * c2        (32x32 -> 64 bit)
    c' = (hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0)
with the key bumped by the Weyl constants between rounds.
Plain Python integers: slow and obviously right.
"""
M0 = 0xD2511F53
M1 = 0xCD9E8D57
W0 = 0x9E3779B9
W1 = 0xBB67AE85
MASK32 = 0xFFFFFFFF


def philox4x32_10(counter, key):
    """counter: 4 uint32, key: 2 uint32 -> 4 uint32 (tuple of Python ints)."""
    c0, c1, c2, c3 = (int(c) & MASK32 for c in counter)
    k0, k1 = (int(k) & MASK32 for k in key)
    for rnd in range(10):
        if rnd:
            k0 = (k0 + W0) & MASK32
            k1 = (k1 + W1) & MASK32
        p0 = M0 * c0
        p1 = M1 * c2
        hi0, lo0 = p0 >> 32, p0 & MASK32
        hi1, lo1 = p1 >> 32, p1 & MASK32
        c0, c1, c2, c3 = hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0
    return c0, c1, c2, c3


def uniform_u64(seed: int, seq_id: int, step: int) -> int:
    """The one 64-bit draw the sampler uses for (rollout seq_id, decode step):
    counter = (step, seq_id low, seq_id high, 0), key = (seed low, seed high);
    u = out1 * 2^32 + out0."""
    out = philox4x32_10((step, seq_id & MASK32, (seq_id >> 32) & MASK32, 0),
                        (seed & MASK32, (seed >> 32) & MASK32))
    return (out[1] << 32) | out[0]
