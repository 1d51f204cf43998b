"""The LABOR-0 shortcut for the longest lists of a symmetric graph lists the vertices with a small variate through the
inverse of the 32-bit mixer that makes the variates (App. A.7, c = 0: R_t = mix(t ^ K0) ^ K1).  The inverse lives in the
HIP sources; this test takes its constants from there, restates it in integer numpy, and checks it against the oracle's
mixer (C, built from the paper's description independently of the HIP path): the composition must be the identity.
A wrong constant, shift or order of steps fails here without a GPU."""
import os
import re

import numpy as np

from oracle import coopref as R

SRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2310_12403_amd", "csrc", "variates.h")
M32 = np.uint64(0xFFFFFFFF)


def body(name):
    text = open(SRC).read()
    start = text.index("uint32_t %s(uint32_t x) {" % name)
    return text[start:text.index("}", start)]


def multipliers(name):
    return [int(h, 16) for h in re.findall(r"x \*= (0x[0-9A-Fa-f]+)u;", body(name))]


def unmix_np(x, m1, m2):
    x = x.astype(np.uint64)
    x ^= x >> np.uint64(16)
    x = (x * np.uint64(m1)) & M32
    x ^= (x >> np.uint64(15)) ^ (x >> np.uint64(30))
    x = (x * np.uint64(m2)) & M32
    x ^= x >> np.uint64(16)
    return x.astype(np.uint32)


def test_multipliers_are_inverse_pairs():
    fwd, inv = multipliers("mix32"), multipliers("unmix32")
    assert len(fwd) == 2 and len(inv) == 2
    # the inverse undoes the steps in reverse order: its first multiplier undoes the mixer's last
    assert (fwd[1] * inv[0]) % (1 << 32) == 1
    assert (fwd[0] * inv[1]) % (1 << 32) == 1
    assert "(x >> 15) ^ (x >> 30)" in body("unmix32")   # x ^= x >> 15 is undone by two terms; x ^= x >> 16 by itself


def test_inverse_of_the_oracle_mixer():
    inv = multipliers("unmix32")
    rng = np.random.default_rng(7)
    xs = np.concatenate([np.array([0, 1, 2, 0x7FFFFFFF, 0x80000000, 0xFFFFFFFF, 0xFFFF0000, 0x0000FFFF], dtype=np.uint32),
                         rng.integers(0, 1 << 32, size=20000, dtype=np.uint64).astype(np.uint32)])
    mixed = np.array([R.mix32(int(x)) for x in xs], dtype=np.uint32)
    assert np.array_equal(unmix_np(mixed, *inv), xs)
    # and the other way round: mix(unmix(u)) = u for the small u that the listing kernel walks through
    us = np.arange(0, 5000, dtype=np.uint32)
    back = np.array([R.mix32(int(t)) for t in unmix_np(us, *inv)], dtype=np.uint32)
    assert np.array_equal(back, us)
