"""Pins for the oracle's Philox4x32-10 and its uniform mapping."""
import os

import numpy as np

from oracle import philox

GOLD = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def test_known_answer_vectors():
    rows = [l.split() for l in open(GOLD) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        w = [int(x, 16) for x in r]
        assert philox.philox4x32_10(w[0:4], w[4:6]) == w[6:10]


def test_single_round_structure_by_hand():
    """One round on a hand-checkable input: ctr=(1,0,0,0), key=(0,0): products are the multipliers."""
    # emulate one round only by the definition: c0' = hi(M1*c2)^c1^k0, c1' = lo(M1*c2), c2' = hi(M0*c0)^c3^k1, c3' = lo(M0*c0)
    c = [1, 0, 0, 0]
    exp = [0, 0, 0, 0xD2511F53]
    p0 = philox.MUL0 * c[0]
    p1 = philox.MUL1 * c[2]
    got = [(p1 >> 32) ^ c[1], p1 & philox.M32, (p0 >> 32) ^ c[3], p0 & philox.M32]
    assert got == exp
    # and the 10-round function differs for neighbouring counters and keys (avalanche)
    a = philox.philox4x32_10([1, 0, 0, 0], [0, 0])
    b = philox.philox4x32_10([2, 0, 0, 0], [0, 0])
    c2 = philox.philox4x32_10([1, 0, 0, 0], [1, 0])
    bits = lambda x, y: sum(bin(p ^ q).count("1") for p, q in zip(x, y))
    assert 40 < bits(a, b) < 90 and 40 < bits(a, c2) < 90


def test_uniform_range_and_moments():
    u = np.array([philox.uniform_for_token(0x1234567890ABCDEF, i) for i in range(20000)])
    assert u.min() >= 0.0 and u.max() < 1.0
    assert abs(u.mean() - 0.5) < 0.01 and abs(u.var() - 1 / 12) < 0.005
    hist, _ = np.histogram(u, bins=16, range=(0, 1))
    chi2 = ((hist - 1250.0) ** 2 / 1250.0).sum()
    assert chi2 < 45.0  # 15 dof, p ~ 1e-4
    # 24-bit grid, seed halves map to key words
    assert all(float(x * 2 ** 24).is_integer() for x in u[:100])
    x = philox.philox4x32_10([7, 0, 0, 0], [0x90ABCDEF, 0x12345678])
    assert philox.uniform_for_token(0x1234567890ABCDEF, 7) == (x[0] >> 8) / 2 ** 24
