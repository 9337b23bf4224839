"""Philox4x32-10 counter-based generator (Salmon, Moraes, Dror, Shaw: "Parallel random
numbers: as easy as 1, 2, 3", SC'11), written with Python integers. Oracle code: test
infrastructure only.

The serving step draws one uniform per sampled token: key = (seed low 32 bits, seed high
32 bits), counter = (index of the output token being sampled, 0, 0, 0), and the uniform is
the top 24 bits of the first output word scaled by 2**-24, so u lies in [0, 1).
"""

M32 = 0xFFFFFFFF
MUL0 = 0xD2511F53
MUL1 = 0xCD9E8D57
WEYL0 = 0x9E3779B9
WEYL1 = 0xBB67AE85


def philox4x32_10(counter, key):
    """counter: 4 words, key: 2 words (each < 2**32) -> 4 output words."""
    c0, c1, c2, c3 = [int(x) & M32 for x in counter]
    k0, k1 = [int(x) & M32 for x in key]
    for rnd in range(10):
        if rnd > 0:
            k0 = (k0 + WEYL0) & M32
            k1 = (k1 + WEYL1) & M32
        p0 = MUL0 * c0
        p1 = MUL1 * c2
        hi0, lo0 = p0 >> 32, p0 & M32
        hi1, lo1 = p1 >> 32, p1 & M32
        c0, c1, c2, c3 = hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0
    return [c0, c1, c2, c3]


def uniform_for_token(seed, token_index):
    """The uniform in [0,1) used to sample output token number token_index of a request."""
    seed = int(seed) & 0xFFFFFFFFFFFFFFFF
    x = philox4x32_10([int(token_index) & M32, 0, 0, 0], [seed & M32, seed >> 32])
    return (x[0] >> 8) * (2.0 ** -24)
