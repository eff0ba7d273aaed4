"""Philox4x32-10 counter-based random number generator (oracle side).

TEST INFRASTRUCTURE ONLY: nothing under oracle/ is part of the product path.

Follows the published Philox construction (Salmon, Moraes, Dror, Shaw,
"Parallel random numbers: as easy as 1, 2, 3", SC'11): a 4x32-bit counter
is run through 10 rounds; each round multiplies two of the counter words
by fixed odd constants, splits the 64-bit products in high and low halves,
xors the high halves with the other two counter words and the round key,
and the key is bumped by two Weyl constants between rounds.

The rollout sampler draws one uniform per (request id, generated-token
index): key = (seed lo, seed hi), counter = (request id lo, request id hi,
generated-token index, 0); the first output word w gives
u = (w >> 8) * 2**-24 in [0, 1).

Pinned by tests/test_oracle_philox.py against the generator's published
known-answer vectors (tests/golden/philox4x32_10_kat.txt).
"""

M0 = 0xD2511F53
M1 = 0xCD9E8D57
W0 = 0x9E3779B9  # golden ratio
W1 = 0xBB67AE85  # sqrt(3) - 1
MASK = 0xFFFFFFFF


def philox4x32_10(counter, key):
    """counter: 4 ints (32-bit words), key: 2 ints -> tuple of 4 32-bit words."""
    c0, c1, c2, c3 = (int(c) & MASK for c in counter)
    k0, k1 = (int(k) & MASK for k in key)
    for _ in range(10):
        p0 = M0 * c0
        p1 = M1 * c2
        hi0, lo0 = p0 >> 32, p0 & MASK
        hi1, lo1 = p1 >> 32, p1 & MASK
        c0, c1, c2, c3 = (hi1 ^ c1 ^ k0) & MASK, lo1, (hi0 ^ c3 ^ k1) & MASK, lo0
        k0 = (k0 + W0) & MASK
        k1 = (k1 + W1) & MASK
    return (c0, c1, c2, c3)


def uniform_for(seed, request_id, gen_index):
    """The uniform in [0,1) used to sample generated token `gen_index` of a request."""
    seed = int(seed) & 0xFFFFFFFFFFFFFFFF
    rid = int(request_id) & 0xFFFFFFFFFFFFFFFF
    w = philox4x32_10((rid & MASK, rid >> 32, int(gen_index) & MASK, 0),
                      (seed & MASK, seed >> 32))
    return (w[0] >> 8) * (2.0 ** -24)
