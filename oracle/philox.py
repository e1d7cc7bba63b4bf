"""Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11), scalar Python integers.

Test infrastructure only -- see the package docstring.

The paper only says "random" for its communicator shuffles (Sec. 4.5.1) and
for nothing else; this build fixes the generator so that both sides of every
parity test can draw the same numbers from a (key, counter) pair.

One block maps a 128-bit counter (c0,c1,c2,c3) and a 64-bit key (k0,k1) to four
32-bit words through ten rounds.  One round:
    (hi0, lo0) = M0 * c0          (64-bit product split into halves)
    (hi1, lo1) = M1 * c2
    (c0,c1,c2,c3) <- (hi1 ^ c1 ^ k0,  lo1,  hi0 ^ c3 ^ k1,  lo0)
and between rounds the key advances by the Weyl constants (k0 += W0, k1 += W1).
Literal output words: parity unpinned (structural pins only).
"""

M0 = 0xD2511F53
M1 = 0xCD9E8D57
W0 = 0x9E3779B9  # floor(2^32 * (sqrt(5)-1)/2)
W1 = 0xBB67AE85  # floor(2^32 * (sqrt(3)-1))
MASK = 0xFFFFFFFF
ROUNDS = 10

TAG_COMM = 1   # stream that draws the shuffled communicators
TAG_SHUF = 2   # stream that flags sample slots for the partner-swap shuffle


def philox_round(c, k):
    p0 = M0 * c[0]
    p1 = M1 * c[2]
    hi0, lo0 = p0 >> 32, p0 & MASK
    hi1, lo1 = p1 >> 32, p1 & MASK
    return (hi1 ^ c[1] ^ k[0], lo1, hi0 ^ c[3] ^ k[1], lo0)


def philox4x32(counter, key, rounds=ROUNDS):
    """Return the 4 output words for `counter` (4 words) under `key` (2 words)."""
    c = tuple(int(x) & MASK for x in counter)
    k = (int(key[0]) & MASK, int(key[1]) & MASK)
    for r in range(rounds):
        if r:
            k = ((k[0] + W0) & MASK, (k[1] + W1) & MASK)
        c = philox_round(c, k)
    return c


def seed_key(seed):
    """64-bit seed -> (low word, high word)."""
    seed = int(seed) & 0xFFFFFFFFFFFFFFFF
    return (seed & MASK, seed >> 32)


class WordStream:
    """Successive 32-bit words: block n = philox(counter=(n, c1, c2, c3)), words
    0..3 of block 0, then of block 1, ..."""

    def __init__(self, seed, c1, c2, c3):
        self.key = seed_key(seed)
        self.tail = (c1, c2, c3)
        self.n = 0
        self.buf = []

    def next32(self):
        if not self.buf:
            self.buf = list(philox4x32((self.n,) + self.tail, self.key))
            self.n += 1
        return self.buf.pop(0)


def philox4x32_np(c0, c1, c2, c3, key, rounds=ROUNDS):
    """The same block function on numpy arrays of counters (written separately
    from the scalar form above, in 64-bit lanes; the tests require the two to
    agree word for word).  Returns four uint32 arrays."""
    import numpy as np
    m32 = np.uint64(MASK)
    s32 = np.uint64(32)
    x0, x1, x2, x3 = (np.asarray(a).astype(np.uint64) & m32
                      for a in np.broadcast_arrays(c0, c1, c2, c3))
    k0, k1 = int(key[0]) & MASK, int(key[1]) & MASK
    for r in range(rounds):
        a = np.uint64(M0) * x0
        b = np.uint64(M1) * x2
        y0 = (b >> s32) ^ x1 ^ np.uint64(k0)
        y2 = (a >> s32) ^ x3 ^ np.uint64(k1)
        x0, x1, x2, x3 = y0, b & m32, y2, a & m32
        k0 = (k0 + W0) & MASK
        k1 = (k1 + W1) & MASK
    return tuple(x.astype(np.uint32) for x in (x0, x1, x2, x3))
