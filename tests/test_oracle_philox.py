"""Pins for the oracle's counter-based generator.

The literal word stream has no published value available here ("parity
unpinned" for the literal words); what is pinned: the Weyl constants by their
closed forms, bijectivity of the round (an inverse round written here undoes
it), agreement of two separately written implementations, and uniformity.
"""
import math
import random

import numpy as np

from oracle import philox as ph


def test_weyl_constants_closed_form():
    # golden-ratio and sqrt(3)-1 fractions of 2^32, exact via integer square roots
    s5 = math.isqrt(5 << 64)          # floor(sqrt(5) * 2^32)
    assert ph.W0 == (s5 - (1 << 32)) >> 1
    s3 = math.isqrt(3 << 64)          # floor(sqrt(3) * 2^32)
    assert ph.W1 == s3 - (1 << 32)


def test_multipliers_are_odd_so_rounds_are_bijective():
    assert ph.M0 & 1 and ph.M1 & 1


def _inverse_round(c, k):
    # forward: (y0,y1,y2,y3) = (hi1^c1^k0, lo1, hi0^c3^k1, lo0) with
    # hi0:lo0 = M0*c0 and hi1:lo1 = M1*c2.  lo = M*c mod 2^32 is invertible.
    inv0 = pow(ph.M0, -1, 1 << 32)
    inv1 = pow(ph.M1, -1, 1 << 32)
    c0 = (c[3] * inv0) & ph.MASK
    c2 = (c[1] * inv1) & ph.MASK
    hi0 = (ph.M0 * c0) >> 32
    hi1 = (ph.M1 * c2) >> 32
    return (c0, c[0] ^ hi1 ^ k[0], c2, c[2] ^ hi0 ^ k[1])


def test_block_function_is_invertible():
    rnd = random.Random(1)
    for _ in range(200):
        ctr = tuple(rnd.getrandbits(32) for _ in range(4))
        key = (rnd.getrandbits(32), rnd.getrandbits(32))
        out = ph.philox4x32(ctr, key)
        keys = [key]
        for _ in range(ph.ROUNDS - 1):
            keys.append(((keys[-1][0] + ph.W0) & ph.MASK, (keys[-1][1] + ph.W1) & ph.MASK))
        c = out
        for k in reversed(keys):
            c = _inverse_round(c, k)
        assert c == ctr


def test_scalar_and_array_forms_agree():
    rnd = random.Random(2)
    ctrs = [[rnd.getrandbits(32) for _ in range(4)] for _ in range(500)]
    ctrs += [[0, 0, 0, 0], [ph.MASK] * 4, [1, 0, 0, 0], [0, 0, 0, 1]]
    for key in [(0, 0), (ph.MASK, ph.MASK), (rnd.getrandbits(32), rnd.getrandbits(32))]:
        a = np.array(ctrs, dtype=np.uint64)
        got = ph.philox4x32_np(a[:, 0], a[:, 1], a[:, 2], a[:, 3], key)
        for i, c in enumerate(ctrs):
            assert tuple(int(g[i]) for g in got) == ph.philox4x32(c, key)


def test_rounds_parameter_and_key_schedule():
    # 10 rounds == 1 round applied ten times with the key advanced in between
    ctr, key = (5, 6, 7, 8), (9, 10)
    c, k = ctr, key
    for r in range(10):
        c = ph.philox_round(c, k)
        k = ((k[0] + ph.W0) & ph.MASK, (k[1] + ph.W1) & ph.MASK)
    assert c == ph.philox4x32(ctr, key)
    assert ph.philox4x32(ctr, key, rounds=7) != c


def test_distinct_counters_and_keys_give_distinct_blocks():
    seen = set()
    for n in range(2000):
        seen.add(ph.philox4x32((n, 0, 0, ph.TAG_COMM), (0, 0)))
        seen.add(ph.philox4x32((n, 0, 0, ph.TAG_SHUF), (0, 0)))
        seen.add(ph.philox4x32((n, 0, 0, ph.TAG_COMM), (1, 0)))
    assert len(seen) == 6000


def test_uniformity_of_words_and_top_bits():
    n = 50000
    w = np.stack(ph.philox4x32_np(np.arange(n), 3, 7, ph.TAG_SHUF, ph.seed_key(0)), axis=1).reshape(-1)
    total = w.size
    # every bit position is set about half the time (5 sigma)
    for b in range(32):
        ones = int(((w >> np.uint32(b)) & np.uint32(1)).sum())
        assert abs(ones - total / 2) < 5 * math.sqrt(total / 4)
    # the top three bits (the shuffle's 1/8 rule) are uniform over 8 bins
    bins = np.bincount((w >> np.uint32(29)).astype(np.int64), minlength=8)
    chi2 = float(((bins - total / 8) ** 2 / (total / 8)).sum())
    assert chi2 < 30.0        # 7 dof, p ~ 1e-4
    # mean of u/2^32
    assert abs(w.astype(np.float64).mean() / 2**32 - 0.5) < 5 / math.sqrt(12 * total)


def test_word_stream_order():
    ws = ph.WordStream(12345678901234567, 4, 0, ph.TAG_COMM)
    key = ph.seed_key(12345678901234567)
    assert key == (12345678901234567 & ph.MASK, 12345678901234567 >> 32)
    expect = list(ph.philox4x32((0, 4, 0, ph.TAG_COMM), key)) + list(ph.philox4x32((1, 4, 0, ph.TAG_COMM), key))
    assert [ws.next32() for _ in range(8)] == expect
