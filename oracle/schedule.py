"""Partner selection and partner rotation (Sec. 4.3, 4.4.1, 4.4.2, 4.5.1).

Test infrastructure only -- see the package docstring.

Notation: p ranks, L = ceil(log2 p) phases, step counter t = 0,1,...,
phase k = t mod L (ascending), rotation index r = (t div L) mod R.
A communicator sigma_r maps a virtual rank v to a world rank; the virtual
topology of the current L steps is laid over sigma_r (Sec. 4.5.1: p random
shuffles of the original communicator, fixed at start-up, the next one taken
after every log p steps).  sigma_0 is the original communicator (identity).
"""

from .philox import WordStream, TAG_COMM

HYPERCUBE = 0
DISSEMINATION = 1


def num_phases(p):
    """L = ceil(log2 p)."""
    L = 0
    while (1 << L) < p:
        L += 1
    return L


def is_pow2(p):
    return p >= 1 and (p & (p - 1)) == 0


def communicator(p, seed, r):
    """sigma_r as a list: virtual rank -> world rank.

    r = 0 is the identity.  r >= 1 is a Fisher-Yates shuffle of the identity
    driven by the word stream with counter tail (r, 0, TAG_COMM):
        for i = p-1 down to 1:  q = floor(u * (i+1) / 2^32),  swap a[i], a[q]
    """
    a = list(range(p))
    if r == 0:
        return a
    ws = WordStream(seed, r, 0, TAG_COMM)
    for i in range(p - 1, 0, -1):
        u = ws.next32()
        q = (u * (i + 1)) >> 32
        a[i], a[q] = a[q], a[i]
    return a


def inverse(sigma):
    inv = [0] * len(sigma)
    for v, j in enumerate(sigma):
        inv[j] = v
    return inv


def phase_and_rotation(p, num_comms, t):
    L = num_phases(p)
    return t % L, (t // L) % num_comms


def partners(p, seed, num_comms, topology, t):
    """(send_to, recv_from): two length-p lists for step t.

    Hypercube (Sec. 4.3, 4.4.1): rank j talks to the rank whose virtual id
    differs in bit k; send_to == recv_from and the map is an involution.
    Dissemination (Sec. 4.4.2): virtual rank i sends to (i + 2^k) mod p and
    receives from (i + p - 2^k) mod p.
    """
    if p < 2:
        raise ValueError("p must be >= 2")
    if num_comms < 1:
        raise ValueError("num_comms must be >= 1")
    if topology == HYPERCUBE and not is_pow2(p):
        raise ValueError("hypercube needs a power-of-two p")
    k, r = phase_and_rotation(p, num_comms, t)
    sigma = communicator(p, seed, r)
    inv = inverse(sigma)
    send = [0] * p
    recv = [0] * p
    for j in range(p):
        v = inv[j]
        if topology == HYPERCUBE:
            send[j] = sigma[v ^ (1 << k)]
            recv[j] = send[j]
        elif topology == DISSEMINATION:
            send[j] = sigma[(v + (1 << k)) % p]
            recv[j] = sigma[(v + p - (1 << k)) % p]
        else:
            raise ValueError("unknown topology")
    return send, recv
