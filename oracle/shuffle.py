"""Rotation of samples (Sec. 4.5.2, Lemma 1), on sample indices only.

Test infrastructure only -- see the package docstring.

`idx` is one int32 array holding every rank's resident sample ids; rank j owns
the slots off[j] .. off[j+1]-1 (block partition).

RING (the paper's rule): after a rank has used a batch it sends that batch to
its ring neighbour j+1; a sample comes back to a rank only after every other
rank has used it.  Each rank's slots are a full circular FIFO: at step t the
head is h_j = (t*b) mod n_j, the b slots from the head (wrapping) are the
batch just used, they leave for rank (j+1) mod p and the batch arriving from
rank (j-1) mod p takes their places in order (these are the back of the queue
once the head has moved on by b).

PARTNER_SWAP (the variant the workload list defines): at step t every rank
flags about 1/8 of its slots with a counter-based draw; the r-th flagged slot
of rank j (in increasing slot order) is swapped with the r-th flagged slot of
its partner c[j], for r below the smaller of the two counts; surplus flagged
slots stay put.  Only defined for involution schedules (hypercube).
"""

import numpy as np
from .philox import philox4x32, philox4x32_np, seed_key, TAG_SHUF


def block_offsets(n_total, p):
    """Rank j holds floor(n/p) + (j < n mod p) consecutive ids."""
    base, extra = divmod(n_total, p)
    off = [0]
    for j in range(p):
        off.append(off[-1] + base + (1 if j < extra else 0))
    return off


def initial_indices(n_total):
    return np.arange(n_total, dtype=np.int32)


def slot_flagged(seed, t, j, i):
    """Slot i of rank j at step t is flagged iff the top three bits of its
    32-bit draw are zero (probability exactly 1/8).  The draw is word (i mod 4)
    of the block with counter (i div 4, j, t, TAG_SHUF)."""
    words = philox4x32((i >> 2, j, t & 0xFFFFFFFF, TAG_SHUF), seed_key(seed))
    return (words[i & 3] >> 29) == 0


def flagged_slots(seed, t, j, n_j):
    """All flagged slots of rank j at step t, ascending.  Same rule as
    slot_flagged, evaluated for every slot at once with the array form of the
    generator (the tests require the two to agree)."""
    nblk = (n_j + 3) // 4
    words = philox4x32_np(np.arange(nblk), j, t & 0xFFFFFFFF, TAG_SHUF, seed_key(seed))
    draws = np.stack(words, axis=1).reshape(-1)[:n_j]   # slot i -> word i%4 of block i//4
    return [int(i) for i in np.nonzero((draws >> np.uint32(29)) == 0)[0]]


def partner_swap_step(idx, off, c, seed, t):
    """In place.  `c` must be an involution without fixed points."""
    p = len(off) - 1
    sel = [flagged_slots(seed, t, j, off[j + 1] - off[j]) for j in range(p)]
    for j in range(p):
        cj = c[j]
        if c[cj] != j or cj == j:
            raise ValueError("partner map is not a fixed-point-free involution")
        if j < cj:
            m = min(len(sel[j]), len(sel[cj]))
            for r in range(m):
                a = off[j] + sel[j][r]
                b = off[cj] + sel[cj][r]
                idx[a], idx[b] = idx[b], idx[a]


def ring_step(idx, off, batch, t):
    """In place.  Every rank moves `batch` ids to its ring successor."""
    p = len(off) - 1
    n = [off[j + 1] - off[j] for j in range(p)]
    if batch < 0 or batch > min(n):
        raise ValueError("batch must fit the smallest rank")
    old = idx.copy()
    for j in range(p):
        src = (j - 1) % p
        h_dst = (t * batch) % n[j]
        h_src = (t * batch) % n[src]
        for r in range(batch):
            idx[off[j] + (h_dst + r) % n[j]] = old[off[src] + (h_src + r) % n[src]]


def ring_current_batch(idx, off, batch, t, j):
    """The ids rank j uses at step t (the b slots from its head)."""
    n_j = off[j + 1] - off[j]
    h = (t * batch) % n_j
    return [int(idx[off[j] + (h + r) % n_j]) for r in range(batch)]


def ring_payload_step(payload, off, batch, t):
    """The ring step applied to the samples themselves: `payload` is [n_total][...],
    row s holds the sample resident in slot s.  Rows move exactly as the indices
    do under ring_step.  In place."""
    src = np.arange(payload.shape[0], dtype=np.int32)
    ring_step(src, off, batch, t)            # src[d] = slot whose content lands in slot d
    payload[...] = payload[src]
