"""Pins for the sample-index rotation (Sec. 4.5.2, Lemma 1) and its
partner-swap variant."""
import math
from collections import deque

import numpy as np
import pytest

from golden_io import load
from oracle import schedule as sc
from oracle import shuffle as sh


def test_block_offsets_imagenet_partition():
    off = sh.block_offsets(1_281_167, 128)
    sizes = np.diff(off)
    assert off[0] == 0 and off[-1] == 1_281_167
    assert (sizes[:15] == 10_010).all() and (sizes[15:] == 10_009).all()
    assert sh.block_offsets(10, 4) == [0, 3, 6, 8, 10]
    assert sh.initial_indices(5).tolist() == [0, 1, 2, 3, 4]
    assert sh.initial_indices(5).dtype == np.int32


# ------------------------------------------------------------------------ ring
def test_ring_hand_example():
    g = load("ring_p3_hand.txt")
    off = sh.block_offsets(12, 3)
    idx = sh.initial_indices(12)
    for t, key in enumerate(["idx1", "idx2", "idx3"]):
        sh.ring_step(idx, off, 2, t)
        assert idx.tolist() == [int(v) for v in g[key]]


@pytest.mark.parametrize("p,n,b", [(4, 32, 2), (3, 31, 3), (5, 23, 4), (2, 9, 1)])
def test_ring_matches_a_fifo_queue_model(p, n, b):
    """Independent model: one deque per rank; pop b from the front, push them on
    the back of the next rank's queue.  The circular-buffer oracle, read from
    its head, must hold the same queue; the batches used must agree."""
    off = sh.block_offsets(n, p)
    idx = sh.initial_indices(n)
    queues = [deque(range(off[j], off[j + 1])) for j in range(p)]
    for t in range(3 * (n // b) + 5):
        batches = [[q.popleft() for _ in range(b)] for q in queues]
        for j in range(p):
            assert sh.ring_current_batch(idx, off, b, t, j) == batches[j]
        for j in range(p):
            queues[(j + 1) % p].extend(batches[j])
        sh.ring_step(idx, off, b, t)
        for j in range(p):
            n_j = off[j + 1] - off[j]
            h = ((t + 1) * b) % n_j
            ring = [int(idx[off[j] + (h + r) % n_j]) for r in range(n_j)]
            assert ring == list(queues[j])
        assert sorted(idx.tolist()) == list(range(n))


def test_ring_sample_returns_only_after_every_other_rank_used_it():
    p, n, b = 4, 32, 2
    off = sh.block_offsets(n, p)
    idx = sh.initial_indices(n)
    visits = {s: [] for s in range(n)}            # sample -> ranks that used it, in time order
    steps = 3 * p * (n // p // b)
    for t in range(steps):
        for j in range(p):
            for s in sh.ring_current_batch(idx, off, b, t, j):
                visits[s].append(j)
        sh.ring_step(idx, off, b, t)
    for s, ranks in visits.items():
        assert len(ranks) >= 2 * p
        for a, nxt in zip(ranks, ranks[1:]):
            assert nxt == (a + 1) % p              # j, j+1, ..., cyclically
        for i in range(len(ranks) - p + 1):
            assert len(set(ranks[i:i + p])) == p   # never twice at one rank within a lap


def test_ring_rejects_batch_larger_than_a_rank():
    off = sh.block_offsets(10, 4)
    with pytest.raises(ValueError):
        sh.ring_step(sh.initial_indices(10), off, 3, 0)
    idx = sh.initial_indices(10)
    sh.ring_step(idx, off, 0, 0)
    assert idx.tolist() == list(range(10))


# ---------------------------------------------------------------- partner swap
def test_flag_rule_scalar_and_array_forms_agree():
    for (seed, t, j, n_j) in [(0, 0, 0, 257), (5, 3, 17, 1000), (2**40 + 3, 1000, 127, 63)]:
        a = sh.flagged_slots(seed, t, j, n_j)
        b = [i for i in range(n_j) if sh.slot_flagged(seed, t, j, i)]
        assert a == b and a == sorted(a)


def test_flag_fraction_is_one_eighth():
    tot = 0; cnt = 0
    for t in range(4):
        for j in range(8):
            cnt += len(sh.flagged_slots(1, t, j, 10_009)); tot += 10_009
    assert abs(cnt - tot / 8) < 5 * math.sqrt(tot * (1 / 8) * (7 / 8))
    # different steps / ranks flag different slots
    assert sh.flagged_slots(1, 0, 0, 2000) != sh.flagged_slots(1, 1, 0, 2000)
    assert sh.flagged_slots(1, 0, 0, 2000) != sh.flagged_slots(1, 0, 1, 2000)


@pytest.mark.parametrize("p,n", [(2, 100), (4, 1001), (8, 4099), (16, 777)])
def test_partner_swap_is_a_permutation_touching_only_flagged_slots_of_partners(p, n):
    off = sh.block_offsets(n, p)
    idx = sh.initial_indices(n)
    owner = np.repeat(np.arange(p), np.diff(off))
    for t in range(2 * sc.num_phases(p) + 1):
        c, _ = sc.partners(p, 3, p, sc.HYPERCUBE, t)
        before = idx.copy()
        sh.partner_swap_step(idx, off, c, 3, t)
        assert sorted(idx.tolist()) == list(range(n))          # still a permutation
        assert len(idx) == n                                   # per-rank counts fixed by layout
        changed = np.nonzero(before != idx)[0]
        for pos in changed:
            j = owner[pos]
            assert sh.slot_flagged(3, t, j, pos - off[j])      # only flagged slots move
            src = int(np.nonzero(before == idx[pos])[0][0])
            assert owner[src] == c[j]                          # and only between partners
        # brute-force recomputation, pair by pair, r-th flagged <-> r-th flagged
        expect = before.copy()
        for j in range(p):
            if j < c[j]:
                fj = [i for i in range(off[j + 1] - off[j]) if sh.slot_flagged(3, t, j, i)]
                fc = [i for i in range(off[c[j] + 1] - off[c[j]]) if sh.slot_flagged(3, t, c[j], i)]
                for a, b in zip(fj, fc):                       # zip stops at the shorter list
                    expect[off[j] + a] = before[off[c[j]] + b]
                    expect[off[c[j]] + b] = before[off[j] + a]
        assert np.array_equal(idx, expect)


def test_partner_swap_rejects_non_involution():
    off = sh.block_offsets(30, 3)
    with pytest.raises(ValueError):
        sh.partner_swap_step(sh.initial_indices(30), off, [1, 2, 0], 0, 0)
    with pytest.raises(ValueError):
        sh.partner_swap_step(sh.initial_indices(20), sh.block_offsets(20, 2), [0, 1], 0, 0)


def test_ring_payload_follows_the_indices():
    # a payload row tagged with its sample id must stay glued to that id
    p, n, b = 4, 37, 3
    off = sh.block_offsets(n, p)
    idx = sh.initial_indices(n)
    payload = np.stack([np.arange(n) * 10, np.arange(n) * 10 + 1, np.arange(n) * 10 + 2], axis=1).astype(np.int32)
    for t in range(25):
        sh.ring_step(idx, off, b, t)
        sh.ring_payload_step(payload, off, b, t)
        assert np.array_equal(payload[:, 0], idx * 10) and np.array_equal(payload[:, 2], idx * 10 + 2)
