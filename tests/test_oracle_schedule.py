"""Pins for partner selection and rotation (Sec. 4.3, 4.4, 4.5.1)."""
import itertools

import pytest

from oracle import schedule as sc

POW2 = [2, 4, 8, 16, 32, 64, 128]


def _is_perm(a):
    return sorted(a) == list(range(len(a)))


@pytest.mark.parametrize("p", POW2)
def test_hypercube_is_fixed_point_free_involution_every_step(p):
    L = sc.num_phases(p)
    for t in range(min(p, 16) * L + 3):
        send, recv = sc.partners(p, 7, p, sc.HYPERCUBE, t)
        assert send == recv
        assert _is_perm(send)
        for j in range(p):
            assert send[j] != j                 # no self-pairs
            assert send[send[j]] == j           # balanced: unique pairs (Sec. 4.3)


@pytest.mark.parametrize("p", POW2)
def test_hypercube_identity_communicator_is_textbook_xor(p):
    L = sc.num_phases(p)
    assert 1 << L == p
    for t in range(3 * L):
        send, _ = sc.partners(p, 0, 1, sc.HYPERCUBE, t)
        assert send == [j ^ (1 << (t % L)) for j in range(p)]
    # first L steps use the original communicator even with rotation on
    for t in range(L):
        send, _ = sc.partners(p, 99, p, sc.HYPERCUBE, t)
        assert send == [j ^ (1 << t) for j in range(p)]


@pytest.mark.parametrize("p", [4, 16, 64])
def test_hypercube_is_conjugation_by_the_communicator(p):
    L = sc.num_phases(p)
    for r in range(1, min(5, p)):
        sigma = sc.communicator(p, 3, r)
        inv = sc.inverse(sigma)
        for k in range(L):
            send, _ = sc.partners(p, 3, p, sc.HYPERCUBE, r * L + k)
            assert send == [sigma[inv[j] ^ (1 << k)] for j in range(p)]
            # virtual ranks that differ in bit k are partners in world ranks
            for v in range(p):
                assert send[sigma[v]] == sigma[v ^ (1 << k)]


def _reach_after_block(p, seed, R, topo, t0):
    """Brute force: bitmask of ranks whose contribution reached j after L steps."""
    L = sc.num_phases(p)
    reach = [1 << j for j in range(p)]
    for t in range(t0, t0 + L):
        send, recv = sc.partners(p, seed, R, topo, t)
        reach = [reach[j] | reach[recv[j]] for j in range(p)]
    return reach


@pytest.mark.parametrize("p", POW2)
def test_hypercube_full_indirect_diffusion_every_log_p_steps(p):
    L = sc.num_phases(p)
    full = (1 << p) - 1
    for blk in range(6):
        assert _reach_after_block(p, 11, p, sc.HYPERCUBE, blk * L) == [full] * p
    # ... and not one step earlier
    if L > 1:
        reach = [1 << j for j in range(p)]
        for t in range(L - 1):
            send, _ = sc.partners(p, 11, p, sc.HYPERCUBE, t)
            reach = [reach[j] | reach[send[j]] for j in range(p)]
        assert all(bin(x).count("1") == p // 2 for x in reach)


@pytest.mark.parametrize("p", [2, 3, 5, 6, 8, 12, 16, 33, 64, 100, 128])
def test_dissemination_full_indirect_diffusion_and_permutations(p):
    L = sc.num_phases(p)
    assert (1 << L) >= p > (1 << (L - 1)) or p == 2
    full = (1 << p) - 1
    for blk in range(4):
        assert _reach_after_block(p, 5, p, sc.DISSEMINATION, blk * L) == [full] * p
    for t in range(3 * L):
        send, recv = sc.partners(p, 5, p, sc.DISSEMINATION, t)
        assert _is_perm(send) and _is_perm(recv)
        for j in range(p):
            assert send[j] != j and recv[j] != j
            assert recv[send[j]] == j and send[recv[j]] == j   # mutually inverse


@pytest.mark.parametrize("p", [2, 5, 8, 16, 100])
def test_dissemination_identity_communicator_is_the_papers_formula(p):
    L = sc.num_phases(p)
    for t in range(2 * L):
        k = t % L
        send, recv = sc.partners(p, 0, 1, sc.DISSEMINATION, t)
        assert send == [(i + 2**k) % p for i in range(p)]
        assert recv == [(i + p - 2**k) % p for i in range(p)]


@pytest.mark.parametrize("p", [4, 8, 32])
def test_without_rotation_partners_recur_with_period_log_p(p):
    L = sc.num_phases(p)
    for topo in (sc.HYPERCUBE, sc.DISSEMINATION):
        rows = [sc.partners(p, 1, 1, topo, t) for t in range(4 * L)]
        for t in range(3 * L):
            assert rows[t] == rows[t + L]
        # direct partners are a log(p)/p fraction: exactly L distinct send targets
        for j in range(p):
            assert len({rows[t][0][j] for t in range(4 * L)}) == L


@pytest.mark.parametrize("p", [4, 8, 32])
def test_rotation_changes_communicator_every_log_p_steps_and_wraps(p):
    L = sc.num_phases(p)
    R = p
    for t in range(R * L):
        assert sc.phase_and_rotation(p, R, t) == (t % L, t // L)
        assert sc.partners(p, 2, R, sc.HYPERCUBE, t) == sc.partners(p, 2, R, sc.HYPERCUBE, t + R * L)
    # with rotation a rank meets more direct partners than L over a full cycle
    met = {sc.partners(p, 2, R, sc.HYPERCUBE, t)[0][0] for t in range(R * L)}
    if p >= 8:
        assert len(met) > L
    # fewer communicators: num_comms = 2 alternates between sigma_0 and sigma_1
    a = sc.partners(p, 2, 2, sc.HYPERCUBE, 0)
    assert a == sc.partners(p, 2, 2, sc.HYPERCUBE, 2 * L)
    assert sc.partners(p, 2, 2, sc.HYPERCUBE, L) == sc.partners(p, 2, R, sc.HYPERCUBE, L)


@pytest.mark.parametrize("p", [2, 3, 16, 128, 1000])
def test_communicators_are_permutations_first_is_identity(p):
    assert sc.communicator(p, 42, 0) == list(range(p))
    seen = set()
    for r in range(1, min(p, 12)):
        s = sc.communicator(p, 42, r)
        assert _is_perm(s)
        inv = sc.inverse(s)
        assert all(inv[s[v]] == v for v in range(p))
        seen.add(tuple(s))
    if p >= 16:
        assert len(seen) == min(p, 12) - 1          # different shuffles
    assert sc.communicator(p, 42, 1) == sc.communicator(p, 42, 1)
    if p >= 16:
        assert sc.communicator(p, 42, 1) != sc.communicator(p, 43, 1)


def test_fisher_yates_is_unbiased_on_small_p():
    # all 24 orders of 4 ranks about equally often over many communicators
    counts = {perm: 0 for perm in itertools.permutations(range(4))}
    trials = 4800
    for r in range(1, trials + 1):
        counts[tuple(sc.communicator(4, 2024, r))] += 1
    expect = trials / 24
    chi2 = sum((c - expect) ** 2 / expect for c in counts.values())
    assert chi2 < 60.0        # 23 dof, p ~ 4e-5
    assert min(counts.values()) > 0


def test_fisher_yates_consumes_one_word_per_swap_in_order():
    # Re-derive sigma_1 for p = 5 from the raw word stream by hand-rolled steps.
    from oracle.philox import philox4x32, seed_key, TAG_COMM
    words = list(philox4x32((0, 1, 0, TAG_COMM), seed_key(9))) + list(philox4x32((1, 1, 0, TAG_COMM), seed_key(9)))
    a = [0, 1, 2, 3, 4]
    for n, i in enumerate([4, 3, 2, 1]):
        q = words[n] * (i + 1) // 2**32
        assert 0 <= q <= i
        a[i], a[q] = a[q], a[i]
    assert sc.communicator(5, 9, 1) == a


def test_argument_errors():
    with pytest.raises(ValueError):
        sc.partners(1, 0, 1, sc.HYPERCUBE, 0)
    with pytest.raises(ValueError):
        sc.partners(6, 0, 1, sc.HYPERCUBE, 0)
    with pytest.raises(ValueError):
        sc.partners(4, 0, 0, sc.HYPERCUBE, 0)
    sc.partners(6, 0, 1, sc.DISSEMINATION, 0)
