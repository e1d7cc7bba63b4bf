"""Pins for the oracle's momentum-SGD update, pairwise averaging, staleness-1
variant and recursive-doubling all-reduce (Eq. 1-2, Sec. 3.1, Sec. 6)."""
import numpy as np
import pytest
import torch

from golden_io import load
from oracle import gossip as og
from oracle import schedule as sc


def _state(p, n, seed=0, dtype=np.float32):
    rng = np.random.default_rng(seed)
    W = rng.normal(0, 0.05, (p, n)).astype(dtype)
    G = rng.normal(0, 1e-3, (p, n)).astype(dtype)
    M = rng.normal(0, 1e-3, (p, n)).astype(dtype)
    return W, G, M


# ---------------------------------------------------------------- momentum SGD
@pytest.mark.parametrize("dtype,tol", [(np.float64, 1e-15), (np.float32, 1e-6)])
def test_momentum_three_steps_hand_values(dtype, tol):
    g = load("momentum_3step.txt")
    W = np.array([g["w0"]], dtype=dtype)
    G = np.array([g["g"]], dtype=dtype)
    M = np.zeros_like(W)
    for _ in range(3):
        og.sgd_step(W, G, M, g["lr"], g["mu"])
    np.testing.assert_allclose(W[0], g["w3"], rtol=tol, atol=tol)
    np.testing.assert_allclose(M[0], g["m3"], rtol=tol, atol=tol)


def test_momentum_matches_library_optimizer_and_geometric_series():
    # constant lr: v<-mu*v+lr*g, w<-w-v equals the library's v<-mu*v+g, w<-w-lr*v
    rng = np.random.default_rng(3)
    w0 = rng.normal(size=64)
    grads = rng.normal(size=(5, 64))
    lr, mu = 0.1, 0.9
    W = w0[None].copy(); M = np.zeros_like(W)
    tw = torch.tensor(w0.copy(), requires_grad=True)
    opt = torch.optim.SGD([tw], lr=lr, momentum=mu)
    for s in range(5):
        og.sgd_step(W, grads[s][None].copy(), M, lr, mu)
        tw.grad = torch.tensor(grads[s].copy())
        opt.step()
    np.testing.assert_allclose(W[0], tw.detach().numpy(), rtol=1e-12, atol=1e-14)
    # geometric series for a constant gradient
    W = w0[None].copy(); M = np.zeros_like(W); G = grads[0][None].copy()
    for _ in range(7):
        og.sgd_step(W, G, M, lr, mu)
    np.testing.assert_allclose(M[0], lr * grads[0] * (1 - mu**7) / (1 - mu), rtol=1e-12)
    tot = sum(lr * (1 - mu**t) / (1 - mu) for t in range(1, 8))
    np.testing.assert_allclose(W[0], w0 - tot * grads[0], rtol=1e-12, atol=1e-14)


def test_zero_momentum_is_plain_descent_and_sign_is_descent():
    W, G, M = _state(2, 100, 1, np.float64)
    w0 = W.copy()
    og.sgd_step(W, G, M, 0.1, 0.0)
    np.testing.assert_allclose(W, w0 - 0.1 * G, rtol=0, atol=1e-18)
    # one small step along -g lowers the quadratic cost C = |w|^2/2 whose gradient is w
    w = np.array([[1.0, -2.0, 3.0]]); g = w.copy(); m = np.zeros_like(w)
    og.sgd_step(w, g, m, 0.1, 0.9)
    assert (np.abs(w) < np.abs(g)).all()


def test_avg_none_equals_sgd_step_and_leaves_g():
    W, G, M = _state(4, 50, 2)
    W2, G2, M2 = W.copy(), G.copy(), M.copy()
    og.gossip_step(W, G, M, [1, 0, 3, 2], 0.1, 0.9, avg_mode=og.AVG_NONE)
    og.sgd_step(W2, G2, M2, 0.1, 0.9)
    assert np.array_equal(W, W2) and np.array_equal(M, M2) and np.array_equal(G, G2)


def test_fp32_ops_are_individually_rounded():
    # element-by-element recomputation with explicit float32 scalars, no fusion
    W, G, M = _state(2, 200, 4)
    W0, G0, M0 = W.copy(), G.copy(), M.copy()
    og.gossip_step(W, G, M, [1, 0], 0.1, 0.9)
    f = np.float32
    for i in range(200):
        T = []
        for j in range(2):
            a = f(f(0.9) * M0[j, i]); b = f(f(0.1) * G0[j, i]); v = f(a + b)
            assert M[j, i] == v
            T.append(f(W0[j, i] - v))
        e = f(f(0.5) * f(T[0] + T[1]))
        assert W[0, i] == e and W[1, i] == e
    assert W.dtype == np.float32 and M.dtype == np.float32


# ---------------------------------------------------------- pairwise averaging
def test_gossip_hand_example_p4():
    g = load("gossip_p4_hand.txt")
    for dtype in (np.float32, np.float64):
        W = np.array(g["w0"], dtype=dtype)[:, None].copy()
        G = np.array(g["g"], dtype=dtype)[:, None].copy()
        M = np.zeros_like(W)
        c0, _ = sc.partners(4, 0, 1, sc.HYPERCUBE, 0)
        c1, _ = sc.partners(4, 0, 1, sc.HYPERCUBE, 1)
        og.gossip_step(W, G, M, c0, g["lr"], g["mu"])
        assert W[:, 0].tolist() == g["w1"]
        og.gossip_step(W, G, M, c1, g["lr"], g["mu"])
        assert W[:, 0].tolist() == g["w2"]
        # staleness-1 and gradient-averaging variants of the first step
        W = np.array(g["w0"], dtype=dtype)[:, None].copy(); M = np.zeros_like(W)
        og.gossip_step(W, G, M, c0, g["lr"], g["mu"], W_stale=W.copy())
        assert W[:, 0].tolist() == g["w1_stale"]
        W = np.array(g["w0"], dtype=dtype)[:, None].copy(); M = np.zeros_like(W)
        og.gossip_step(W, G, M, c0, g["lr"], g["mu"], avg_mode=og.AVG_GRAD)
        assert W[:, 0].tolist() == g["w1_gradavg"]
        assert G[:, 0].tolist() == g["g"]                      # G is not written
        og.allreduce_recursive_doubling(G, average=True)
        assert G[:, 0].tolist() == g["g_allreduce_avg"]


@pytest.mark.parametrize("p", [2, 4, 8, 16])
def test_average_preserves_cross_rank_sum_and_partners_agree_bitwise(p):
    W, G, M = _state(p, 257, 5)
    L = sc.num_phases(p)
    for t in range(3 * L):
        c, _ = sc.partners(p, 1, p, sc.HYPERCUBE, t)
        T, _ = og.local_update(W, G, M, 0.1, 0.9)
        tsum = T.astype(np.float64).sum(axis=0)
        og.gossip_step(W, G, M, c, 0.1, 0.9)
        wsum = W.astype(np.float64).sum(axis=0)
        bound = p * 2.0**-23 * np.abs(T).max()
        assert np.abs(wsum - tsum).max() <= bound
        for j in range(p):
            assert np.array_equal(W[j], W[c[j]])
    # exact in float64 up to rounding
    W, G, M = _state(p, 64, 6, np.float64)
    T, _ = og.local_update(W, G, M, 0.1, 0.9)
    c, _ = sc.partners(p, 1, p, sc.HYPERCUBE, 0)
    og.gossip_step(W, G, M, c, 0.1, 0.9)
    np.testing.assert_allclose(W.sum(axis=0), T.sum(axis=0), rtol=0, atol=1e-15)


def test_p2_step_is_the_plain_two_vector_mean():
    W, G, M = _state(2, 100, 7, np.float64)
    T, V = og.local_update(W, G, M, 0.1, 0.9)
    og.gossip_step(W, G, M, [1, 0], 0.1, 0.9)
    np.testing.assert_allclose(W[0], T.mean(axis=0), rtol=0, atol=1e-17)
    np.testing.assert_allclose(W[1], T.mean(axis=0), rtol=0, atol=1e-17)
    assert np.array_equal(M, V)                               # momentum stays local


@pytest.mark.parametrize("p", [2, 4, 8, 16, 32])
@pytest.mark.parametrize("topo", [sc.HYPERCUBE, sc.DISSEMINATION])
def test_log_p_averaging_steps_reach_the_global_mean(p, topo):
    # lr = 0: L aligned steps leave every rank at the mean of the initial weights
    L = sc.num_phases(p)
    for block in (0, 2):                                      # block 2 uses a shuffled communicator
        W, G, M = _state(p, 300, 8 + block)
        M[...] = 0
        mean64 = W.astype(np.float64).mean(axis=0)
        for t in range(block * L, (block + 1) * L):
            send, recv = sc.partners(p, 4, p, topo, t)
            og.gossip_step(W, G, M, recv, 0.0, 0.9)
        for j in range(p):
            assert np.abs(W[j] - mean64).max() <= L * 2.0**-24 * np.abs(mean64).max() + 1e-9
        if topo == sc.HYPERCUBE:
            for j in range(1, p):
                assert np.array_equal(W[0], W[j])             # the same pairwise tree everywhere


def test_identical_ranks_track_single_rank_sgd_and_allreduce_sgd_bitwise():
    p, n = 8, 500
    W1, G1, M1 = _state(1, n, 9)
    Wg, Gg, Mg = (np.repeat(a, p, axis=0) for a in (W1, G1, M1))
    Wa, Ga, Ma = Wg.copy(), Gg.copy(), Mg.copy()
    for t in range(6):
        c, _ = sc.partners(p, 0, p, sc.HYPERCUBE, t)
        og.gossip_step(Wg, Gg, Mg, c, 0.1, 0.9)
        Ga[...] = Gg
        og.allreduce_sgd_step(Wa, Ga, Ma, 0.1, 0.9)
        og.sgd_step(W1, G1, M1, 0.1, 0.9)
        for j in range(p):
            assert np.array_equal(Wg[j], W1[0]) and np.array_equal(Wa[j], W1[0])
            assert np.array_equal(Mg[j], M1[0]) and np.array_equal(Ma[j], M1[0])


def test_permutation_not_involution_uses_the_given_partner():
    # dissemination data path: rank j averages with recv[j] (a 3-cycle here)
    W = np.array([[1.0], [10.0], [100.0]]); G = np.zeros_like(W); M = np.zeros_like(W)
    og.gossip_step(W, G, M, [2, 0, 1], 0.1, 0.9)
    assert W[:, 0].tolist() == [50.5, 5.5, 55.0]


# ------------------------------------------------------------------ staleness 1
def test_staleness_sum_closed_form_and_reduction_to_sync():
    p, n = 8, 128
    W, G, M = _state(p, n, 10, np.float64)
    W_old = W.copy()
    _, V = og.local_update(W, G, M, 0.1, 0.9)
    c, _ = sc.partners(p, 0, p, sc.HYPERCUBE, 1)
    og.gossip_step(W, G, M, c, 0.1, 0.9, W_stale=W_old)
    np.testing.assert_allclose(W.sum(axis=0), W_old.sum(axis=0) - 0.5 * V.sum(axis=0), rtol=0, atol=1e-15)
    # zero velocity on the partner side -> stale == sync
    W, G, M = _state(p, n, 11)
    G[...] = 0; M[...] = 0
    Ws, Gs, Ms = W.copy(), G.copy(), M.copy()
    og.gossip_step(W, G, M, c, 0.1, 0.9, W_stale=W.copy())
    og.gossip_step(Ws, Gs, Ms, c, 0.1, 0.9)
    assert np.array_equal(W, Ws)


def test_grad_averaging_p2_equals_allreduce_sgd_bitwise():
    W, G, M = _state(2, 300, 12)
    W[1] = W[0]; M[1] = M[0]
    Wa, Ga, Ma = W.copy(), G.copy(), M.copy()
    og.gossip_step(W, G, M, [1, 0], 0.1, 0.9, avg_mode=og.AVG_GRAD)
    og.allreduce_sgd_step(Wa, Ga, Ma, 0.1, 0.9)
    assert np.array_equal(W, Wa) and np.array_equal(M, Ma)


# ------------------------------------------------------------------- all-reduce
@pytest.mark.parametrize("p", [2, 4, 8, 16, 64])
def test_allreduce_all_ranks_identical_and_close_to_float64_sum(p):
    _, G, _ = _state(p, 333, 13)
    G0 = G.copy()
    og.allreduce_recursive_doubling(G, average=False)
    for j in range(1, p):
        assert np.array_equal(G[0], G[j])
    L = sc.num_phases(p)
    s64 = G0.astype(np.float64).sum(axis=0)
    assert (np.abs(G[0] - s64) <= L * 2.0**-24 * np.abs(G0).astype(np.float64).sum(axis=0) + 1e-30).all()
    # the fixed balanced pairwise tree, written out recursively
    def tree(lo, hi):
        if hi - lo == 1:
            return G0[lo]
        mid = (lo + hi) // 2
        return tree(lo, mid) + tree(mid, hi)
    assert np.array_equal(G[0], tree(0, p))


@pytest.mark.parametrize("p", [2, 8, 32])
def test_allreduce_average_equals_log_p_hypercube_averaging_steps(p):
    # halving at every level == one exact scaling by 1/p at the end, absent underflow
    _, G, _ = _state(p, 200, 14)
    A = G.copy()
    og.allreduce_recursive_doubling(A, average=True)
    Wv = G.copy(); Z = np.zeros_like(G); M = np.zeros_like(G)
    for t in range(sc.num_phases(p)):
        c, _ = sc.partners(p, 0, 1, sc.HYPERCUBE, t)
        og.gossip_step(Wv, Z, M, c, 0.0, 0.0)
    assert np.array_equal(A, Wv)
    bound = sc.num_phases(p) * 2.0**-24 * np.abs(G).astype(np.float64).mean(axis=0)
    assert (np.abs(A[0] - G.astype(np.float64).mean(axis=0)) <= bound + 1e-30).all()


def test_allreduce_rejects_non_power_of_two():
    with pytest.raises(ValueError):
        og.allreduce_recursive_doubling(np.zeros((3, 4), np.float32))
    with pytest.raises(ValueError):
        og.allreduce_recursive_doubling(np.zeros((1, 4), np.float32))


def test_fp32_oracle_tracks_float64_oracle():
    p, n = 8, 2000
    W, G, M = _state(p, n, 15)
    M[...] = 0
    W64, G64, M64 = (a.astype(np.float64) for a in (W, G, M))
    for t in range(9):
        c, _ = sc.partners(p, 0, p, sc.HYPERCUBE, t)
        og.gossip_step(W, G, M, c, 0.1, 0.9)
        og.gossip_step(W64, G64, M64, c, np.float32(0.1), np.float32(0.9))
    scale = np.abs(W64).max()
    assert np.abs(W - W64).max() <= 9 * 4 * 2.0**-24 * scale


def test_allreduce_every_log_p_block_is_local_steps_then_model_mean():
    # Sec. 7.5: O(1) amortised communication by combining the models every log p steps
    p, n = 8, 200
    W, G, M = _state(p, n, 16, np.float64)
    W0, M0 = W.copy(), M.copy()
    og.allreduce_every_log_p_block(W, G, M, 0.1, 0.9)
    # closed form per rank after 3 local steps with constant g: w3 = w0 - sum_t v_t, v_t = mu^t m0 + lr g (1-mu^t)/(1-mu)
    vs = [0.9**t * M0 + 0.1 * G * (1 - 0.9**t) / (1 - 0.9) for t in (1, 2, 3)]
    local = W0 - sum(vs)
    np.testing.assert_allclose(M, vs[-1], rtol=1e-12, atol=1e-18)
    for j in range(p):
        np.testing.assert_allclose(W[j], local.mean(axis=0), rtol=1e-12, atol=1e-16)
    # identical ranks: the block equals three plain SGD steps bit for bit
    W1, G1, M1 = _state(1, n, 17)
    Wp, Gp, Mp = (np.repeat(a, p, axis=0) for a in (W1, G1, M1))
    og.allreduce_every_log_p_block(Wp, Gp, Mp, 0.1, 0.9)
    for _ in range(3):
        og.sgd_step(W1, G1, M1, 0.1, 0.9)
    assert all(np.array_equal(Wp[j], W1[0]) for j in range(p))
