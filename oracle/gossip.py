"""Momentum-SGD update, pairwise model averaging, all-reduce comparator.

Test infrastructure only -- see the package docstring.

W, G, M are [p][N] arrays (weights, gradients, momentum of the p ranks).  The
arithmetic type is the arrays' dtype: float32 is the precision of the paper's
runs (every single *, +, - rounded on its own, no fused multiply-add: numpy
evaluates one operation per call), float64 serves as the "truth" variant.
`c` is the step's partner list (rank j averages with rank c[j]).

Update rule (Eq. 1-2 read as descent, momentum in the convention of the
framework the paper builds on: the learning rate sits inside the velocity):
    v = mu*M + lr*G ;  M <- v ;  T = W - v
Averaging (Sec. 6): the new weights of rank j are (T[j] + T[c[j]]) / 2, where T
are the weights after the local gradient update and c is the permutation of the
step.  Momentum stays local.
"""

import numpy as np

AVG_MODEL = 0
AVG_GRAD = 1
AVG_NONE = 2


def _scalars(W, lr, mu):
    dt = W.dtype.type
    return dt(lr), dt(mu), dt(0.5)


def local_update(W, G, M, lr, mu):
    """Eq. 1-2 with momentum.  Returns (T, V): post-update weights and velocity."""
    lr, mu, _ = _scalars(W, lr, mu)
    a = mu * M
    b = lr * G
    V = a + b
    T = W - V
    return T, V


def sgd_step(W, G, M, lr, mu):
    """Plain momentum-SGD on every rank, no communication (Sec. 4.1).  In place."""
    T, V = local_update(W, G, M, lr, mu)
    W[...] = T
    M[...] = V


def gossip_step(W, G, M, c, lr, mu, avg_mode=AVG_MODEL, W_stale=None):
    """One GossipGraD step for all ranks at once.  In place on W and M.

    AVG_MODEL (Sec. 6):  W[j] <- (T[j] + T[c[j]]) / 2.
      With W_stale given (asynchronous variant, staleness 1): the partner's
      contribution is the weights it held on entry to this step,
      W[j] <- (T[j] + W_stale[c[j]]) / 2.  Callers pass a copy of W.
    AVG_GRAD: the partners' gradients are averaged before the local update,
      gbar = (G[j] + G[c[j]]) / 2 ;  v = mu*M + lr*gbar ;  M <- v ;  W <- W - v.
    AVG_NONE: local update only.
    All of T is formed before any W is overwritten.
    """
    p = W.shape[0]
    c = np.asarray(c, dtype=np.int64)
    assert c.shape == (p,)
    lr_, mu_, half = _scalars(W, lr, mu)
    if avg_mode == AVG_NONE:
        sgd_step(W, G, M, lr, mu)
        return
    if avg_mode == AVG_GRAD:
        Gbar = np.empty_like(G)
        for j in range(p):
            Gbar[j] = half * (G[j] + G[c[j]])
        T, V = local_update(W, Gbar, M, lr, mu)
        W[...] = T
        M[...] = V
        return
    if avg_mode != AVG_MODEL:
        raise ValueError("unknown avg_mode")
    T, V = local_update(W, G, M, lr, mu)
    other = T if W_stale is None else W_stale
    Wn = np.empty_like(W)
    for j in range(p):
        Wn[j] = half * (T[j] + other[c[j]])
    W[...] = Wn
    M[...] = V


def allreduce_recursive_doubling(G, average=True):
    """Recursive-doubling all-reduce over p = 2^L ranks (Sec. 3.1: the log p
    term of the all-to-all reduction).  Round k: every rank adds the buffer of
    the rank whose id differs in bit k; a fresh array per round.  With
    `average` the sum is multiplied by 1/p afterwards.  In place on G."""
    p = G.shape[0]
    if p < 2 or (p & (p - 1)):
        raise ValueError("needs a power-of-two p >= 2")
    S = G.copy()
    k = 0
    while (1 << k) < p:
        S2 = np.empty_like(S)
        for j in range(p):
            S2[j] = S[j] + S[j ^ (1 << k)]
        S = S2
        k += 1
    if average:
        S = S * G.dtype.type(G.dtype.type(1.0) / G.dtype.type(p))
    G[...] = S


def allreduce_sgd_step(W, G, M, lr, mu):
    """The baseline the paper compares with (Sec. 3.1): all-reduce the
    gradients, then every rank applies the same momentum-SGD update.  G is
    overwritten with the averaged gradient."""
    allreduce_recursive_doubling(G, average=True)
    sgd_step(W, G, M, lr, mu)


def allreduce_every_log_p_block(W, G, M, lr, mu):
    """The alternative of Sec. 7.5: every rank runs log2(p) local momentum-SGD
    steps on its own, then the models are combined by one all-reduce (average of
    the weights).  Momentum stays local.  Advances log2(p) steps in place."""
    p = W.shape[0]
    L = p.bit_length() - 1
    for _ in range(L):
        sgd_step(W, G, M, lr, mu)
    allreduce_recursive_doubling(W, average=True)
