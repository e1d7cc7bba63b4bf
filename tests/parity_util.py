"""Helpers shared by the GPU parity tests: run the oracle and the HIP path on
the same seeded inputs and gate the difference.

Gate (fp32 parameters): per rank, max_i |gpu - oracle| <= 1e-6 * max(|oracle_i|,
1e-3 * max|oracle|) -- the "within 1e-6 relative" bar; both sides evaluate the
same fp32 operations in the same order with no fused multiply-add, so the
number of elements that differ in any bit is also reported and expected to be 0.
"""
import numpy as np

import gg_synth
from oracle import gossip as og
from oracle import schedule as sc

REL_TOL = 1e-6


def assert_close_fp32(gpu, ora, what):
    gpu = np.asarray(gpu)
    ora = np.asarray(ora)
    assert gpu.shape == ora.shape and gpu.dtype == np.float32, what
    for j in range(ora.shape[0]):
        floor = 1e-3 * float(np.abs(ora[j]).max()) if ora[j].size else 0.0
        bound = REL_TOL * np.maximum(np.abs(ora[j]), floor)
        err = np.abs(gpu[j].astype(np.float64) - ora[j].astype(np.float64))
        bad = int((err > bound).sum())
        assert bad == 0, "%s rank %d: %d elements beyond 1e-6 relative (max err %g)" % (what, j, bad, err.max())
    return int((gpu.view(np.uint32) != ora.view(np.uint32)).sum())


def host_state(p, n, stride=None, seed=0, **kw):
    """Seeded W, G, M on the host as torch tensors [p][stride]."""
    return gg_synth.make_state(p, n, stride, seed=seed, device="cpu", **kw)


def oracle_run(W, G, M, n, p, seed, steps, topology=sc.HYPERCUBE, num_comms=0, lr=gg_synth.LR,
               mu=gg_synth.MOMENTUM, avg_mode=og.AVG_MODEL, staleness=0, first_step=0):
    """Advance numpy copies of the first n columns with the oracle; returns (W, M)."""
    Wn = W[:, :n].numpy().copy()
    Gn = G[:, :n].numpy().copy()
    Mn = M[:, :n].numpy().copy()
    R = p if num_comms == 0 else num_comms
    for t in range(first_step, first_step + steps):
        send, recv = sc.partners(p, seed, R, topology, t)
        stale = Wn.copy() if staleness else None
        og.gossip_step(Wn, Gn, Mn, recv, lr, mu, avg_mode=avg_mode, W_stale=stale)
    return Wn, Mn
