"""Seeded differential sweep on the GPU: random rank counts, sizes, strides, base
misalignments, modes, topologies, segment ranges and launch shapes, each compared
bit for bit with the CPU oracle through the C ABI."""
import numpy as np
import pytest
import torch

import gg_synth
import paper_1803_05880_amd as gg
from oracle import gossip as og
from oracle import schedule as sc

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _case(rng):
    topology = int(rng.integers(0, 2))
    p = int(2 ** rng.integers(1, 7)) if topology == 0 or rng.random() < 0.5 else int(rng.integers(2, 70))
    n = int(rng.choice([1, 5, 63, 64, 257, 4096, 10_007, 65_536, 131_075, 300_001]))
    stride = n + int(rng.choice([0, 1, 3, 4, 8, 60, 252, 1020]))
    shift = int(rng.choice([0, 0, 1, 2, 4, 8, 64]))        # floats by which every base pointer is moved
    mode = [dict(), dict(staleness=1), dict(avg_mode=gg.AVG_GRAD), dict(avg_mode=gg.AVG_NONE)][int(rng.integers(0, 4))]
    double = bool(rng.integers(0, 2)) and mode.get("avg_mode", 0) != gg.AVG_NONE
    seg = None
    if rng.random() < 0.4 and n > 8:
        lo = int(rng.integers(0, n // 2))
        hi = int(rng.integers(lo, n + 1))
        seg = np.array(sorted({lo, hi, int(rng.integers(lo, hi + 1))}), dtype=np.int64)
        if len(seg) < 2:
            seg = np.array([lo, lo], dtype=np.int64)
    tune = {}
    if rng.random() < 0.5:
        tune = {gg.TUNE_THREADS: int(rng.choice([64, 128, 256])), gg.TUNE_CHUNKS: int(rng.choice([1, 2, 4, 8])),
                gg.TUNE_BLOCKS_PER_CU: int(rng.choice([0, 3, 7, 20])), gg.TUNE_WALK_STEP: int(rng.choice([1, 5, 32, 64])),
                gg.TUNE_WALK_BARRIER: int(rng.choice([0, 1]))}
    return dict(topology=topology, p=p, n=n, stride=stride, shift=shift, mode=mode, double=double, seg=seg, tune=tune,
                steps=int(rng.integers(1, 5)), first=int(rng.integers(0, 200)), seed=int(rng.integers(0, 2**40)))


def _shifted(t, shift):
    raw = torch.zeros(t.numel() + shift, device=DEV)
    view = raw[shift:].view(t.shape)
    view.copy_(t)
    return view


@pytest.mark.parametrize("block", range(6))
def test_random_configurations_match_the_oracle(block):
    rng = np.random.default_rng(1000 + block)
    for _ in range(12):
        c = _case(rng)
        p, n, stride = c["p"], c["n"], c["stride"]
        W, G, M = gg_synth.make_state(p, n, stride, seed=c["seed"] % 1000)
        M[:, :n].normal_(0, 1e-3, generator=torch.Generator().manual_seed(7))
        W[:, n:] = 3.0
        ctx = gg.Context(p=p, n=n, rank_stride=stride, seed=c["seed"], topology=c["topology"], lr=0.1, momentum=0.9,
                         **c["mode"])
        for k, v in c["tune"].items():
            ctx.set_tuning(k, v)
        w, g, m = (_shifted(t, c["shift"]) for t in (W, G, M))
        w2 = _shifted(torch.full_like(W, 9.0), c["shift"]) if c["double"] else None
        lo, hi = (0, n) if c["seg"] is None else (int(c["seg"][0]), int(c["seg"][-1]))
        Wo, Go, Mo = (a.numpy().copy() for a in (W, G, M))
        for t in range(c["first"], c["first"] + c["steps"]):
            ctx.gossip_step(t, w, g, m, w_next=w2, seg_offsets=c["seg"])
            if c["double"]:
                # only [lo, hi) is written to w_next: carry the rest over, then swap roles
                w2[:, :lo] = w[:, :lo]
                w2[:, hi:] = w[:, hi:]
                w, w2 = w2, w
            recv = sc.partners(p, c["seed"], p, c["topology"], t)[1]
            ws, gs, ms = (np.ascontiguousarray(a[:, lo:hi]) for a in (Wo, Go, Mo))
            og.gossip_step(ws, gs, ms, recv, 0.1, 0.9, avg_mode=c["mode"].get("avg_mode", 0),
                           W_stale=ws.copy() if c["mode"].get("staleness") else None)
            Wo[:, lo:hi], Mo[:, lo:hi] = ws, ms
        torch.cuda.synchronize()
        assert np.array_equal(w.cpu().numpy(), Wo), c
        assert np.array_equal(m.cpu().numpy(), Mo), c
        assert np.array_equal(g.cpu().numpy(), Go), c
        ctx.close()
