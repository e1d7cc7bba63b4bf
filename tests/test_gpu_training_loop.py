"""The hot path inside a (toy) training loop on the GPU: p virtual ranks fit one
linear model by least squares on synthetic data, each rank on the samples its
resident index set currently holds.  Gradients come from plain torch ops (the
stand-in for forward/backward); the update, the exchange and the sample rotation
are the library's.  Checks the behaviour the paper argues for (Sec. 4.1, 4.5, 6):
without communication the replicas stay apart, with gossip + partner rotation
they agree on one model that is as good as the all-reduce baseline's, and the
ring rotation shows every rank every sample."""
import pytest
import torch

import gg_synth
import paper_1803_05880_amd as gg

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _train(mode, steps=400, p=8, d=512, n_samples=4096, batch=64, seed=0):
    gen = torch.Generator(device=DEV).manual_seed(seed)
    X = torch.randn(n_samples, d, device=DEV, generator=gen)
    w_true = torch.randn(d, device=DEV, generator=gen)
    # per-rank bias in the labels: every shard alone has a different optimum
    shard_shift = torch.randn(p, device=DEV, generator=gen).repeat_interleave(n_samples // p) * 2.0
    y = X @ w_true + shard_shift + 0.01 * torch.randn(n_samples, device=DEV, generator=gen)
    stride = gg.aligned_stride(d)
    W = torch.zeros(p, stride, device=DEV)
    G = torch.zeros(p, stride, device=DEV)
    M = torch.zeros(p, stride, device=DEV)
    idx = gg_synth.make_indices(n_samples, DEV)
    off = gg_synth.block_offsets(n_samples, p)
    per_rank = n_samples // p
    ctx = gg.Context(p=p, n=d, rank_stride=stride, seed=seed, lr=0.02, momentum=0.9,
                     avg_mode=gg.AVG_NONE if mode == "none" else gg.AVG_MODEL)
    seen = torch.zeros(p, n_samples, dtype=torch.bool, device=DEV)
    for t in range(steps):
        head = (t * batch) % per_rank if mode != "none" else (t * batch) % per_rank
        cols = (head + torch.arange(batch, device=DEV)) % per_rank
        rows = idx.view(p, per_rank)[:, cols].long()                 # [p][batch] sample ids used this step
        seen[torch.arange(p, device=DEV)[:, None], rows] = True
        Xb, yb = X[rows], y[rows]                                    # [p][batch][d], [p][batch]
        resid = torch.einsum("pbd,pd->pb", Xb, W[:, :d]) - yb
        G[:, :d] = torch.einsum("pbd,pb->pd", Xb, resid) / batch     # least-squares gradient per rank
        if mode == "allreduce":
            ctx.allreduce_onepass(G, average=True)
            ctx.sgd_step(W, G, M)
        else:
            ctx.gossip_step(t, W, G, M)
        if mode != "none":
            ctx.shuffle(t, gg.SHUF_RING, idx, off, batch=batch)       # used batch moves to the ring neighbour
    torch.cuda.synchronize()
    w = W[:, :d]
    consensus = float((w - w.mean(0)).norm(dim=1).max() / w.mean(0).norm())
    loss = float(((X @ w.mean(0) - y) ** 2).mean())
    ctx.close()
    return consensus, loss, seen


def test_gossip_reaches_consensus_and_matches_allreduce_quality():
    c_none, l_none, seen_none = _train("none")
    c_gossip, l_gossip, seen_gossip = _train("gossip")
    c_ar, l_ar, _ = _train("allreduce")
    assert c_ar < 1e-6                                   # all-reduce SGD keeps the replicas identical
    assert c_none > 10 * c_gossip and l_none > 1.5 * l_ar   # no communication: replicas stay apart (Sec. 4.1)
    assert c_gossip < 0.05                               # gossip + rotation: one model (Sec. 6, corollary)
    assert l_gossip < 1.1 * l_ar                         # and as good as the all-reduce baseline's
    # ring rotation: every rank has seen (almost) every sample; without it only its own shard (Lemma 1)
    assert float(seen_gossip.float().mean()) > 0.9
    assert abs(float(seen_none.float().mean()) - 1.0 / 8) < 1e-6
