"""GPU parity of the layer-wise pipelined step (Sec. 5, 5.1): the per-layer segments are
grouped into buckets in back-propagation order and each bucket's gossip update runs on a
side stream as soon as "its" piece of a stand-in computation on the main stream is done
(the flow bench.py times).  The result must not depend on the cutting, the streams or
the stand-in: bit-equal to one whole-buffer call and to the oracle."""
import numpy as np
import pytest
import torch

import bench
import gg_synth
import paper_1803_05880_amd as gg
from oracle import gossip as og
from oracle import schedule as sc
from parity_util import assert_close_fp32

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _run_pipelined(ctx, W, G, M, buckets, steps, piece):
    main = torch.cuda.current_stream()
    side = torch.cuda.Stream()
    for t in range(steps):
        bench.pipelined_step(torch, ctx, t, W, G, M, buckets, main, side, piece)
    torch.cuda.synchronize()


@pytest.mark.parametrize("topology", [gg.TOPO_HYPERCUBE, gg.TOPO_DISSEMINATION])
def test_pipelined_buckets_equal_flat_step_and_oracle_small(topology):
    p, n, seed, steps = 8, 1_000_003, 4, 5
    stride = gg.aligned_stride(n)
    seg, scales = gg_synth.segment_layout(n, 161, seed=seed, lo=64, hi=200_000)
    buckets = bench.make_buckets(seg, n, n // 24)
    assert len(buckets) > 8 and buckets[0][1] == n and buckets[-1][0] == 0
    W, G, M = gg_synth.make_state(p, n, stride, seed=seed, seg_offsets=seg, seg_scales=scales)
    ctx = gg.Context(p=p, n=n, rank_stride=stride, seed=seed, lr=gg_synth.LR, momentum=gg_synth.MOMENTUM,
                     topology=topology)
    wa, ga, ma = W.to(DEV), G.to(DEV), M.to(DEV)
    wb, gb, mb = W.to(DEV), G.to(DEV), M.to(DEV)
    sink = torch.zeros(1, device=DEV)
    _run_pipelined(ctx, wa, ga, ma, buckets, steps, lambda: gg.busy_probe(20_000, 256, sink))
    for t in range(steps):
        ctx.gossip_step(t, wb, gb, mb)
    torch.cuda.synchronize()
    assert torch.equal(wa, wb) and torch.equal(ma, mb)
    Wo, Go, Mo = (a[:, :n].numpy().copy() for a in (W, G, M))
    otopo = sc.HYPERCUBE if topology == gg.TOPO_HYPERCUBE else sc.DISSEMINATION
    for t in range(steps):
        og.gossip_step(Wo, Go, Mo, sc.partners(p, seed, p, otopo, t)[1], gg_synth.LR, gg_synth.MOMENTUM)
    assert assert_close_fp32(wa.cpu()[:, :n].numpy(), Wo, "W") == 0
    assert assert_close_fp32(ma.cpu()[:, :n].numpy(), Mo, "M") == 0
    ctx.close()


@pytest.mark.parametrize("stand_in", ["arithmetic", "memory_streaming"])
def test_pipelined_buckets_config3_shape(stand_in):
    # p = 16 x ResNet50-sized rows in 161 segments, the bucket list bench.py uses, both stand-ins
    p, n, seed, steps = 16, gg_synth.RESNET50_PARAMS, 0, 4
    stride = gg.aligned_stride(n)
    seg, scales = gg_synth.segment_layout(n, 161, seed=seed)
    buckets = bench.make_buckets(seg, n, n // 24)
    W, G, M = gg_synth.make_state(p, n, stride, seed=seed, device=DEV, seg_offsets=seg, seg_scales=scales)
    cols = np.unique(np.concatenate([np.arange(lo, hi) for lo, hi in
                                     gg_synth.sample_windows(n, num_random=64, width=1024, seed=2)] +
                                    [np.arange(max(0, lo - 96), min(n, lo + 96)) for lo, _ in buckets]))   # bucket cuts
    cd = torch.as_tensor(cols, device=DEV)
    take = lambda t: t.index_select(1, cd).cpu().numpy()
    Wo, Go, Mo = take(W), take(G), take(M)
    wb, mb = W.clone(), M.clone()
    ctx = gg.Context(p=p, n=n, rank_stride=stride, seed=seed, lr=gg_synth.LR, momentum=gg_synth.MOMENTUM)
    if stand_in == "arithmetic":
        sink = torch.zeros(1, device=DEV)
        piece = lambda: gg.busy_probe(40_000, 1024, sink)
    else:
        slab = torch.zeros(64 * 1024 * 1024, device=DEV)
        piece = lambda: gg.stream_probe(8, 1024, slab)
    _run_pipelined(ctx, W, G, M, buckets, steps, piece)
    for t in range(steps):
        ctx.gossip_step(t, wb, G, mb)
        og.gossip_step(Wo, Go, Mo, sc.partners(p, seed, p, sc.HYPERCUBE, t)[1], gg_synth.LR, gg_synth.MOMENTUM)
    torch.cuda.synchronize()
    assert torch.equal(W, wb) and torch.equal(M, mb)
    assert assert_close_fp32(take(W), Wo, "W") == 0
    assert assert_close_fp32(take(M), Mo, "M") == 0
    ctx.close()
