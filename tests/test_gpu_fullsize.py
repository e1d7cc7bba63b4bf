"""GPU parity at the full workload sizes, in the launch configuration bench.py
times (default tuning, rank stride rounded up to 1024 elements).

The step is elementwise in the parameter index, so the oracle restricted to a
set of columns is exactly the restriction of the full result: the oracle runs
on sampled windows (first/last 4096, every 64 Mi-element boundary, random
windows) of all p ranks, fed with the initial device buffers read back for
those columns.  Inputs are generated on the GPU by the seeded generator."""
import numpy as np
import pytest
import torch

import gg_synth
import paper_1803_05880_amd as gg
from oracle import gossip as og
from oracle import schedule as sc
from parity_util import assert_close_fp32

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _columns(n, num_random):
    cols = np.unique(np.concatenate([np.arange(lo, hi) for lo, hi in
                                     gg_synth.sample_windows(n, num_random=num_random, width=1024, seed=1)]))
    return cols


def _take(t, cols_dev):
    return t.index_select(1, cols_dev).cpu().numpy()


def _bench_stride(n):
    return (n + 1023) // 1024 * 1024


@pytest.mark.parametrize("staleness", [0, 1])
def test_config4_scale_out_shape_sampled_windows(staleness):
    # p=64 x ResNet50-sized buffers; synchronous, and staleness 1 through a double buffer
    p, n, seed = 64, gg_synth.RESNET50_PARAMS, 0
    stride = _bench_stride(n)
    W, G, M = gg_synth.make_state(p, n, stride, seed=seed, device=DEV)
    cols = _columns(n, 256)
    cd = torch.as_tensor(cols, device=DEV)
    Wo, Go, Mo = _take(W, cd), _take(G, cd), _take(M, cd)
    W0o, M0o = Wo.copy(), Mo.copy()
    ctx = gg.Context(p=p, n=n, rank_stride=stride, seed=seed, lr=gg_synth.LR, momentum=gg_synth.MOMENTUM,
                     staleness=staleness)
    W2 = torch.empty_like(W) if staleness else None
    bufs = [W, W2]
    steps = 8                                            # L = 6: crosses into the first shuffled communicator
    for t in range(steps):
        if staleness:
            ctx.gossip_step(t, bufs[t & 1], G, M, w_next=bufs[(t & 1) ^ 1])
        else:
            ctx.gossip_step(t, W, G, M)
        c = sc.partners(p, seed, p, sc.HYPERCUBE, t)[1]
        assert ctx.partner(t)[1].tolist() == c
        og.gossip_step(Wo, Go, Mo, c, gg_synth.LR, gg_synth.MOMENTUM, W_stale=Wo.copy() if staleness else None)
    torch.cuda.synchronize()
    Wfinal = bufs[steps & 1] if staleness else W
    if not staleness:
        # reported, not gated at 1e-6: drift of the fp32 path from a float64 run of the same steps
        W64, G64, M64 = (a.astype(np.float64) for a in (W0o, Go, M0o))
        for t in range(steps):
            og.gossip_step(W64, G64, M64, sc.partners(p, seed, p, sc.HYPERCUBE, t)[1], np.float32(gg_synth.LR),
                           np.float32(gg_synth.MOMENTUM))
        drift = np.abs(Wo - W64).max() / np.abs(W64).max()
        print("fp32 vs float64 after %d steps: max |dW| / max |W| = %.3g" % (steps, drift))
        assert drift < steps * 4 * 2.0 ** -24
    dw = assert_close_fp32(_take(Wfinal, cd), Wo, "W")
    dm = assert_close_fp32(_take(M, cd), Mo, "M")
    assert dw == 0 and dm == 0
    assert torch.count_nonzero(Wfinal[:, n:]) == 0       # padding untouched
    # property that holds at any size: partners hold identical weights after a synchronous step
    if not staleness:
        c = ctx.partner(steps - 1)[1]
        for j in (0, 17, 63):
            assert torch.equal(W[j, :n], W[int(c[j]), :n])
    ctx.close()


def test_config5_full_method_step_sampled_windows_and_shuffle():
    # p=128 x ResNet50-sized buffers + partner-swap shuffle of 1,281,167 ids
    from oracle import shuffle as sh
    p, n, seed = 128, gg_synth.RESNET50_PARAMS, 0
    stride = _bench_stride(n)
    W, G, M = gg_synth.make_state(p, n, stride, seed=seed, device=DEV)
    cols = _columns(n, 256)
    cd = torch.as_tensor(cols, device=DEV)
    Wo, Go, Mo = _take(W, cd), _take(G, cd), _take(M, cd)
    off = sh.block_offsets(gg_synth.IMAGENET1K_TRAIN, p)
    idx = gg_synth.make_indices(gg_synth.IMAGENET1K_TRAIN, DEV)
    idx_o = sh.initial_indices(gg_synth.IMAGENET1K_TRAIN)
    ctx = gg.Context(p=p, n=n, rank_stride=stride, seed=seed, lr=gg_synth.LR, momentum=gg_synth.MOMENTUM)
    for t in [0, 1, 6, 7, 8]:                            # L = 7: steps 7, 8 use a shuffled communicator
        ctx.gossip_step(t, W, G, M)
        ctx.shuffle(t, gg.SHUF_PARTNER_SWAP, idx, off)
        c = sc.partners(p, seed, p, sc.HYPERCUBE, t)[1]
        og.gossip_step(Wo, Go, Mo, c, gg_synth.LR, gg_synth.MOMENTUM)
        sh.partner_swap_step(idx_o, off, c, seed, t)
    torch.cuda.synchronize()
    assert assert_close_fp32(_take(W, cd), Wo, "W") == 0
    assert assert_close_fp32(_take(M, cd), Mo, "M") == 0
    assert np.array_equal(idx.cpu().numpy(), idx_o)
    ctx.close()


def test_config3_segments_and_allreduce_comparator_sampled_windows():
    # p=16 x ResNet50-sized buffers in 161 per-layer segments with per-layer gradient scales;
    # the recursive-doubling all-reduce + SGD runs on a copy of the same buffers
    p, n, seed = 16, gg_synth.RESNET50_PARAMS, 0
    stride = _bench_stride(n)
    seg, scales = gg_synth.segment_layout(n, 161, seed=seed)
    assert seg[0] == 0 and seg[-1] == n and len(seg) == 162 and (np.diff(seg) >= 1).all()
    W, G, M = gg_synth.make_state(p, n, stride, seed=seed, device=DEV, seg_offsets=seg, seg_scales=scales)
    cols = _columns(n, 256)
    cd = torch.as_tensor(cols, device=DEV)
    Wo, Go, Mo = _take(W, cd), _take(G, cd), _take(M, cd)
    Wa, Ga, Ma = W.clone(), G.clone(), M.clone()
    Wao, Gao, Mao = Wo.copy(), Go.copy(), Mo.copy()
    ctx = gg.Context(p=p, n=n, rank_stride=stride, seed=seed, lr=gg_synth.LR, momentum=gg_synth.MOMENTUM)
    for t in range(32):
        ctx.gossip_step(t, W, G, M, seg_offsets=seg)
        og.gossip_step(Wo, Go, Mo, sc.partners(p, seed, p, sc.HYPERCUBE, t)[1], gg_synth.LR, gg_synth.MOMENTUM)
    for t in range(3):
        Ga.copy_(G)
        if t == 1:
            ctx.allreduce_onepass(Ga, average=True)
        else:
            ctx.allreduce_baseline(Ga, average=True)
        ctx.sgd_step(Wa, Ga, Ma)
        Gao[...] = Go
        og.allreduce_sgd_step(Wao, Gao, Mao, gg_synth.LR, gg_synth.MOMENTUM)
    torch.cuda.synchronize()
    assert assert_close_fp32(_take(W, cd), Wo, "W gossip") == 0
    assert assert_close_fp32(_take(M, cd), Mo, "M gossip") == 0
    assert assert_close_fp32(_take(Wa, cd), Wao, "W allreduce") == 0
    assert assert_close_fp32(_take(Ma, cd), Mao, "M allreduce") == 0
    assert assert_close_fp32(_take(Ga, cd), Gao, "G allreduce") == 0
    # any size: after the all-reduce every rank holds the same gradient bits
    assert torch.equal(Ga[0, :n], Ga[p - 1, :n])
    ctx.close()


# ---------------------------------------------------------------------------------------------
# The configured step counts, the paper's preferred topology and gradient averaging at full size
# ---------------------------------------------------------------------------------------------
def _sampled(W, G, M, n, num_random):
    cols = _columns(n, num_random)
    cd = torch.as_tensor(cols, device=DEV)
    return cd, _take(W, cd), _take(G, cd), _take(M, cd)


def _assert_bit_equal(cd, Wdev, Mdev, Wo, Mo, what):
    dw = assert_close_fp32(_take(Wdev, cd), Wo, "W " + what)
    dm = assert_close_fp32(_take(Mdev, cd), Mo, "M " + what)
    assert dw == 0 and dm == 0, "%s: differing bits W %d, M %d" % (what, dw, dm)


def _run_full(p, steps, checkpoints, topology=gg.TOPO_HYPERCUBE, staleness=0, avg_mode=gg.AVG_MODEL,
              double_buffer=False, num_random=64, shuffle=False, seed=0):
    """Run `steps` consecutive steps at N = 25,557,032 on the GPU and on the sampled-window
    oracle, comparing at every step listed in `checkpoints` (steps already done) and at the end."""
    from oracle import shuffle as sh
    n = gg_synth.RESNET50_PARAMS
    stride = _bench_stride(n)
    W, G, M = gg_synth.make_state(p, n, stride, seed=seed, device=DEV)
    cd, Wo, Go, Mo = _sampled(W, G, M, n, num_random)
    ctx = gg.Context(p=p, n=n, rank_stride=stride, seed=seed, lr=gg_synth.LR, momentum=gg_synth.MOMENTUM,
                     topology=topology, staleness=staleness, avg_mode=avg_mode)
    bufs = [W, torch.full_like(W, float("nan")) if double_buffer else None]
    cur = 0
    if shuffle:
        off = sh.block_offsets(gg_synth.IMAGENET1K_TRAIN, p)
        idx = gg_synth.make_indices(gg_synth.IMAGENET1K_TRAIN, DEV)
        idx_o = sh.initial_indices(gg_synth.IMAGENET1K_TRAIN)
    otopo = sc.HYPERCUBE if topology == gg.TOPO_HYPERCUBE else sc.DISSEMINATION
    for t in range(steps):
        if double_buffer:
            ctx.gossip_step(t, bufs[cur], G, M, w_next=bufs[cur ^ 1])
            cur ^= 1
        else:
            ctx.gossip_step(t, W, G, M)
        send, recv = sc.partners(p, seed, p, otopo, t)
        gs, gr = ctx.partner(t)
        assert gs.tolist() == send and gr.tolist() == recv
        og.gossip_step(Wo, Go, Mo, recv, gg_synth.LR, gg_synth.MOMENTUM, avg_mode=avg_mode,
                       W_stale=Wo.copy() if staleness else None)
        if shuffle:
            ctx.shuffle(t, gg.SHUF_PARTNER_SWAP, idx, off)
            sh.partner_swap_step(idx_o, off, recv, seed, t)
        if t + 1 in checkpoints or t + 1 == steps:
            torch.cuda.synchronize()
            _assert_bit_equal(cd, bufs[cur], M, Wo, Mo, "after %d steps" % (t + 1))
            if shuffle:
                assert np.array_equal(idx.cpu().numpy(), idx_o), "indices after %d steps" % (t + 1)
    assert np.array_equal(_take(G, cd), Go)              # g is never written
    if not double_buffer:
        assert torch.count_nonzero(W[:, n:]) == 0        # padding untouched
    assert torch.count_nonzero(M[:, n:]) == 0
    ctx.close()
    return bufs[cur]


@pytest.mark.parametrize("staleness", [0, 1])
def test_config4_all_64_steps(staleness):
    # the configured run: 64 consecutive steps, i.e. communicators 0..10 of the 64, L = 6;
    # staleness 1 goes through the double buffer
    _run_full(64, 64, checkpoints=(1, 31), staleness=staleness, double_buffer=bool(staleness))


def test_config5_all_128_steps_with_shuffle_every_step():
    # the configured run: 128 consecutive steps (communicators 0..18, L = 7), the partner-swap
    # shuffle of the 1,281,167 ids at every step
    _run_full(128, 128, checkpoints=(1, 64), shuffle=True, num_random=48)


@pytest.mark.parametrize("staleness,double_buffer", [(0, False), (0, True), (1, False), (1, True)])
def test_config4_shape_dissemination(staleness, double_buffer):
    # the paper's preferred topology (Sec. 4.4.2) at p = 64 x ResNet50-sized rows: 2L + 2 = 14 steps
    # cover every phase twice (long cycles included) and cross into two shuffled communicators
    _run_full(64, 14, checkpoints=(1, 6, 7), topology=gg.TOPO_DISSEMINATION, staleness=staleness,
              double_buffer=double_buffer)


@pytest.mark.parametrize("topology", [gg.TOPO_HYPERCUBE, gg.TOPO_DISSEMINATION])
def test_config4_shape_gradient_averaging(topology):
    # the gradient-buffer reading of the exchange (Sec. 5) at p = 64 x ResNet50-sized rows
    _run_full(64, 14, checkpoints=(1, 7), topology=topology, avg_mode=gg.AVG_GRAD)


def test_config5_shape_dissemination():
    # p = 128: the longest partner cycle (all 128 ranks at phase 0) down to pairs, 9 steps = every phase and
    # two steps on a shuffled communicator
    _run_full(128, 9, checkpoints=(1, 7), topology=gg.TOPO_DISSEMINATION, num_random=32)


@pytest.mark.parametrize("p", [64, 128])
def test_allreduce_forms_at_full_size(p):
    # the comparator at p = 64 and p = 128 x ResNet50-sized rows: the one-pass walk (a register stack of
    # log2 p partial sums) and the L rounds give the same bits over the whole buffer, and the oracle's on
    # sampled windows; every rank ends with the same gradient
    n = gg_synth.RESNET50_PARAMS
    stride = _bench_stride(n)
    gen = torch.Generator(device=DEV).manual_seed(p)
    G = torch.zeros((p, stride), device=DEV)
    G[:, :n].normal_(0.0, gg_synth.G_STD, generator=gen)
    cols = _columns(n, 32)
    cd = torch.as_tensor(cols, device=DEV)
    Go = _take(G, cd)
    ctx = gg.Context(p=p, n=n, rank_stride=stride)
    g1, g2 = G.clone(), G
    ctx.allreduce_onepass(g1, average=True)
    ctx.allreduce_baseline(g2, average=True)
    torch.cuda.synchronize()
    assert torch.equal(g1, g2)
    assert torch.equal(g1[0], g1[p - 1]) and torch.equal(g1[0], g1[p // 2])
    assert torch.count_nonzero(g1[:, n:]) == 0
    og.allreduce_recursive_doubling(Go, average=True)
    assert assert_close_fp32(_take(g1, cd), Go, "G") == 0
    ctx.close()
