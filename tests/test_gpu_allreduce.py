"""GPU parity: recursive-doubling all-reduce (both forms) + SGD against the
oracle (Sec. 3.1, Sec. 4.1), and the fixed point it shares with gossip."""
import numpy as np
import pytest
import torch

import paper_1803_05880_amd as gg
from oracle import gossip as og
from parity_util import assert_close_fp32, host_state

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("form", ["baseline", "onepass"])
@pytest.mark.parametrize("average", [True, False])
@pytest.mark.parametrize("p,n,stride", [(2, 5, 5), (4, 100_003, 100_004), (8, 262_151, 262_152), (16, 70_001, 70_001),
                                        (64, 10_000, 10_000), (128, 4_100, 4_100), (256, 1_031, 1_032), (1024, 515, 516)])
def test_allreduce_matches_oracle_bitwise(form, average, p, n, stride):
    _, G, _ = host_state(p, n, stride, seed=11)
    G[:, n:] = 5.0
    ctx = gg.Context(p=p, n=n, rank_stride=stride)
    g = G.to(DEV)
    getattr(ctx, "allreduce_" + form)(g, average=average)
    torch.cuda.synchronize()
    Go = G[:, :n].numpy().copy()
    og.allreduce_recursive_doubling(Go, average=average)
    out = g.cpu()
    assert assert_close_fp32(out[:, :n].numpy(), Go, "G") == 0
    assert (out[:, n:] == 5.0).all()
    ctx.close()


@pytest.mark.parametrize("shape", [
    # chunks per thread, wavefronts per workgroup, tile step, workgroups per CU, barrier, log2(ranks per barrier)
    (2, 2, 32, 3, 1, 2), (1, 8, 32, 3, 1, 0), (4, 2, 16, 0, 1, 3), (4, 1, 1, 4, 0, 1), (1, 1, 5, 0, 0, 2), (8, 1, 32, 3, 1, 1),
    (0, 2, 32, 3, 1, 2),
])
@pytest.mark.parametrize("p,n,stride", [(2, 20_005, 20_008), (8, 262_151, 262_152), (64, 70_003, 70_004), (128, 33_001, 33_004)])
def test_onepass_walk_shapes_never_change_results(shape, p, n, stride):
    # the workgroup shape of the one-pass walk and the general kernel (chunks = 0) give the oracle's bits
    chunks, waves, step, cap, barrier, group = shape
    _, G, _ = host_state(p, n, stride, seed=21)
    G[:, n:] = 5.0
    ctx = gg.Context(p=p, n=n, rank_stride=stride)
    for key, val in ((gg.TUNE_WALK_CHUNKS, 1), (gg.TUNE_WALK_WAVES, waves), (gg.TUNE_WALK_CHUNKS, chunks),
                     (gg.TUNE_WALK_STEP, step), (gg.TUNE_WALK_WG_PER_CU, cap), (gg.TUNE_WALK_BARRIER, barrier),
                     (gg.TUNE_WALK_GROUP_LOG2, group)):
        ctx.set_tuning(key, val)
    g = G.to(DEV)
    ctx.allreduce_onepass(g, average=True)
    torch.cuda.synchronize()
    Go = G[:, :n].numpy().copy()
    og.allreduce_recursive_doubling(Go, average=True)
    out = g.cpu()
    assert assert_close_fp32(out[:, :n].numpy(), Go, "G") == 0
    assert (out[:, n:] == 5.0).all()
    ctx.close()


def test_allreduce_sgd_step_and_fixed_point_with_gossip():
    p, n = 8, 300_000
    W, G, M = host_state(p, n, n, seed=12)
    ctx = gg.Context(p=p, n=n, lr=0.1, momentum=0.9)
    w, g, m = W.to(DEV), G.to(DEV), M.to(DEV)
    Wo, Go, Mo = W.numpy().copy(), G.numpy().copy(), M.numpy().copy()
    for _ in range(3):
        g.copy_(G.to(DEV))
        ctx.allreduce_baseline(g, average=True)
        ctx.sgd_step(w, g, m)
        Go[...] = G.numpy()
        og.allreduce_sgd_step(Wo, Go, Mo, 0.1, 0.9)
    torch.cuda.synchronize()
    assert np.array_equal(w.cpu().numpy(), Wo) and np.array_equal(m.cpu().numpy(), Mo)
    # identical ranks: gossip, all-reduce SGD and single-rank SGD coincide bit for bit
    W1, G1, M1 = host_state(p, n, n, seed=13, identical_ranks=True)
    wa, ga, ma = W1.to(DEV), G1.to(DEV), M1.to(DEV)
    wb, gb, mb = W1.to(DEV), G1.to(DEV), M1.to(DEV)
    for t in range(5):
        ctx.gossip_step(t, wa, ga, ma)
        gb.copy_(G1.to(DEV))
        ctx.allreduce_onepass(gb, average=True)
        ctx.sgd_step(wb, gb, mb)
    torch.cuda.synchronize()
    assert torch.equal(wa, wb) and torch.equal(ma, mb)
    assert all(torch.equal(wa[0], wa[j]) for j in range(1, p))
    ctx.close()


def test_allreduce_needs_power_of_two():
    ctx = gg.Context(p=6, n=16, topology=gg.TOPO_DISSEMINATION)
    g = torch.zeros(6, 16, device=DEV)
    with pytest.raises(gg.GGError) as e:
        ctx.allreduce_baseline(g)
    assert e.value.code == gg.binding.GG_ERR_NOT_POW2
    ctx.close()


def test_allreduce_every_log_p_steps_block_matches_oracle():
    # Sec. 7.5: log2(p) local steps, then one all-reduce of the models
    p, n, stride = 16, 250_003, 250_004
    W, G, M = host_state(p, n, stride, seed=14)
    ctx = gg.Context(p=p, n=n, rank_stride=stride, lr=0.1, momentum=0.9)
    w, g, m = W.to(DEV), G.to(DEV), M.to(DEV)
    Wo, Go, Mo = (a[:, :n].numpy().copy() for a in (W, G, M))
    for block in range(2):
        for _ in range(4):
            ctx.sgd_step(w, g, m)
        if block:
            ctx.allreduce_onepass(w, average=True)
        else:
            ctx.allreduce_baseline(w, average=True)
        og.allreduce_every_log_p_block(Wo, Go, Mo, 0.1, 0.9)
    torch.cuda.synchronize()
    assert assert_close_fp32(w.cpu()[:, :n].numpy(), Wo, "W") == 0
    assert assert_close_fp32(m.cpu()[:, :n].numpy(), Mo, "M") == 0
    ctx.close()
