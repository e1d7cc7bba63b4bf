"""GPU parity: sample-index rotation (Sec. 4.5.2), bit-exact against the oracle."""
import numpy as np
import pytest
import torch

import gg_synth
import paper_1803_05880_amd as gg
from oracle import schedule as sc
from oracle import shuffle as sh

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("p,n_total", [(2, 10), (2, 100_001), (4, 1_001), (8, 40_963), (16, 777), (64, 70_000),
                                       (128, 1_281_167), (4, 1_281_167)])
def test_partner_swap_bit_exact(p, n_total):
    seed = 21
    off = sh.block_offsets(n_total, p)
    idx_o = sh.initial_indices(n_total)
    idx_g = gg_synth.make_indices(n_total, DEV)
    ctx = gg.Context(p=p, n=4, seed=seed)
    L = sc.num_phases(p)
    steps = [0, 1, L, L + 1, 2 * L + 1] if n_total > 200_000 else list(range(2 * L + 2))
    for t in steps:
        c, _ = sc.partners(p, seed, p, sc.HYPERCUBE, t)
        sh.partner_swap_step(idx_o, off, c, seed, t)
        ctx.shuffle(t, gg.SHUF_PARTNER_SWAP, idx_g, off)
        got = idx_g.cpu().numpy()
        assert np.array_equal(got, idx_o), "step %d" % t
    assert np.array_equal(np.sort(got), np.arange(n_total))
    if n_total >= 1000:
        assert not np.array_equal(got, np.arange(n_total))
    ctx.close()


def test_partner_swap_uneven_and_empty_ranks():
    p = 4
    off = np.array([0, 0, 5000, 5003, 20_000], dtype=np.int64)       # an empty rank, a tiny one
    idx_o = sh.initial_indices(20_000)
    idx_g = gg_synth.make_indices(20_000, DEV)
    ctx = gg.Context(p=p, n=4, seed=3)
    for t in range(6):
        c, _ = sc.partners(p, 3, p, sc.HYPERCUBE, t)
        sh.partner_swap_step(idx_o, off.tolist(), c, 3, t)
        ctx.shuffle(t, gg.SHUF_PARTNER_SWAP, idx_g, off)
    assert np.array_equal(idx_g.cpu().numpy(), idx_o)
    ctx.close()


@pytest.mark.parametrize("p,n_total,batch", [(3, 12, 2), (4, 32, 2), (5, 23, 4), (8, 100_003, 32), (16, 50_000, 3125),
                                             (128, 1_281_167, 32), (7, 1000, 0)])
@pytest.mark.parametrize("topology", [gg.TOPO_DISSEMINATION])
def test_ring_bit_exact(p, n_total, batch, topology):
    off = sh.block_offsets(n_total, p)
    idx_o = sh.initial_indices(n_total)
    idx_g = gg_synth.make_indices(n_total, DEV)
    ctx = gg.Context(p=p, n=4, topology=topology)
    n_min = min(np.diff(off))
    steps = list(range(7)) + [n_min // max(batch, 1) + 1, 10**9 + 7]
    for t in steps:
        sh.ring_step(idx_o, off, batch, t)
        ctx.shuffle(t, gg.SHUF_RING, idx_g, off, batch=batch)
        assert np.array_equal(idx_g.cpu().numpy(), idx_o), "step %d" % t
    ctx.close()


def test_shuffle_argument_errors():
    ctx = gg.Context(p=4, n=4)
    idx = gg_synth.make_indices(100, DEV)
    E = gg.binding
    with pytest.raises(gg.GGError) as e:
        ctx.shuffle(0, gg.SHUF_RING, idx, [0, 25, 50, 75, 100], batch=26)
    assert e.value.code == E.GG_ERR_ARG
    with pytest.raises(gg.GGError) as e:
        ctx.shuffle(0, gg.SHUF_RING, idx, [1, 25, 50, 75, 100], batch=2)
    assert e.value.code == E.GG_ERR_ARG
    with pytest.raises(gg.GGError) as e:
        ctx.shuffle(0, gg.SHUF_RING, idx, [0, 50, 25, 75, 100], batch=2)
    assert e.value.code == E.GG_ERR_ARG
    with pytest.raises(gg.GGError) as e:
        ctx.shuffle(0, 5, idx, [0, 25, 50, 75, 100])
    assert e.value.code == E.GG_ERR_ARG
    ctx.close()
    ctx = gg.Context(p=6, n=4, topology=gg.TOPO_DISSEMINATION)
    with pytest.raises(gg.GGError) as e:
        ctx.shuffle(0, gg.SHUF_PARTNER_SWAP, idx, [0, 10, 20, 30, 40, 50, 60])
    assert e.value.code == E.GG_ERR_UNSUPPORTED
    torch.cuda.synchronize()
    assert np.array_equal(idx.cpu().numpy(), np.arange(100))
    ctx.close()
