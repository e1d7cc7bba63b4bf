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


@pytest.mark.parametrize("off", [[0, 0, 5000, 5003, 20_000],            # one workgroup per pair
                                 [0, 0, 70_000, 70_003, 200_000],       # many tiles per rank: count/scatter/swap kernels
                                 [0, 40_961, 40_961, 81_922, 81_923]])
def test_partner_swap_uneven_and_empty_ranks(off):
    p = 4
    off = np.array(off, dtype=np.int64)                              # an empty rank, a tiny one
    idx_o = sh.initial_indices(int(off[-1]))
    idx_g = gg_synth.make_indices(int(off[-1]), DEV)
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


@pytest.mark.parametrize("p,n_total,batch,sample_words", [(2, 10, 3, 8), (3, 12, 2, 4), (4, 64, 4, 12), (8, 1000, 17, 5),
                                                          (16, 4096, 32, 3072), (128, 128 * 40, 32, 1024)])
def test_ring_payload_bit_exact_and_glued_to_indices(p, n_total, batch, sample_words):
    off = sh.block_offsets(n_total, p)
    rng = np.random.default_rng(5)
    pay_o = rng.integers(-2**31, 2**31 - 1, size=(n_total, sample_words), dtype=np.int64).astype(np.int32)
    pay_o[:, 0] = np.arange(n_total)                        # tag: word 0 is the sample id
    pay_g = torch.from_numpy(pay_o.copy()).to(DEV)
    idx_g = gg_synth.make_indices(n_total, DEV)
    ctx = gg.Context(p=p, n=4, topology=gg.TOPO_DISSEMINATION)
    for t in [0, 1, 2, 3, 11, 10**6 + 3]:
        sh.ring_payload_step(pay_o, off, batch, t)
        ctx.shuffle_payload(t, pay_g, off, batch)
        ctx.shuffle(t, gg.SHUF_RING, idx_g, off, batch=batch)
        got = pay_g.cpu().numpy()
        assert np.array_equal(got, pay_o), "step %d" % t
        assert np.array_equal(got[:, 0], idx_g.cpu().numpy())   # payload rows follow their indices
    ctx.close()


@pytest.mark.parametrize("shape", [
    # chunks per thread, wavefronts per workgroup, tile step, workgroups per CU, barrier per rank
    (2, 2, 32, 3, 1), (1, 8, 32, 3, 1), (8, 1, 3, 0, 0), (4, 2, 16, 4, 1), (1, 1, 1, 0, 0), (0, 1, 32, 3, 1),
])
@pytest.mark.parametrize("p,n_total,batch,sample_words", [(5, 5 * 9, 7, 3076), (16, 16 * 5, 5, 260), (64, 64 * 3, 2, 49_152)])
def test_ring_payload_walk_shapes_never_change_results(shape, p, n_total, batch, sample_words):
    # samples that are not a whole number of 1 KB tiles, queues that wrap, and the image size of Table 5
    chunks, waves, step, cap, barrier = shape
    off = sh.block_offsets(n_total, p)
    rng = np.random.default_rng(6)
    pay_o = rng.integers(-2**31, 2**31 - 1, size=(n_total, sample_words), dtype=np.int64).astype(np.int32)
    pay_g = torch.from_numpy(pay_o.copy()).to(DEV)
    ctx = gg.Context(p=p, n=4, topology=gg.TOPO_DISSEMINATION)
    for key, val in ((gg.TUNE_WALK_CHUNKS, 1), (gg.TUNE_WALK_WAVES, waves), (gg.TUNE_WALK_CHUNKS, chunks),
                     (gg.TUNE_WALK_STEP, step), (gg.TUNE_WALK_WG_PER_CU, cap), (gg.TUNE_WALK_BARRIER, barrier)):
        ctx.set_tuning(key, val)
    for t in [0, 1, 2, 7, 10**9 + 1]:
        sh.ring_payload_step(pay_o, off, batch, t)
        ctx.shuffle_payload(t, pay_g, off, batch)
        assert np.array_equal(pay_g.cpu().numpy(), pay_o), "step %d" % t
    ctx.close()


def test_ring_payload_unaligned_rows_take_the_word_path():
    p, n_total, batch = 4, 40, 3
    off = sh.block_offsets(n_total, p)
    pay_o = np.arange(n_total * 7, dtype=np.int32).reshape(n_total, 7)      # 28-byte rows
    pay_g = torch.from_numpy(pay_o.copy()).to(DEV)
    ctx = gg.Context(p=p, n=4)
    for t in range(5):
        sh.ring_payload_step(pay_o, off, batch, t)
        ctx.shuffle_payload(t, pay_g, off, batch)
    assert np.array_equal(pay_g.cpu().numpy(), pay_o)
    with pytest.raises(gg.GGError):
        ctx.shuffle_payload(0, pay_g, off, 11)
    ctx.close()
