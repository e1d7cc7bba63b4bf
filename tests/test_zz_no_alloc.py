"""GPU test of gg_shuffle_noalloc, the entry point for callers that cannot allocate:
its output must equal gg_shuffle's bit for bit, on calls in a row that share the
library's one fixed scratch array, the later ones with smaller inputs."""
import numpy as np
import pytest
import torch

import gg_synth
import paper_1803_05880_amd as gg

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _both(ctx, step, mode, n_total, off, batch=0):
    """Run the allocating and the non-allocating entry point on equal inputs; return both results."""
    rng = torch.Generator(device="cpu").manual_seed(n_total + step)
    ids = torch.randperm(n_total, generator=rng, dtype=torch.int64).to(torch.int32)
    a, b = ids.to(DEV), ids.to(DEV)
    ctx.shuffle(step, mode, a, off, batch=batch)
    ctx.shuffle_noalloc(step, mode, b, off, batch=batch)
    torch.cuda.synchronize()
    return a.cpu().numpy(), b.cpu().numpy(), ids.numpy()


def test_noalloc_shuffle_equals_shuffle_on_calls_in_a_row():
    p = 128
    ctx = gg.Context(p=p, n=4, seed=3)
    # 1,281,167 ids (three-kernel path is not taken: 10,010 slots per rank), then far fewer, then uneven ranks
    sizes = [gg_synth.IMAGENET1K_TRAIN, 100_003, 5_000]
    for call, n_total in enumerate(sizes):
        off = gg_synth.block_offsets(n_total, p)
        want, got, before = _both(ctx, 7 + call, gg.SHUF_PARTNER_SWAP, n_total, off)
        assert np.array_equal(got, want), "partner swap, call %d" % call
        assert not np.array_equal(got, before) and np.array_equal(np.sort(got), np.sort(before))
    for call, (n_total, batch) in enumerate([(200_000, 1_000), (9_001, 70)]):
        off = gg_synth.block_offsets(n_total, p)
        want, got, before = _both(ctx, 11 + call, gg.SHUF_RING, n_total, off, batch=batch)
        assert np.array_equal(got, want), "ring, call %d" % call
        assert not np.array_equal(got, before)
    ctx.close()


def test_noalloc_shuffle_many_tiles_per_rank_then_smaller():
    # few ranks holding many tiles each take the count / scatter / apply kernels and the per-tile counts
    p = 4
    ctx = gg.Context(p=p, n=4, seed=5)
    for call, n_total in enumerate([gg_synth.IMAGENET1K_TRAIN, 300_001, 40_000]):
        off = np.array([0, n_total // 2, n_total // 2 + 17, n_total - 5, n_total], dtype=np.int64)   # uneven ranks
        want, got, before = _both(ctx, call, gg.SHUF_PARTNER_SWAP, n_total, off)
        assert np.array_equal(got, want), "call %d" % call
        assert np.array_equal(np.sort(got), np.sort(before))
    ctx.close()


def test_noalloc_shuffle_rejects_what_does_not_fit_and_leaves_the_indices_alone():
    p = 4
    ctx = gg.Context(p=p, n=4)
    n_total = gg.binding.NOALLOC_MAX_INDICES + 1
    idx = gg_synth.make_indices(n_total, DEV)
    with pytest.raises(gg.GGError) as e:
        ctx.shuffle_noalloc(0, gg.SHUF_PARTNER_SWAP, idx, gg_synth.block_offsets(n_total, p))
    assert e.value.code == gg.binding.GG_ERR_LIMIT
    torch.cuda.synchronize()
    assert torch.equal(idx, gg_synth.make_indices(n_total, DEV))
    ctx.shuffle_noalloc(0, gg.SHUF_PARTNER_SWAP, idx[:gg.binding.NOALLOC_MAX_INDICES],
                        gg_synth.block_offsets(gg.binding.NOALLOC_MAX_INDICES, p))      # the maximum itself fits
    torch.cuda.synchronize()
    assert torch.equal(torch.sort(idx[:gg.binding.NOALLOC_MAX_INDICES]).values,
                       gg_synth.make_indices(gg.binding.NOALLOC_MAX_INDICES, DEV))
    ctx.close()
    # too many (rank, tile) counters: 1024 ranks, one of them with 65 tiles
    ctx = gg.Context(p=1024, n=4)
    off = np.concatenate([[0], np.cumsum([65 * 4096] + [1] * 1023)]).astype(np.int64)
    idx = gg_synth.make_indices(int(off[-1]), DEV)
    with pytest.raises(gg.GGError) as e:
        ctx.shuffle_noalloc(0, gg.SHUF_PARTNER_SWAP, idx, off)
    assert e.value.code == gg.binding.GG_ERR_LIMIT
    ctx.close()


def test_noalloc_shuffle_under_graph_capture_replays():
    # the use the entry point exists for: captured once, replayed with eager work in between
    p, n_total = 16, 50_000
    off = gg_synth.block_offsets(n_total, p)
    ctx = gg.Context(p=p, n=4, seed=9)
    ids = gg_synth.make_indices(n_total, DEV)
    ref = ids.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        ctx.shuffle_noalloc(0, gg.SHUF_PARTNER_SWAP, ids, off, stream=side)           # warm-up outside capture
        side.synchronize()
        ids.copy_(ref)
        with torch.cuda.graph(graph, stream=side):
            ctx.shuffle_noalloc(0, gg.SHUF_PARTNER_SWAP, ids, off, stream=torch.cuda.current_stream())
    torch.cuda.synchronize()
    for replay in range(3):
        graph.replay()
        torch.cuda.synchronize()
        ctx.shuffle(0, gg.SHUF_PARTNER_SWAP, ref, off)                                   # eager, allocating path
        torch.cuda.synchronize()
        assert torch.equal(ids, ref), "replay %d" % replay
    ctx.close()
