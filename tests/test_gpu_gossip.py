"""GPU parity: gg_gossip_step / gg_sgd_step against the CPU oracle, element by
element, through the C ABI (Eq. 1-2, Sec. 4.3-4.5.1, Sec. 6)."""
import numpy as np
import pytest
import torch

import gg_synth
import paper_1803_05880_amd as gg
from oracle import gossip as og
from oracle import schedule as sc
from parity_util import assert_close_fp32, host_state, oracle_run

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _run_gpu(W, G, M, n, stride, p, seed, steps, first_step=0, double_buffer=False, seg=None, tune=None, **cfg):
    ctx = gg.Context(p=p, n=n, rank_stride=stride, seed=seed, lr=gg_synth.LR, momentum=gg_synth.MOMENTUM, **cfg)
    for key, val in (tune.items() if isinstance(tune, dict) else tune or ()):
        ctx.set_tuning(key, val)
    w, g, m = W.to(DEV), G.to(DEV), M.to(DEV)
    w2 = torch.full_like(w, float("nan")) if double_buffer else None
    if double_buffer:
        w2[:, n:] = w[:, n:]                           # the second buffer's padding must stay as it is, too
    for t in range(first_step, first_step + steps):
        if double_buffer:
            ctx.gossip_step(t, w, g, m, w_next=w2, seg_offsets=seg)
            w, w2 = w2, w
        else:
            ctx.gossip_step(t, w, g, m, seg_offsets=seg)
    torch.cuda.synchronize()
    assert torch.equal(g.cpu(), G)                     # gradients are never written
    out = w.cpu(), m.cpu()
    ctx.close()
    return out


def _check(p, n, stride, steps, seed=0, first_step=0, double_buffer=False, tune=None, **cfg):
    W, G, M = host_state(p, n, stride, seed=seed)
    if stride > n:                                     # padding must never be touched
        W[:, n:] = 7.0
        M[:, n:] = -7.0
    wg, mg = _run_gpu(W, G, M, n, stride, p, seed, steps, first_step, double_buffer, tune=tune, **cfg)
    Wo, Mo = oracle_run(W, G, M, n, p, seed, steps, topology=cfg.get("topology", 0),
                        num_comms=cfg.get("num_comms", 0), avg_mode=cfg.get("avg_mode", 0),
                        staleness=cfg.get("staleness", 0), first_step=first_step)
    dw = assert_close_fp32(wg[:, :n].numpy(), Wo, "W")
    dm = assert_close_fp32(mg[:, :n].numpy(), Mo, "M")
    assert dw == 0 and dm == 0, "bit differences: W %d, M %d" % (dw, dm)
    if stride > n:
        assert (wg[:, n:] == 7.0).all() and (mg[:, n:] == -7.0).all()


def test_config1_tiny_gossip_full_parity():
    # p=4, N=1,048,576, 8 steps with rotating partners, seed 0
    _check(4, 1_048_576, 1_048_576, 8)


@pytest.mark.parametrize("num_comms", [1, 0])
def test_config2_googlenet_sized_full_parity(num_comms):
    # p=8, N=6,800,000, 3*log2(p) = 9 steps; without rotation partners recur exactly
    _check(8, gg_synth.GOOGLENET_PARAMS, gg_synth.GOOGLENET_PARAMS, 9, num_comms=num_comms)


@pytest.mark.parametrize("p,n,stride", [
    (2, 1, 1), (2, 3, 3), (2, 5, 8), (4, 4, 4), (4, 1023, 1024), (4, 100_003, 100_003),
    (8, 262_144 + 7, 262_144 + 8), (16, 70_001, 70_004), (32, 4099, 4100), (2, 2_000_003, 2_000_004),
])
def test_ragged_sizes_strides_and_tails(p, n, stride):
    # several tiles plus a ragged tail; odd strides force the scalar path
    _check(p, n, stride, 2 * sc.num_phases(p) + 1, seed=3)


def test_empty_buffers_are_a_no_op():
    ctx = gg.Context(p=4, n=0, rank_stride=4)
    w = torch.ones(4, 4, device=DEV); g = torch.ones(4, 4, device=DEV) * 2; m = torch.ones(4, 4, device=DEV) * 3
    ctx.gossip_step(0, w, g, m)
    torch.cuda.synchronize()
    assert (w == 1).all() and (m == 3).all()
    ctx.close()


@pytest.mark.parametrize("mode", [
    dict(staleness=1), dict(staleness=1, double_buffer=True), dict(avg_mode=gg.AVG_GRAD),
    dict(avg_mode=gg.AVG_NONE), dict(double_buffer=True),
])
@pytest.mark.parametrize("p,n,stride", [(8, 300_007, 300_008), (2, 65_536, 65_536), (16, 9_999, 9_999)])
def test_variants_hypercube(mode, p, n, stride):
    _check(p, n, stride, 2 * sc.num_phases(p) + 2, seed=5, **mode)


@pytest.mark.parametrize("mode", [dict(), dict(staleness=1), dict(avg_mode=gg.AVG_GRAD),
                                  dict(staleness=1, double_buffer=True), dict(double_buffer=True)])
@pytest.mark.parametrize("p,n,stride", [(8, 300_007, 300_008), (6, 50_001, 50_004), (5, 4097, 4097), (2, 1000, 1000),
                                        (16, 33_000, 33_000), (3, 70_000, 70_000)])
def test_dissemination_data_path(mode, p, n, stride):
    _check(p, n, stride, 2 * sc.num_phases(p) + 2, seed=6, topology=gg.TOPO_DISSEMINATION, **mode)


WALK_SHAPES = [
    # chunks per thread, wavefronts per workgroup, tile step, workgroups per CU, barrier per hop
    (2, 2, 32, 3, 1), (1, 8, 32, 3, 1), (8, 1, 32, 0, 0), (4, 2, 16, 4, 1), (1, 1, 1, 0, 0), (2, 4, 3, 7, 0),
    (4, 1, 64, 3, 1), (1, 4, 4096, 3, 1), (0, 2, 32, 3, 1),
]


@pytest.mark.parametrize("shape", WALK_SHAPES)
@pytest.mark.parametrize("mode", [dict(), dict(staleness=1), dict(avg_mode=gg.AVG_GRAD),
                                  dict(staleness=1, double_buffer=True), dict(double_buffer=True)])
@pytest.mark.parametrize("p,n,stride", [(64, 70_003, 70_004), (12, 5_001, 5_001), (7, 3_000, 3_000), (6, 300_007, 300_008)])
def test_dissemination_walk_shapes_never_change_results(shape, mode, p, n, stride):
    # the workgroup shape of the cycle walk (chunks, wavefronts, tile step, occupancy cap, hop barrier) and the
    # general kernel (chunks = 0) give the same bits
    chunks, waves, step, cap, barrier = shape
    tune = [(gg.TUNE_WALK_CHUNKS, 1), (gg.TUNE_WALK_WAVES, waves), (gg.TUNE_WALK_CHUNKS, chunks),
            (gg.TUNE_WALK_STEP, step), (gg.TUNE_WALK_WG_PER_CU, cap), (gg.TUNE_WALK_BARRIER, barrier)]
    _check(p, n, stride, sc.num_phases(p) + 2, seed=26, topology=gg.TOPO_DISSEMINATION, tune=tune, **mode)


@pytest.mark.parametrize("tune", [
    {gg.TUNE_THREADS: 64, gg.TUNE_CHUNKS: 1}, {gg.TUNE_THREADS: 128, gg.TUNE_CHUNKS: 4},
    {gg.TUNE_THREADS: 256, gg.TUNE_CHUNKS: 8}, {gg.TUNE_BLOCKS_PER_CU: 0, gg.TUNE_CHUNKS: 2}, {gg.TUNE_BLOCKS_PER_CU: 3},
    {gg.TUNE_BLOCKS_PER_CU: 8, gg.TUNE_CHUNKS: 4},
    {gg.TUNE_NONTEMPORAL: 0},
])
def test_launch_shapes_never_change_results(tune):
    _check(8, 1_500_003, 1_500_004, 4, seed=7, tune=tune)
    _check(8, 200_001, 200_004, 3, seed=7, tune=tune, topology=gg.TOPO_DISSEMINATION)


@pytest.mark.parametrize("topology,p", [(gg.TOPO_HYPERCUBE, 1024), (gg.TOPO_DISSEMINATION, 1024),
                                        (gg.TOPO_DISSEMINATION, 1000)])
def test_maximum_rank_count(topology, p):
    # GG_MAX_RANKS virtual ranks: full pair table / longest cycles, a rotated communicator included
    _check(p, 1_027, 1_028, 3, seed=17, first_step=sc.num_phases(p) - 1, topology=topology)


def test_late_steps_and_rotation_wrap():
    p = 8
    L = 3
    _check(p, 10_000, 10_000, 4, seed=8, first_step=p * L - 2)          # crosses the wrap to communicator 0
    _check(p, 10_000, 10_000, 2, seed=8, first_step=(1 << 40) + 5)


def test_segments_cut_the_same_range_identically_and_leave_the_rest():
    p, n = 4, 200_000
    W, G, M = host_state(p, n, n, seed=9)
    lo, hi = 1_001, 150_003
    cuts = np.array([lo, 1_002, 5_000, 5_000, 77_777, hi], dtype=np.int64)      # includes an empty segment
    w_a, m_a = _run_gpu(W, G, M, n, n, p, 9, 3, seg=cuts)
    w_b, m_b = _run_gpu(W, G, M, n, n, p, 9, 3, seg=np.array([lo, hi], dtype=np.int64))
    assert torch.equal(w_a, w_b) and torch.equal(m_a, m_b)
    assert torch.equal(w_a[:, :lo], W[:, :lo]) and torch.equal(w_a[:, hi:], W[:, hi:])
    assert torch.equal(m_a[:, :lo], M[:, :lo]) and torch.equal(m_a[:, hi:], M[:, hi:])
    Wo, Mo = oracle_run(W[:, lo:hi], G[:, lo:hi], M[:, lo:hi], hi - lo, p, 9, 3)
    assert np.array_equal(w_a[:, lo:hi].numpy(), Wo) and np.array_equal(m_a[:, lo:hi].numpy(), Mo)
    # whole-range segment table == no table
    off, _ = gg_synth.segment_layout(n, 161, seed=1)
    w_c, m_c = _run_gpu(W, G, M, n, n, p, 9, 3, seg=off)
    w_d, m_d = _run_gpu(W, G, M, n, n, p, 9, 3)
    assert torch.equal(w_c, w_d) and torch.equal(m_c, m_d)


def test_sgd_step_and_unaligned_base_pointers():
    p, n, stride = 4, 50_001, 50_004
    W, G, M = host_state(p, n, stride, seed=10)
    M.normal_(0, 1e-3, generator=torch.Generator().manual_seed(1))
    ctx = gg.Context(p=p, n=n, rank_stride=stride, lr=0.1, momentum=0.9)
    # shift every buffer by one float so that no base address is 16-byte aligned
    bufs = []
    for t in (W, G, M):
        raw = torch.zeros(p * stride + 1, device=DEV)
        view = raw[1:].view(p, stride)
        view.copy_(t)
        bufs.append(view)
    w, g, m = bufs
    ctx.sgd_step(w, g, m)
    ctx.gossip_step(1, w, g, m)
    torch.cuda.synchronize()
    Wo, Go, Mo = W[:, :n].numpy().copy(), G[:, :n].numpy().copy(), M[:, :n].numpy().copy()
    og.sgd_step(Wo, Go, Mo, 0.1, 0.9)
    og.gossip_step(Wo, Go, Mo, sc.partners(p, 0, p, 0, 1)[1], 0.1, 0.9)
    assert np.array_equal(w.cpu()[:, :n].numpy(), Wo) and np.array_equal(m.cpu()[:, :n].numpy(), Mo)
    ctx.close()


def test_denormals_and_specials_survive():
    p, n = 2, 64
    W = torch.zeros(p, n); G = torch.zeros(p, n); M = torch.zeros(p, n)
    W[0, :8] = torch.tensor([1e-40, -1e-40, 1e-45, 3e-39, 0.0, -0.0, 1e38, -1e38])
    W[1, :8] = torch.tensor([1e-40, 2e-40, 0.0, -1e-39, 1e-45, 0.0, 3e38, 1e38])
    G[0, :8] = 1e-39
    M[1, :8] = 2e-39
    wg, mg = _run_gpu(W, G, M, n, n, p, 0, 1)
    Wo, Mo = oracle_run(W, G, M, n, p, 0, 1)
    with np.errstate(all="ignore"):
        assert np.array_equal(wg.numpy().view(np.uint32), Wo.view(np.uint32))
        assert np.array_equal(mg.numpy().view(np.uint32), Mo.view(np.uint32))
    assert (np.abs(Mo[np.nonzero(Mo)]) < 1e-37).all() and np.count_nonzero(Mo) > 0   # denormals were exercised


def test_argument_errors_on_device():
    import ctypes
    ctx = gg.Context(p=4, n=64)
    w = torch.zeros(4, 64, device=DEV); g = torch.zeros(4, 64, device=DEV); m = torch.zeros(4, 64, device=DEV)
    L = gg.lib()
    P = lambda t: ctypes.c_void_p(t.data_ptr())
    E = gg.binding
    assert L.gg_gossip_step(ctx._h, -1, P(w), P(g), P(m), None, None, 0, None) == E.GG_ERR_ARG
    assert L.gg_gossip_step(ctx._h, 0, None, P(g), P(m), None, None, 0, None) == E.GG_ERR_ARG
    assert L.gg_gossip_step(ctx._h, 0, P(w), P(g), P(w), None, None, 0, None) == E.GG_ERR_ARG
    assert L.gg_gossip_step(ctx._h, 0, P(w), P(g), P(m), P(w), None, 0, None) == E.GG_ERR_ARG
    assert L.gg_gossip_step(ctx._h, 0, ctypes.c_void_p(w.data_ptr() + 2), P(g), P(m), None, None, 0, None) == E.GG_ERR_ALIGN
    bad = np.array([0, 65], np.int64)
    assert L.gg_gossip_step(ctx._h, 0, P(w), P(g), P(m), None, bad.ctypes.data_as(ctypes.c_void_p), 1, None) == E.GG_ERR_ARG
    bad = np.array([10, 5], np.int64)
    assert L.gg_gossip_step(ctx._h, 0, P(w), P(g), P(m), None, bad.ctypes.data_as(ctypes.c_void_p), 1, None) == E.GG_ERR_ARG
    assert L.gg_gossip_step(ctx._h, 0, P(w), P(g), P(m), None, None, 1, None) == E.GG_ERR_ARG
    torch.cuda.synchronize()
    assert (w == 0).all() and (m == 0).all()
    ctx.close()


def test_calls_follow_the_stream_they_are_given():
    # steps issued on two user streams chained by events must equal the single-stream run
    p, n = 8, 400_000
    W, G, M = host_state(p, n, n, seed=18)
    ref_w, ref_m = _run_gpu(W, G, M, n, n, p, 18, 6)
    ctx = gg.Context(p=p, n=n, rank_stride=n, seed=18, lr=gg_synth.LR, momentum=gg_synth.MOMENTUM)
    w, g, m = W.to(DEV), G.to(DEV), M.to(DEV)
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    prev = None
    for t in range(6):
        s = streams[t & 1]
        if prev is not None:
            s.wait_event(prev)
        ctx.gossip_step(t, w, g, m, stream=s)
        prev = torch.cuda.Event()
        prev.record(s)
    torch.cuda.synchronize()
    assert torch.equal(w.cpu(), ref_w) and torch.equal(m.cpu(), ref_m)
    ctx.close()


def test_repeated_calls_are_deterministic():
    p, n = 16, 123_457
    W, G, M = host_state(p, n, n + 3, seed=19)
    a = _run_gpu(W, G, M, n, n + 3, p, 19, 5)
    b = _run_gpu(W, G, M, n, n + 3, p, 19, 5)
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])


@pytest.mark.parametrize("topology,p,step", [(gg.TOPO_HYPERCUBE, 8, 4), (gg.TOPO_DISSEMINATION, 8, 3),
                                             (gg.TOPO_DISSEMINATION, 48, 0)])
def test_step_can_be_captured_in_a_graph_and_replayed(topology, p, step):
    # the call only enqueues kernels (no allocation, no host state) -- also the very first call of a
    # context, also a dissemination phase with one long partner cycle: a captured step replays to the
    # same bits as eager calls of the same step, replay after replay
    n = 300_003
    stride = n + 1
    W, G, M = host_state(p, n, stride, seed=20)
    w, g, m = W.to(DEV), G.to(DEV), M.to(DEV)
    we, me = W.to(DEV), M.to(DEV)
    ctx = gg.Context(p=p, n=n, rank_stride=stride, seed=20, lr=gg_synth.LR, momentum=gg_synth.MOMENTUM,
                     topology=topology)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        ctx.gossip_step(step, w, g, m)                   # the context's first call is the captured one
    torch.cuda.synchronize()
    assert torch.equal(w.cpu(), W) and torch.equal(m.cpu(), M)      # capture does not execute
    for replay in range(3):
        graph.replay()
        ctx.gossip_step(step, we, g, me)
        torch.cuda.synchronize()
        assert torch.equal(w, we) and torch.equal(m, me), "replay %d" % replay
    ctx.close()


def test_resume_with_a_fresh_context_continues_bit_exactly():
    # the library keeps no step counter: a new context with the same seed resumes at any step
    p, n = 8, 150_000
    W, G, M = host_state(p, n, n, seed=21)
    full_w, full_m = _run_gpu(W, G, M, n, n, p, 21, 7)
    half_w, half_m = _run_gpu(W, G, M, n, n, p, 21, 3)
    res_w, res_m = _run_gpu(half_w, G, half_m, n, n, p, 21, 4, first_step=3)
    assert torch.equal(res_w, full_w) and torch.equal(res_m, full_m)


def test_learning_rate_schedule_through_set_hyper():
    # lr drops by 10x after two steps (the paper's step schedule in miniature)
    p, n = 4, 100_000
    W, G, M = host_state(p, n, n, seed=22)
    ctx = gg.Context(p=p, n=n, rank_stride=n, seed=22, lr=0.1, momentum=0.9)
    w, g, m = W.to(DEV), G.to(DEV), M.to(DEV)
    Wo, Go, Mo = W.numpy().copy(), G.numpy().copy(), M.numpy().copy()
    for t in range(5):
        lr = 0.1 if t < 2 else 0.01
        ctx.set_hyper(lr, 0.9)
        ctx.gossip_step(t, w, g, m)
        og.gossip_step(Wo, Go, Mo, sc.partners(p, 22, p, 0, t)[1], lr, 0.9)
    torch.cuda.synchronize()
    assert np.array_equal(w.cpu().numpy(), Wo) and np.array_equal(m.cpu().numpy(), Mo)
    with pytest.raises(gg.GGError):
        ctx.set_hyper(float("nan"), 0.9)
    ctx.close()


def test_infinities_and_nans_propagate_like_the_oracle():
    p, n = 2, 64
    W = torch.zeros(p, n); G = torch.zeros(p, n); M = torch.zeros(p, n)
    W[0, :6] = torch.tensor([float("inf"), float("-inf"), float("inf"), float("nan"), 1.0, 3e38])
    W[1, :6] = torch.tensor([1.0, 2.0, float("-inf"), 5.0, float("nan"), 3e38])
    G[0, 6] = float("inf"); M[1, 7] = float("nan")
    wg, mg = _run_gpu(W, G, M, n, n, p, 0, 1)
    with np.errstate(all="ignore"):
        Wo, Mo = oracle_run(W, G, M, n, p, 0, 1)
    for got, exp in ((wg.numpy(), Wo), (mg.numpy(), Mo)):
        assert np.array_equal(np.isnan(got), np.isnan(exp))
        ok = ~np.isnan(exp)
        assert np.array_equal(got[ok], exp[ok])          # infinities and finite values bit for bit
    assert np.isnan(Wo).sum() >= 4 and np.isinf(Wo).sum() >= 2
