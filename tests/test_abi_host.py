"""Host-side checks of the C-ABI library that need no GPU: the shared object
loads, exports every symbol the header declares, validates arguments, and its
partner schedule (pure host code) equals the oracle's bit for bit."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_1803_05880_amd as gg
from oracle import schedule as sc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = "".join(open(os.path.join(ROOT, "include", h)).read() for h in sorted(os.listdir(os.path.join(ROOT, "include")))
                   if h.endswith(".h"))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gg_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_functions()
    assert {"gg_init", "gg_destroy", "gg_partner", "gg_gossip_step", "gg_shuffle", "gg_allreduce_baseline",
            "gg_sgd_step", "gg_strerror"} <= set(names)
    raw = ctypes.CDLL(gg.LIB_PATH)
    for name in names:
        assert hasattr(raw, name), name


def test_config_struct_layout_matches_header():
    # the header's field order and widths: 2x int32, 2x int64, 4x int32, uint64, 2x float
    assert ctypes.sizeof(gg.GGConfig) == 56
    assert gg.GGConfig.n.offset == 8 and gg.GGConfig.rank_stride.offset == 16
    assert gg.GGConfig.seed.offset == 40 and gg.GGConfig.lr.offset == 48 and gg.GGConfig.momentum.offset == 52


@pytest.mark.parametrize("topology", [gg.TOPO_HYPERCUBE, gg.TOPO_DISSEMINATION])
@pytest.mark.parametrize("p", [2, 4, 8, 16, 64, 128])
def test_partner_tables_bit_exact_over_a_full_rotation_cycle(p, topology):
    seed = 1234567 + p
    ctx = gg.Context(p=p, n=16, seed=seed, topology=topology)
    L = sc.num_phases(p)
    steps = list(range(p * L + L)) if p <= 64 else list(range(0, p * L + L, 3))
    for t in steps:
        send, recv = ctx.partner(t)
        o_send, o_recv = sc.partners(p, seed, p, topology, t)
        assert send.dtype == np.int32 and send.tolist() == o_send and recv.tolist() == o_recv
    ctx.close()


@pytest.mark.parametrize("p", [3, 5, 6, 12, 100, 1000])
def test_dissemination_any_p_and_num_comms(p):
    for R in (1, 3):
        ctx = gg.Context(p=p, n=1, seed=9, topology=gg.TOPO_DISSEMINATION, num_comms=R)
        for t in [0, 1, 2, 5, 11, 12, 40, 2**40 + 1]:
            send, recv = ctx.partner(t)
            o_send, o_recv = sc.partners(p, 9, R, sc.DISSEMINATION, t)
            assert send.tolist() == o_send and recv.tolist() == o_recv
        ctx.close()


def test_seed_uses_both_key_words():
    a = gg.Context(p=32, n=1, seed=5).partner(5 * 7)[0]
    b = gg.Context(p=32, n=1, seed=5 + (1 << 32)).partner(5 * 7)[0]
    o = sc.partners(32, 5 + (1 << 32), 32, sc.HYPERCUBE, 35)[0]
    assert a.tolist() != b.tolist() and b.tolist() == o


def _init_code(**kw):
    base = dict(p=4, topology=0, n=8, rank_stride=8, num_comms=0, avg_mode=0, staleness=0, reserved=0, seed=0,
                lr=0.1, momentum=0.9)
    base.update(kw)
    cfg = gg.GGConfig(**base)
    h = ctypes.c_void_p()
    code = gg.lib().gg_init(ctypes.byref(cfg), ctypes.byref(h))
    if code == 0:
        gg.lib().gg_destroy(h)
    else:
        assert not h.value                      # nothing written on error
    return code


def test_init_argument_validation():
    assert _init_code() == 0
    assert _init_code(p=1) == gg.binding.GG_ERR_ARG
    assert _init_code(p=gg.MAX_RANKS + 1, topology=1) == gg.binding.GG_ERR_ARG
    assert _init_code(p=6) == gg.binding.GG_ERR_NOT_POW2
    assert _init_code(p=6, topology=1) == 0
    assert _init_code(n=-1) == gg.binding.GG_ERR_ARG
    assert _init_code(rank_stride=7) == gg.binding.GG_ERR_ARG
    assert _init_code(topology=2) == gg.binding.GG_ERR_ARG
    assert _init_code(avg_mode=3) == gg.binding.GG_ERR_ARG
    assert _init_code(staleness=2) == gg.binding.GG_ERR_ARG
    assert _init_code(staleness=1, avg_mode=1) == gg.binding.GG_ERR_ARG
    assert _init_code(num_comms=-1) == gg.binding.GG_ERR_ARG
    assert _init_code(num_comms=4097) == gg.binding.GG_ERR_ARG
    assert _init_code(reserved=1) == gg.binding.GG_ERR_ARG
    assert _init_code(lr=float("nan")) == gg.binding.GG_ERR_ARG
    assert gg.lib().gg_init(None, None) == gg.binding.GG_ERR_ARG


def test_partner_argument_validation_and_strerror():
    ctx = gg.Context(p=4, n=8)
    buf = np.zeros(4, np.int32)
    ptr = buf.ctypes.data_as(ctypes.c_void_p)
    L = gg.lib()
    assert L.gg_partner(ctx._h, -1, ptr, None) == gg.binding.GG_ERR_ARG
    assert L.gg_partner(ctx._h, 0, None, None) == gg.binding.GG_ERR_ARG
    assert L.gg_partner(None, 0, ptr, None) == gg.binding.GG_ERR_ARG
    assert L.gg_partner(ctx._h, 0, ptr, None) == 0 and buf.tolist() == [1, 0, 3, 2]
    assert L.gg_set_tuning(ctx._h, 0, 100) == gg.binding.GG_ERR_ARG
    assert L.gg_set_tuning(ctx._h, 1, 3) == gg.binding.GG_ERR_ARG
    assert L.gg_set_tuning(ctx._h, 10, 0) == gg.binding.GG_ERR_ARG       # no such key
    assert L.gg_set_tuning(ctx._h, 1, 4) == 0
    for code in range(-7, 1):
        assert L.gg_strerror(code)
    assert L.gg_strerror(0) == b"ok"
    ctx.close()


def test_compute_entry_points_fail_loudly_without_a_gpu():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    ctx = gg.Context(p=4, n=8)
    dummy = ctypes.c_void_p(256)                 # never dereferenced: the device check comes first
    L = gg.lib()
    assert L.gg_gossip_step(ctx._h, 0, dummy, ctypes.c_void_p(512), ctypes.c_void_p(768), None, None, 0,
                            None) == gg.binding.GG_ERR_HIP
    assert L.gg_sgd_step(ctx._h, dummy, ctypes.c_void_p(512), ctypes.c_void_p(768), None) == gg.binding.GG_ERR_HIP
    assert L.gg_allreduce_baseline(ctx._h, dummy, 1, None) == gg.binding.GG_ERR_HIP
    off = np.array([0, 2, 4, 6, 8], np.int64)
    assert L.gg_shuffle(ctx._h, 0, 0, dummy, off.ctypes.data_as(ctypes.c_void_p), 0, None) == gg.binding.GG_ERR_HIP
    with pytest.raises(TypeError):
        ctx.sgd_step(torch.zeros(32), torch.zeros(32), torch.zeros(32))   # CPU tensors are refused
    ctx.close()


def test_probe_entry_points_validate_arguments():
    L = gg.lib()
    E = gg.binding
    assert L.gg_copy_probe(None, ctypes.c_void_p(256), 16, None) == E.GG_ERR_ARG
    assert L.gg_copy_probe(ctypes.c_void_p(256), ctypes.c_void_p(512), 24, None) == E.GG_ERR_ARG
    assert L.gg_copy_probe(ctypes.c_void_p(260), ctypes.c_void_p(512), 16, None) == E.GG_ERR_ALIGN
    assert L.gg_copy_probe(ctypes.c_void_p(256), ctypes.c_void_p(512), 0, None) == 0
    assert L.gg_busy_probe(10, 0, ctypes.c_void_p(256), None) == E.GG_ERR_ARG
    assert L.gg_busy_probe(-1, 4, ctypes.c_void_p(256), None) == E.GG_ERR_ARG
    assert L.gg_busy_probe(10, 4, None, None) == E.GG_ERR_ARG
    ctx = gg.Context(p=4, n=8)
    assert L.gg_stream_probe(10, 4, None, 16, None) == E.GG_ERR_ARG
    assert L.gg_stream_probe(10, 0, ctypes.c_void_p(256), 16, None) == E.GG_ERR_ARG
    assert L.gg_stream_probe(10, 4, ctypes.c_void_p(256), 24, None) == E.GG_ERR_ARG
    assert L.gg_stream_probe(10, 4, ctypes.c_void_p(260), 16, None) == E.GG_ERR_ALIGN
    assert L.gg_stream_probe(10, 4, ctypes.c_void_p(256), 0, None) == 0
    assert len(L.gg_build_id()) == 64
    assert L.gg_set_tuning(ctx._h, E.TUNE_WALK_CHUNKS, 3) == E.GG_ERR_ARG and L.gg_set_tuning(ctx._h, E.TUNE_WALK_CHUNKS, 0) == 0
    assert L.gg_set_tuning(ctx._h, E.TUNE_WALK_WAVES, 2) == 0
    assert L.gg_set_tuning(ctx._h, E.TUNE_WALK_CHUNKS, 8) == E.GG_ERR_ARG      # 8 chunks x 2 wavefronts > 8
    assert L.gg_set_tuning(ctx._h, E.TUNE_WALK_WAVES, 1) == 0 and L.gg_set_tuning(ctx._h, E.TUNE_WALK_CHUNKS, 8) == 0
    assert L.gg_set_tuning(ctx._h, E.TUNE_WALK_STEP, 0) == E.GG_ERR_ARG
    assert L.gg_set_tuning(ctx._h, 2, 2) == E.GG_ERR_ARG and L.gg_set_tuning(ctx._h, 2, 3) == 0
    off = np.array([0, 2, 4, 6, 8], np.int64).ctypes.data_as(ctypes.c_void_p)
    assert L.gg_shuffle_payload(ctx._h, 0, ctypes.c_void_p(256), 6, off, 1, None) == E.GG_ERR_ARG    # not a multiple of 4
    assert L.gg_shuffle_payload(ctx._h, 0, ctypes.c_void_p(256), 8, off, 3, None) == E.GG_ERR_ARG    # batch > min n_j
    assert L.gg_shuffle_payload(ctx._h, -1, ctypes.c_void_p(256), 8, off, 1, None) == E.GG_ERR_ARG
    ctx.close()


def test_partner_matches_oracle_on_random_configurations():
    from hypothesis import given, settings, strategies as st

    @settings(max_examples=60, deadline=None)
    @given(st.integers(2, 200), st.integers(0, 2**64 - 1), st.integers(0, 10**12), st.integers(1, 7),
           st.sampled_from([gg.TOPO_HYPERCUBE, gg.TOPO_DISSEMINATION]))
    def check(p, seed, step, num_comms, topology):
        if topology == gg.TOPO_HYPERCUBE:
            p = 1 << max(1, p.bit_length() % 8)
        ctx = gg.Context(p=p, n=1, seed=seed, topology=topology, num_comms=num_comms)
        send, recv = ctx.partner(step)
        o_send, o_recv = sc.partners(p, seed, num_comms, topology, step)
        ctx.close()
        assert send.tolist() == o_send and recv.tolist() == o_recv

    check()


def test_aligned_stride_helper():
    assert gg.aligned_stride(25_557_032) == 25_558_016 and gg.aligned_stride(1024) == 1024 and gg.aligned_stride(1) == 1024
    assert gg.aligned_stride(25_557_032, 64) == 25_557_056
