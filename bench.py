#!/usr/bin/env python3
"""Benchmark of the GossipGraD hot path on one MI355X.

One "step" is one pass of the whole hot path for all p virtual ranks: the
partner schedule lookup, the fused momentum-SGD update + pairwise model average
(one launch) and the partner-swap shuffle of the sample indices (on a second
stream, beside the update).
Inputs are synthetic and resident in HBM before the timed region starts.

Workload (default): p = 64 virtual ranks x N = 25,557,032 fp32 parameters
(ResNet50-sized; w, g, m = 19.6 GB), hypercube partners with rotation,
synchronous model averaging, plus 1,281,167 int32 sample ids block-partitioned
over the ranks.  The metric is effective HBM GB/s with the algorithmic minimum
of 20 bytes per rank and parameter (read w, g, m; write w, m).

Prints ONE JSON line.  Also reported in it: the kernel's roofline fraction from
HIP events, the other workload shapes run one after another in the same process,
the staleness-1 double-buffer variant, the dissemination topology phase by
phase, the all-reduce comparators, the layer-wise exchange overlapped with a
stand-in computation, a plain copy kernel, and the CPU oracle timed at the
workload shapes that fit the host.
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
BYTES_PER_RANK_PARAM = 20      # read w, g, m + write w, m
SHUFFLE_N = 1_281_167
WORKLOADS = {
    "C1": dict(p=4, n=1_048_576, steps=8),
    "C2": dict(p=8, n=6_800_000, steps=9),
    "C3": dict(p=16, n=25_557_032, steps=32),
    "C4": dict(p=64, n=25_557_032, steps=64),
    "C5": dict(p=128, n=25_557_032, steps=128),
}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="C4", choices=sorted(WORKLOADS))
    ap.add_argument("--stride-align", type=int, default=1024,
                    help="rank_stride is N rounded up to a multiple of this many elements (layout choice)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="time only the headline step")
    ap.add_argument("--no-workloads", action="store_true", help="skip the other workload shapes")
    ap.add_argument("--threads", type=int, default=None)
    ap.add_argument("--chunks", type=int, default=None)
    ap.add_argument("--blocks-per-cu", type=int, default=None)
    ap.add_argument("--nontemporal", type=int, default=None)
    return ap.parse_args()


def event_ms(pairs):
    return [a.elapsed_time(b) for a, b in pairs]


def time_loop(torch, fn, steps, warmup):
    """Run fn(t) for warmup+steps steps; returns (wall ms/step, per-call event ms list)."""
    for t in range(warmup):
        fn(t, None)
    torch.cuda.synchronize()
    pairs = []
    t0 = time.perf_counter()
    for t in range(warmup, warmup + steps):
        fn(t, pairs)
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) * 1e3 / steps
    return wall, pairs


def pmc_traffic(workload, digest):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 counter
    summary -- only when that summary was taken from a library built from the very sources
    in this tree; otherwise (None, reason)."""
    path = os.path.join(ROOT, "profiles", "gossip_pair_kernel_%s_pmc.txt" % workload)
    try:
        text = open(path).read()
    except OSError:
        return None, "no counter summary for this workload under profiles/"
    m = re.search(r"^traffic_bytes_per_launch:\s*([0-9.eE+]+)", text, re.M)
    h = re.search(r"^library_source_sha256:\s*([0-9a-f]+)", text, re.M)
    if not m or not h:
        return None, "counter summary carries no traffic figure or no source digest"
    if h.group(1) != digest:
        return None, "counter summary was taken from other library sources (%s...)" % h.group(1)[:12]
    return float(m.group(1)), "profiles/" + os.path.basename(path)


def pair_kernel_name(args):
    """Name of the kernel gg_gossip_step launches for hypercube steps under the tuning in force
    (mirrors the library's choice: the lean kernel serves the default launch shape)."""
    threads = 64 if args.threads is None else args.threads
    chunks = 1 if args.chunks is None else args.chunks
    nt = "nontemporal" if (args.nontemporal is None or args.nontemporal) else "temporal"
    if threads == 64 and chunks == 1:
        return "gossip_pair_lean_kernel<MODE_SYNC, %s>" % nt
    return "gossip_pair_kernel<v4f, MODE_SYNC, %d chunks, %s> (%d threads)" % (chunks, nt, threads)


def _oracle_rate(p, n, steps, budget_s):
    """Oracle gossip steps at p x n (fresh draws of the workload's distributions), single
    thread; returns (GB/s by the 20-byte accounting, seconds per step, steps run)."""
    import numpy as np
    from oracle import gossip as og, schedule as sc
    rng = np.random.default_rng(0)
    W = np.empty((p, n), np.float32)
    G = np.empty((p, n), np.float32)
    for j in range(p):
        W[j] = rng.standard_normal(n, dtype=np.float32) * np.float32(0.05)
        G[j] = rng.standard_normal(n, dtype=np.float32) * np.float32(1e-3)
    M = np.zeros_like(W)
    t0 = time.perf_counter()
    done = 0
    while done < steps and (done < 1 or time.perf_counter() - t0 < budget_s):
        og.gossip_step(W, G, M, sc.partners(p, 0, p, sc.HYPERCUBE, done)[1], 0.1, 0.9)
        done += 1
    dt = (time.perf_counter() - t0) / done
    return BYTES_PER_RANK_PARAM * p * n / dt / 1e9, dt, done


def cpu_baseline(workload, p, n, lr, mu):
    """The oracle as it stands, timed on the host's cores beside the GPU figure.

    value: the bench workload's rate.  For C1-C3 that is the full shape.  C4 and C5 (19.6
    and 39.3 GB of state plus the oracle's temporaries) are timed at p = 16 ranks of the
    same N and scale linearly in p (the step is elementwise per pair), so their GB/s is
    the p = 16 figure, marked extrapolated.  Also: every other shape that fits, and the
    unchanged oracle run on column slices by one thread per core."""
    import concurrent.futures as cf
    import numpy as np
    from oracle import gossip as og, schedule as sc
    per = {}
    for name, budget in (("C1", 2.0), ("C2", 4.0), ("C3", 12.0)):
        w = WORKLOADS[name]
        gbs, dt, done = _oracle_rate(w["p"], w["n"], min(w["steps"], 6), budget)
        per[name] = {"GBps": round(gbs, 3), "s_per_step": round(dt, 4), "steps_timed": done, "shape": "full"}
    for name in ("C4", "C5"):
        w = WORKLOADS[name]
        per[name] = {"GBps": per["C3"]["GBps"], "s_per_step": round(per["C3"]["s_per_step"] * w["p"] / 16, 3),
                     "shape": "extrapolated: timed at p=16 ranks of the same N, linear in p"}

    # all host cores: the oracle unchanged, one column slice of a 1 Mi-parameter sample per thread
    n_s = 1_048_576
    rng = np.random.default_rng(0)
    W = rng.normal(0, 0.05, (p, n_s)).astype(np.float32)
    G = rng.normal(0, 1e-3, (p, n_s)).astype(np.float32)
    M = np.zeros_like(W)
    cores = max(1, min(os.cpu_count() or 1, 64))
    cuts = np.linspace(0, n_s, cores + 1).astype(np.int64)
    slices = [tuple(np.ascontiguousarray(a[:, cuts[i]:cuts[i + 1]]) for a in (W, G, M)) for i in range(cores)]
    pool = cf.ThreadPoolExecutor(cores)

    def threaded(t):
        c = sc.partners(p, 0, p, sc.HYPERCUBE, t)[1]
        list(pool.map(lambda s: og.gossip_step(s[0], s[1], s[2], c, lr, mu), slices))

    threaded(0)
    t0 = time.perf_counter()
    steps = 0
    while steps < 200 and (steps < 2 or time.perf_counter() - t0 < 4.0):
        steps += 1
        threaded(steps)
    dtc = (time.perf_counter() - t0) / steps
    pool.shutdown()
    mine = per[workload]
    return {
        "value": mine["GBps"],
        "unit": "GB/s",
        "cores": 1,
        "kind": "oracle",
        "sample": ("%s: oracle gossip step, numpy fp32, single thread, %s; %s s/step"
                   % (workload, mine["shape"] if mine["shape"] != "full" else
                      "full shape p=%d x N=%d, %d steps" % (p, n, mine["steps_timed"]), mine["s_per_step"])),
        "per_workload": per,
        "all_cores": {"value": round(BYTES_PER_RANK_PARAM * p * n_s / dtc / 1e9, 3), "unit": "GB/s", "cores": cores,
                      "sample": "p=%d x first %d params cut into %d column slices, one thread each, %d steps; %.3f s/step"
                                % (p, n_s, cores, steps, dtc)},
        "host_cpus": os.cpu_count(),
    }


def make_buckets(seg, n, target):
    """Group per-layer segments (ascending offsets seg[0..]) into buckets of at least
    `target` elements in back-propagation order (last layer first).  Returns [lo, hi)
    element ranges, highest first, that tile [0, n) exactly.  Cuts are moved up to
    256-byte boundaries: the few elements below a rounded-up cut belong to layers
    that are ready later, so they simply travel with the next bucket."""
    up = lambda x: n if x >= n else (int(x) + 63) // 64 * 64
    buckets, hi = [], len(seg) - 1
    while hi > 0:
        lo = hi
        while lo > 0 and seg[hi] - seg[lo] < target:
            lo -= 1
        b = (up(seg[lo]) if lo > 0 else 0, up(seg[hi]))
        if b[1] > b[0]:
            buckets.append(b)
        hi = lo
    return buckets


def pipelined_step(torch, ctx, step, W, G, M, buckets, main, side, compute_piece):
    """One layer-wise step (Sec. 5, 5.1): the stand-in computation runs piece by piece on
    the main stream; as soon as the piece that "produces" a bucket's gradients is done,
    that bucket's gossip update is enqueued on the side stream.  The main stream waits
    for the last bucket at the end (the paper's wait for all exchanges)."""
    for lo, hi in buckets:
        compute_piece()
        e = torch.cuda.Event()
        e.record(main)
        side.wait_event(e)
        ctx.gossip_step(step, W, G, M, seg_offsets=[lo, hi], stream=side)
    done = torch.cuda.Event()
    done.record(side)
    main.wait_event(done)


def layerwise_overlap(torch, gg, gg_synth, ctx, W, G, M, n, gossip_ms, scratch, reps=5):
    """Layer-wise exchange overlapped with computation (Sec. 5, 5.1): the buffer is cut
    into 161 per-layer segments, grouped into ~20 buckets in back-propagation order.
    Compute is sized 3.5x the exchange, the ratio the paper reports (96 ms vs 27 ms).
    Two stand-ins: an arithmetic-only kernel (the exchange has the memory system to
    itself: an upper bound on what can hide) and one that also streams memory."""
    seg, _ = gg_synth.segment_layout(n, 161, seed=0)
    buckets = make_buckets(seg, n, n // 24)
    main = torch.cuda.current_stream()
    side = torch.cuda.Stream()
    sink = torch.zeros(1, device=W.device)

    def timed(fn, k):
        fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(main)
        for _ in range(k):
            fn()
        b.record(main)
        torch.cuda.synchronize()
        return a.elapsed_time(b) / k

    step = [0]

    def gossip_only():
        for lo, hi_ in buckets:
            ctx.gossip_step(step[0], W, G, M, seg_offsets=[lo, hi_])
        step[0] += 1

    t_g = timed(gossip_only, reps)
    target_piece_ms = 3.5 * gossip_ms / len(buckets)
    out = {"buckets": len(buckets), "segments": 161, "gossip_bucketed_ms": round(t_g, 4)}

    def measure(piece):
        def compute_only():
            for _ in buckets:
                piece()

        def pipelined():
            pipelined_step(torch, ctx, step[0], W, G, M, buckets, main, side, piece)
            step[0] += 1

        t_c = timed(compute_only, reps)
        t_p = timed(pipelined, reps)
        return t_c, t_p, max(0.0, min(1.0, (t_c + t_g - t_p) / t_g))

    # (1) arithmetic only
    probe_iters = 100_000
    t_probe = timed(lambda: gg.busy_probe(probe_iters, 1024, sink), 3)
    iters = max(1, int(probe_iters * target_piece_ms / t_probe))
    t_c, t_p, hid = measure(lambda: gg.busy_probe(iters, 1024, sink))
    out.update({"compute_ms": round(t_c, 4), "pipelined_ms": round(t_p, 4), "exchange_hidden_fraction": round(hid, 4),
                "note": "arithmetic-only stand-in: the exchange has all of HBM to itself, an upper bound"})

    # (2) stand-ins that stream memory while they compute: each piece reads and rewrites a slab
    # of a scratch buffer sized for a stated share of the HBM peak over the piece's duration,
    # with the arithmetic per byte tuned so that the piece lasts as long as in (1).  Like (1)
    # it runs 1024 workgroups, so the exchange finds wavefront slots beside it.
    out["memory_streaming_compute"] = []
    for duty in (0.25, 0.5):
        slab_bytes = int(duty * HBM_PEAK_GBS * 1e9 * target_piece_ms * 1e-3 / 2) // 4096 * 4096
        slab_bytes = min(slab_bytes, scratch.numel() * 4 // 4096 * 4096)
        slab = scratch.view(-1)[: slab_bytes // 4]
        it2, piece_ms = 0, timed(lambda: gg.stream_probe(0, 1024, slab), 3)    # pure streaming time of one piece
        if piece_ms < target_piece_ms:
            it2 = 64
            for _ in range(8):                                   # arithmetic per chunk until the piece lasts long enough
                piece_ms = timed(lambda: gg.stream_probe(it2, 1024, slab), 3)
                if abs(piece_ms - target_piece_ms) < 0.02 * target_piece_ms:
                    break
                it2 = max(1, min(it2 * 4, int(it2 * target_piece_ms / piece_ms + 0.5)))
            piece_ms = timed(lambda: gg.stream_probe(it2, 1024, slab), 3)
        t_c2, t_p2, hid2 = measure(lambda: gg.stream_probe(it2, 1024, slab))
        out["memory_streaming_compute"].append({
            "target_share_of_hbm_peak": duty, "slab_MB": round(slab_bytes / 1e6, 1),
            "compute_GBps_alone": round(2.0 * slab_bytes / (piece_ms * 1e-3) / 1e9, 1),
            "compute_ms": round(t_c2, 4), "pipelined_ms": round(t_p2, 4), "exchange_hidden_fraction": round(hid2, 4),
        })
    return out


def other_workloads(torch, gg, gg_synth, skip, stride_align, lr, mu, dev):
    """The other workload shapes, one after another in this process: kernel time of the
    gossip step from events (hypercube, synchronous), GB/s by the 20-byte accounting.
    C1 and C2 fit the on-chip caches (flagged); C3 runs on its 161-segment table and
    beside it the recursive-doubling and one-pass all-reduce + SGD on the same buffers."""
    out = {}
    stream = torch.cuda.current_stream()
    for name in ("C1", "C2", "C3", "C4", "C5"):
        if name == skip:
            continue
        wl = WORKLOADS[name]
        p, n = wl["p"], wl["n"]
        stride = (n + stride_align - 1) // stride_align * stride_align
        seg = scales = None
        if name == "C3":
            seg, scales = gg_synth.segment_layout(n, 161, seed=0)
        W, G, M = gg_synth.make_state(p, n, stride, seed=0, device=dev, seg_offsets=seg, seg_scales=scales)
        ctx = gg.Context(p=p, n=n, rank_stride=stride, seed=0, lr=lr, momentum=mu)
        idx = off = None
        if name == "C5":
            off = gg_synth.block_offsets(SHUFFLE_N, p)
            idx = gg_synth.make_indices(SHUFFLE_N, dev)
            ctx.shuffle(0, gg.SHUF_PARTNER_SWAP, idx, off)
        side = torch.cuda.Stream()

        def step(t, pairs):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(stream)
            ctx.gossip_step(t, W, G, M, seg_offsets=seg)
            b.record(stream)
            if idx is not None:
                ctx.shuffle(t, gg.SHUF_PARTNER_SWAP, idx, off, stream=side)
            if pairs is not None:
                pairs.append((a, b))
        steps = min(wl["steps"], 32)
        wall, pr = time_loop(torch, step, steps, 3)
        ms = sorted(event_ms(pr))
        avg = sum(ms) / len(ms)
        algo = BYTES_PER_RANK_PARAM * p * n
        row = {"p": p, "n": n, "steps_timed": steps, "kernel_ms_avg": round(avg, 4), "kernel_ms_min": round(ms[0], 4),
               "GBps": round(algo / (avg * 1e-3) / 1e9, 1), "frac_of_hbm_peak": round(algo / (avg * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
               "step_ms_wall": round(wall, 4)}
        if name in ("C1", "C2"):
            row["cache_resident"] = True        # 50 MB / 653 MB of state against 256 MB of last-level cache
        if name == "C3":
            row["segments"] = 161
            L = p.bit_length() - 1

            def ar(t, pairs, one=False):
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record(stream)
                (ctx.allreduce_onepass if one else ctx.allreduce_baseline)(G, average=True)
                ctx.sgd_step(W, G, M)
                b.record(stream)
                if pairs is not None:
                    pairs.append((a, b))
            _, pr = time_loop(torch, ar, 4, 1)
            ar_ms = sum(event_ms(pr)) / len(pr)
            _, pr = time_loop(torch, lambda t, q: ar(t, q, True), 4, 1)
            ar1_ms = sum(event_ms(pr)) / len(pr)
            row["allreduce_sgd"] = {"recursive_doubling_ms": round(ar_ms, 4), "onepass_ms": round(ar1_ms, 4),
                                    "gossip_vs_recursive_doubling_time_ratio": round(avg / ar_ms, 4),
                                    "gossip_vs_onepass_time_ratio": round(avg / ar1_ms, 4),
                                    "bytes_moved_ratio_message_level": round(1.0 / L, 4),
                                    "bytes_moved_ratio_hbm_level": round(20.0 / (8.0 * L + 20.0), 4)}
        out[name] = row
        ctx.close()
        del W, G, M, idx
        torch.cuda.empty_cache()
    return out


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: the virtual ranks share one MI355X's HBM; --gpus %d is not "
              "supported (run with --gpus 1)" % args.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    import gg_synth
    import paper_1803_05880_amd as gg

    if not torch.cuda.is_available():
        print("no GPU visible: bench.py needs an MI355X", file=sys.stderr)
        sys.exit(1)
    # never time a library built from other sources than the ones in this tree: a stale build is
    # rebuilt before it is loaded, and the loaded library must report the digest of these sources
    digest = gg.ensure_current()
    wl = WORKLOADS[args.workload]
    p, n = wl["p"], wl["n"]
    stride = (n + args.stride_align - 1) // args.stride_align * args.stride_align
    lr, mu = gg_synth.LR, gg_synth.MOMENTUM
    dev = "cuda:0"
    torch.cuda.set_device(0)

    W, G, M = gg_synth.make_state(p, n, stride, seed=0, device=dev)
    off = gg_synth.block_offsets(SHUFFLE_N, p)
    idx = gg_synth.make_indices(SHUFFLE_N, dev)
    ctx = gg.Context(p=p, n=n, rank_stride=stride, seed=0, lr=lr, momentum=mu)
    tuned = False
    for key, val in ((gg.TUNE_THREADS, args.threads), (gg.TUNE_CHUNKS, args.chunks),
                     (gg.TUNE_BLOCKS_PER_CU, args.blocks_per_cu), (gg.TUNE_NONTEMPORAL, args.nontemporal)):
        if val is not None:
            ctx.set_tuning(key, val)
            tuned = True
    stream = torch.cuda.current_stream()

    def ev():
        return torch.cuda.Event(enable_timing=True)

    # ---- headline: gossip step + shuffle
    def full_step(t, pairs):
        if pairs is None:
            ctx.gossip_step(t, W, G, M)
        else:
            a, b = ev(), ev()
            a.record(stream)
            ctx.gossip_step(t, W, G, M)
            b.record(stream)
            pairs.append((a, b))
        # the index shuffle does not depend on the parameter update: it runs beside it on
        # its own stream (the paper overlaps the sample rotation with computation, Sec. 5)
        ctx.shuffle(t, gg.SHUF_PARTNER_SWAP, idx, off, stream=side_stream)

    side_stream = torch.cuda.Stream()
    ctx.shuffle(0, gg.SHUF_PARTNER_SWAP, idx, off)      # first use allocates the library's scratch
    torch.cuda.synchronize()
    ms_step, pairs = time_loop(torch, full_step, args.steps, args.warmup)
    k_ms = event_ms(pairs)
    k_avg = sum(k_ms) / len(k_ms)
    algo_bytes = BYTES_PER_RANK_PARAM * p * n
    value = algo_bytes / (ms_step * 1e-3) / 1e9
    achieved = algo_bytes / (k_avg * 1e-3) / 1e9
    traffic, traffic_source = (None, "launch shape differs from the profiled default") if tuned else \
        pmc_traffic(args.workload, digest)

    out = {
        "metric": "fused gossip+SGD step: effective HBM GB/s and % of MI355X peak (p ranks x N params)",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBS, 2),
        "config": {
            "workload": "%s: p=%d virtual ranks x N=%d fp32 params (w,g,m %.2f GB), hypercube partners with "
                        "rotation (R=p), synchronous model average + momentum SGD (lr 0.1, mu 0.9), plus "
                        "partner-swap shuffle of %d int32 sample ids" % (args.workload, p, n, 12.0 * p * stride / 1e9,
                                                                         SHUFFLE_N),
            "p": p, "n": n, "rank_stride": stride, "bytes_per_step": algo_bytes,
        },
        "roofline": {
            "bound": "hbm",
            "kernel": pair_kernel_name(args),
            "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 4),
            "traffic": traffic,
            "traffic_source": traffic_source,
            "algorithmic_bytes_per_launch": algo_bytes,
            "kernel_ms_avg": round(k_avg, 4),
            "kernel_ms_med": round(sorted(k_ms)[len(k_ms) // 2], 4),
            "kernel_ms_min": round(min(k_ms), 4),
        },
        "library_source_sha256": digest,
    }

    if not args.no_extras:
        extras = {}
        reps = max(3, min(args.steps, 16))

        # shuffle alone
        def shuf(t, pairs):
            a, b = ev(), ev()
            a.record(stream)
            ctx.shuffle(t, gg.SHUF_PARTNER_SWAP, idx, off)
            b.record(stream)
            if pairs is not None:
                pairs.append((a, b))
        _, pr = time_loop(torch, shuf, reps, 2)
        extras["shuffle_ms"] = round(sum(event_ms(pr)) / len(pr), 4)

        # ring rotation of the sample payload: 64 resident samples per rank, batch 32,
        # 256x256x3-byte samples (Table 5); bytes moved = read + write of p*batch samples
        sample_bytes, resident, batch = 196_608, 64, 32
        pay = torch.zeros((p * resident, sample_bytes // 4), dtype=torch.int32, device=dev)
        pay.random_(0, 2**31 - 1)
        poff = gg_synth.block_offsets(p * resident, p)

        def payload(t, pairs):
            a, b = ev(), ev()
            a.record(stream)
            ctx.shuffle_payload(t, pay, poff, batch)
            b.record(stream)
            if pairs is not None:
                pairs.append((a, b))
        _, pr = time_loop(torch, payload, reps, 2)
        pay_ms = sum(event_ms(pr)) / len(pr)
        extras["payload_ring_shuffle"] = {"ms": round(pay_ms, 4), "batch": batch, "sample_bytes": sample_bytes,
                                          "GBps": round(2.0 * p * batch * sample_bytes / (pay_ms * 1e-3) / 1e9, 1)}
        del pay

        # plain copy kernel on a W-sized buffer (read + write = 2 x bytes)
        scratch = torch.empty_like(W)

        def cp(t, pairs):
            a, b = ev(), ev()
            a.record(stream)
            gg.copy_probe(scratch, W)
            b.record(stream)
            if pairs is not None:
                pairs.append((a, b))
        _, pr = time_loop(torch, cp, reps, 2)
        cp_ms = sum(event_ms(pr)) / len(pr)
        extras["copy_kernel_GBps"] = round(2.0 * 4 * p * stride / (cp_ms * 1e-3) / 1e9, 1)
        extras["gossip_pct_of_copy_kernel"] = round(100.0 * achieved / extras["copy_kernel_GBps"], 1)

        # the runtime's own device-to-device copy of the same buffer, for reference
        def rt_copy(t, pairs):
            a, b = ev(), ev()
            a.record(stream)
            scratch.copy_(W)
            b.record(stream)
            if pairs is not None:
                pairs.append((a, b))
        _, pr = time_loop(torch, rt_copy, reps, 2)
        rt_ms = sum(event_ms(pr)) / len(pr)
        extras["runtime_d2d_copy_GBps"] = round(2.0 * 4 * p * stride / (rt_ms * 1e-3) / 1e9, 1)

        # staleness-1 variant with a double buffer (scratch doubles as the second w)
        ctx_s = gg.Context(p=p, n=n, rank_stride=stride, seed=0, lr=lr, momentum=mu, staleness=1)
        bufs = [W, scratch]

        def stale(t, pairs):
            a, b = ev(), ev()
            a.record(stream)
            ctx_s.gossip_step(t, bufs[t & 1], G, M, w_next=bufs[(t & 1) ^ 1])
            b.record(stream)
            if pairs is not None:
                pairs.append((a, b))
        _, pr = time_loop(torch, stale, reps, 2)
        st_ms = sum(event_ms(pr)) / len(pr)
        extras["staleness1_double_buffer"] = {"kernel_ms": round(st_ms, 4),
                                              "GBps": round(algo_bytes / (st_ms * 1e-3) / 1e9, 1)}
        ctx_s.close()

        # gradient averaging (the gradient-buffer reading of the exchange, Sec. 5)
        ctx_g = gg.Context(p=p, n=n, rank_stride=stride, seed=0, lr=lr, momentum=mu, avg_mode=gg.AVG_GRAD)

        def gradavg(t, pairs):
            a, b = ev(), ev()
            a.record(stream)
            ctx_g.gossip_step(t, W, G, M)
            b.record(stream)
            if pairs is not None:
                pairs.append((a, b))
        _, pr = time_loop(torch, gradavg, reps, 2)
        ga_ms = sum(event_ms(pr)) / len(pr)
        extras["gradient_averaging"] = {"kernel_ms": round(ga_ms, 4), "GBps": round(algo_bytes / (ga_ms * 1e-3) / 1e9, 1)}
        ctx_g.close()

        # dissemination topology (the paper's preferred one, Sec. 4.4.2): one step per phase k
        ctx_d = gg.Context(p=p, n=n, rank_stride=stride, seed=0, lr=lr, momentum=mu, topology=gg.TOPO_DISSEMINATION)
        L_d = max(1, (p - 1).bit_length())
        per_phase = []
        for k in range(L_d):
            def dis(t, pairs, k=k):
                a, b = ev(), ev()
                a.record(stream)
                ctx_d.gossip_step(k + L_d * t, W, G, M)
                b.record(stream)
                if pairs is not None:
                    pairs.append((a, b))
            _, pr = time_loop(torch, dis, 6, 1)
            per_phase.append(sum(event_ms(pr)) / len(pr))
        ctx_d.close()
        mean_gbps = algo_bytes * len(per_phase) / (sum(per_phase) * 1e-3) / 1e9
        extras["dissemination"] = {
            "ms_per_phase": [round(x, 4) for x in per_phase],
            "GBps_per_phase": [round(algo_bytes / (x * 1e-3) / 1e9, 1) for x in per_phase],
            "GBps_mean": round(mean_gbps, 1),
            "frac_of_hbm_peak_mean": round(mean_gbps / HBM_PEAK_GBS, 4),
        }

        # layer-wise exchange overlapped with a stand-in compute kernel
        extras["layerwise_overlap"] = layerwise_overlap(torch, gg, gg_synth, ctx, W, G, M, n, k_avg, scratch)

        # all-reduce + SGD comparator on the same buffers (G is clobbered: last)
        L = p.bit_length() - 1

        def ar(t, pairs):
            a, b = ev(), ev()
            a.record(stream)
            ctx.allreduce_baseline(G, average=True)
            ctx.sgd_step(W, G, M)
            b.record(stream)
            if pairs is not None:
                pairs.append((a, b))
        _, pr = time_loop(torch, ar, max(3, reps // 2), 1)
        ar_ms = sum(event_ms(pr)) / len(pr)

        def ar1(t, pairs):
            a, b = ev(), ev()
            a.record(stream)
            ctx.allreduce_onepass(G, average=True)
            ctx.sgd_step(W, G, M)
            b.record(stream)
            if pairs is not None:
                pairs.append((a, b))
        _, pr = time_loop(torch, ar1, max(3, reps // 2), 1)
        ar1_ms = sum(event_ms(pr)) / len(pr)

        def onepass_alone(t, pairs):
            a, b = ev(), ev()
            a.record(stream)
            ctx.allreduce_onepass(G, average=True)
            b.record(stream)
            if pairs is not None:
                pairs.append((a, b))
        _, pr = time_loop(torch, onepass_alone, max(3, reps // 2), 1)
        op_ms = sum(event_ms(pr)) / len(pr)

        def sgd_alone(t, pairs):
            a, b = ev(), ev()
            a.record(stream)
            ctx.sgd_step(W, G, M)
            b.record(stream)
            if pairs is not None:
                pairs.append((a, b))
        _, pr = time_loop(torch, sgd_alone, max(3, reps // 2), 1)
        sgd_ms = sum(event_ms(pr)) / len(pr)
        # Sec. 7.5 alternative: log2(p) local steps, then one all-reduce of the models
        def every_logp(t, pairs):
            a, b = ev(), ev()
            a.record(stream)
            for _ in range(L):
                ctx.sgd_step(W, G, M)
            ctx.allreduce_onepass(W, average=True)
            b.record(stream)
            if pairs is not None:
                pairs.append((a, b))
        _, pr = time_loop(torch, every_logp, 3, 1)
        logp_ms = sum(event_ms(pr)) / len(pr)
        extras["allreduce_every_log_p"] = {"ms_per_step": round(logp_ms / L, 4),
                                           "gossip_vs_every_log_p_time_ratio": round(k_avg / (logp_ms / L), 4)}
        extras["allreduce_sgd"] = {
            "recursive_doubling_ms": round(ar_ms, 4),
            "onepass_ms": round(ar1_ms, 4),
            "onepass_kernel_alone": {"ms": round(op_ms, 4), "GBps": round(8.0 * p * n / (op_ms * 1e-3) / 1e9, 1)},
            "sgd_kernel_alone": {"ms": round(sgd_ms, 4), "GBps": round(algo_bytes / (sgd_ms * 1e-3) / 1e9, 1)},
            "gossip_vs_recursive_doubling_time_ratio": round(k_avg / ar_ms, 4),
            "gossip_vs_onepass_time_ratio": round(k_avg / ar1_ms, 4),
            "bytes_moved_ratio_message_level": round(1.0 / L, 4),
            "bytes_moved_ratio_hbm_level": round(20.0 / (8.0 * L + 20.0), 4),
        }
        del scratch
        out["extras"] = extras
    ctx.close()
    del W, G, M
    torch.cuda.empty_cache()

    if not args.no_extras and not args.no_workloads:
        out["extras"]["workloads"] = other_workloads(torch, gg, gg_synth, args.workload, args.stride_align, lr, mu, dev)

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.workload, p, n, lr, mu)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
