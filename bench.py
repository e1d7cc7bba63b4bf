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
HIP events, the staleness-1 double-buffer variant, the recursive-doubling
all-reduce + SGD comparator on the same buffers, a plain copy kernel, and the
CPU oracle timed on a bounded sample of the same workload.
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
WORKLOADS = {
    "C4": dict(p=64, n=25_557_032, shuffle_n=1_281_167),
    "C5": dict(p=128, n=25_557_032, shuffle_n=1_281_167),
    "C3": dict(p=16, n=25_557_032, shuffle_n=1_281_167),
    "C2": dict(p=8, n=6_800_000, shuffle_n=1_281_167),
    "C1": dict(p=4, n=1_048_576, shuffle_n=1_281_167),
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


def pmc_traffic_bytes(workload):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3
    counter summary, or None when no summary for this workload exists."""
    path = os.path.join(ROOT, "profiles", "gossip_pair_kernel_%s_pmc.txt" % workload)
    try:
        m = re.search(r"^traffic_bytes_per_launch:\s*([0-9.eE+]+)", open(path).read(), re.M)
        return float(m.group(1)) if m else None
    except OSError:
        return None


def cpu_baseline(p, lr, mu):
    """The oracle as it stands, on a bounded sample: the first n_s parameters of
    p ranks (fresh draws of the same distributions).  Timed single-threaded (the
    headline figure of this object) and, because the step is elementwise in the
    parameter index, once more with the sample's columns cut into one slice per
    host core, each slice run by the unchanged oracle in its own thread."""
    import concurrent.futures as cf
    import numpy as np
    from oracle import gossip as og, schedule as sc
    n_s, budget_s, max_steps = 1_048_576, 7.0, 400
    rng = np.random.default_rng(0)
    W = rng.normal(0, 0.05, (p, n_s)).astype(np.float32)
    G = rng.normal(0, 1e-3, (p, n_s)).astype(np.float32)
    M = np.zeros_like(W)

    def run(step_fn):
        step_fn(0)                                                     # warm-up
        t0 = time.perf_counter()
        steps = 0
        while steps < max_steps and (steps < 2 or time.perf_counter() - t0 < budget_s):
            steps += 1
            step_fn(steps)
        return (time.perf_counter() - t0) / steps, steps

    dt1, steps1 = run(lambda t: og.gossip_step(W, G, M, sc.partners(p, 0, p, sc.HYPERCUBE, t)[1], lr, mu))

    cores = max(1, min(os.cpu_count() or 1, 64))
    cuts = np.linspace(0, n_s, cores + 1).astype(np.int64)
    slices = [tuple(np.ascontiguousarray(a[:, cuts[i]:cuts[i + 1]]) for a in (W, G, M)) for i in range(cores)]
    pool = cf.ThreadPoolExecutor(cores)

    def threaded(t):
        c = sc.partners(p, 0, p, sc.HYPERCUBE, t)[1]
        list(pool.map(lambda s: og.gossip_step(s[0], s[1], s[2], c, lr, mu), slices))

    dtc, stepsc = run(threaded)
    pool.shutdown()
    gbs = lambda dt: round(BYTES_PER_RANK_PARAM * p * n_s / dt / 1e9, 3)
    return {
        "value": gbs(dt1),
        "unit": "GB/s",
        "cores": 1,
        "kind": "oracle",
        "sample": "p=%d ranks x first %d params, %d gossip steps, numpy fp32 (single thread); %.3f s/step"
                  % (p, n_s, steps1, dt1),
        "all_cores": {"value": gbs(dtc), "unit": "GB/s", "cores": cores,
                      "sample": "same sample cut into %d column slices, one thread each, %d steps; %.3f s/step"
                                % (cores, stepsc, dtc)},
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


def layerwise_overlap(torch, gg, gg_synth, ctx, W, G, M, n, gossip_ms, reps=5):
    """Layer-wise exchange overlapped with computation (Sec. 5, 5.1): the buffer is cut
    into 161 per-layer segments, grouped into ~24 buckets in back-propagation order
    (last layer first); a stand-in compute kernel runs piece by piece on the main
    stream and each bucket's gossip update is enqueued on a side stream as soon as
    "its" piece is done.  Compute is sized 3.5x the exchange, the ratio the paper
    reports (96 ms vs 27 ms).  Returns the three timings and the hidden fraction."""
    seg, _ = gg_synth.segment_layout(n, 161, seed=0)
    buckets = make_buckets(seg, n, n // 24)
    main = torch.cuda.current_stream()
    side = torch.cuda.Stream()
    sink = torch.zeros(1, device=W.device)
    blocks = 1024

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

    probe_iters = 100_000
    t_probe = timed(lambda: gg.busy_probe(probe_iters, blocks, sink), 3)
    iters = max(1, int(probe_iters * (3.5 * gossip_ms / len(buckets)) / t_probe))

    def compute_only():
        for _ in buckets:
            gg.busy_probe(iters, blocks, sink)

    step = [0]

    def gossip_only():
        for lo, hi_ in buckets:
            ctx.gossip_step(step[0], W, G, M, seg_offsets=[lo, hi_])
        step[0] += 1

    def pipelined():
        for lo, hi_ in buckets:
            gg.busy_probe(iters, blocks, sink)
            e = torch.cuda.Event()
            e.record(main)
            side.wait_event(e)
            ctx.gossip_step(step[0], W, G, M, seg_offsets=[lo, hi_], stream=side)
        done = torch.cuda.Event()
        done.record(side)
        main.wait_event(done)
        step[0] += 1

    t_c = timed(compute_only, reps)
    t_g = timed(gossip_only, reps)
    t_p = timed(pipelined, reps)
    return {
        "buckets": len(buckets), "segments": 161,
        "compute_ms": round(t_c, 4), "gossip_bucketed_ms": round(t_g, 4), "pipelined_ms": round(t_p, 4),
        "exchange_hidden_fraction": round(max(0.0, min(1.0, (t_c + t_g - t_p) / t_g)), 4),
    }


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
    wl = WORKLOADS[args.workload]
    p, n = wl["p"], wl["n"]
    stride = (n + args.stride_align - 1) // args.stride_align * args.stride_align
    lr, mu = gg_synth.LR, gg_synth.MOMENTUM
    dev = "cuda:0"
    torch.cuda.set_device(0)

    W, G, M = gg_synth.make_state(p, n, stride, seed=0, device=dev)
    off = gg_synth.block_offsets(wl["shuffle_n"], p)
    idx = gg_synth.make_indices(wl["shuffle_n"], dev)
    ctx = gg.Context(p=p, n=n, rank_stride=stride, seed=0, lr=lr, momentum=mu)
    for key, val in ((gg.TUNE_THREADS, args.threads), (gg.TUNE_CHUNKS, args.chunks),
                     (gg.TUNE_BLOCKS_PER_CU, args.blocks_per_cu), (gg.TUNE_NONTEMPORAL, args.nontemporal)):
        if val is not None:
            ctx.set_tuning(key, val)
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
                                                                         wl["shuffle_n"]),
            "p": p, "n": n, "rank_stride": stride, "bytes_per_step": algo_bytes,
        },
        "roofline": {
            "bound": "hbm",
            "kernel": "gossip_pair_lean_kernel<MODE_SYNC, nontemporal>",
            "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 4),
            "traffic": pmc_traffic_bytes(args.workload),
            "algorithmic_bytes_per_launch": algo_bytes,
            "kernel_ms_avg": round(k_avg, 4),
            "kernel_ms_med": round(sorted(k_ms)[len(k_ms) // 2], 4),
            "kernel_ms_min": round(min(k_ms), 4),
        },
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

        # dissemination topology (the paper's preferred one, Sec. 4.4.2): one step per phase k
        ctx_d = gg.Context(p=p, n=n, rank_stride=stride, seed=0, lr=lr, momentum=mu, topology=gg.TOPO_DISSEMINATION)
        L_d = max(1, (p - 1).bit_length())
        ctx_d.gossip_step(0, W, G, M)                    # first use allocates the carry column
        torch.cuda.synchronize()
        per_phase = []
        for k in range(L_d):
            def dis(t, pairs, k=k):
                a, b = ev(), ev()
                a.record(stream)
                ctx_d.gossip_step(k + L_d * t, W, G, M)
                b.record(stream)
                if pairs is not None:
                    pairs.append((a, b))
            _, pr = time_loop(torch, dis, 4, 1)
            per_phase.append(sum(event_ms(pr)) / len(pr))
        ctx_d.close()
        extras["dissemination"] = {
            "ms_per_phase": [round(x, 4) for x in per_phase],
            "GBps_mean": round(algo_bytes * len(per_phase) / (sum(per_phase) * 1e-3) / 1e9, 1),
        }

        # layer-wise exchange overlapped with a stand-in compute kernel
        extras["layerwise_overlap"] = layerwise_overlap(torch, gg, gg_synth, ctx, W, G, M, n, k_avg)

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
            "gossip_vs_recursive_doubling_time_ratio": round(k_avg / ar_ms, 4),
            "gossip_vs_onepass_time_ratio": round(k_avg / ar1_ms, 4),
            "bytes_moved_ratio_message_level": round(1.0 / L, 4),
            "bytes_moved_ratio_hbm_level": round(20.0 / (8.0 * L + 20.0), 4),
        }
        out["extras"] = extras
    ctx.close()

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(p, lr, mu)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
