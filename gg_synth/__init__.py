"""Seeded synthetic inputs for the GossipGraD hot path.

Serves both the CPU oracle's tests and the HIP path's tests/benchmark; holds
none of the method's arithmetic and imports neither side.  The buffers stand in
for the parameter sets of the networks the paper trains (ResNet50 ~25M
parameters, Sec. 5.2; GoogLeNet, Sec. 7.4) and for the ImageNet-1K training
index range (1,281,167 samples, Table 5): only counts and shapes are taken.

Values are data: they are drawn once on whichever device is asked for (CPU or
GPU) from a seeded torch generator, and handed to the other side by copy.
"""

import math
import numpy as np
import torch

RESNET50_PARAMS = 25_557_032
GOOGLENET_PARAMS = 6_800_000
IMAGENET1K_TRAIN = 1_281_167

# The five workload shapes.  lr / momentum / std values are the same everywhere.
CONFIGS = {
    "C1": dict(p=4, n=1_048_576, steps=8),
    "C2": dict(p=8, n=GOOGLENET_PARAMS, steps=9),
    "C3": dict(p=16, n=RESNET50_PARAMS, steps=32, nseg=161),
    "C4": dict(p=64, n=RESNET50_PARAMS, steps=64, staleness=1),
    "C5": dict(p=128, n=RESNET50_PARAMS, steps=128, shuffle_n=IMAGENET1K_TRAIN),
}
LR = 0.1
MOMENTUM = 0.9
W_STD = 0.05
G_STD = 1e-3
SEG_LO, SEG_HI = 64, 2_359_296


def segment_layout(n, nseg, seed=0, lo=SEG_LO, hi=SEG_HI):
    """Per-layer segment offsets and gradient scales for the segmented workload.

    Sizes are drawn log-uniform in [lo, hi] and rescaled to sum to n: each gets
    floor(raw * n / sum(raw)) (at least 1) and the remainder goes one element
    each to the segments with the largest fractional parts.  Scales ~ U(0.1, 10).
    Returns (offsets int64[nseg+1], scales float64[nseg]).
    """
    rng = np.random.default_rng(seed)
    raw = np.exp(rng.uniform(math.log(lo), math.log(hi), size=nseg))
    share = raw * (n / raw.sum())
    sizes = np.maximum(1, np.floor(share).astype(np.int64))
    rest = n - int(sizes.sum())
    order = np.argsort(-(share - np.floor(share)), kind="stable")
    i = 0
    while rest != 0:
        s = order[i % nseg]
        if rest > 0:
            sizes[s] += 1
            rest -= 1
        elif sizes[s] > 1:
            sizes[s] -= 1
            rest += 1
        i += 1
    offsets = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    scales = rng.uniform(0.1, 10.0, size=nseg)
    return offsets, scales


def make_state(p, n, rank_stride=None, seed=0, device="cpu", seg_offsets=None,
               seg_scales=None, w_std=W_STD, g_std=G_STD, identical_ranks=False):
    """Weights ~ N(0, w_std), gradients ~ N(0, g_std) (optionally scaled per
    segment), momentum zero.  Returns float32 tensors W, G, M of shape
    [p][rank_stride]; columns n.. (padding) are zero."""
    rank_stride = n if rank_stride is None else rank_stride
    assert rank_stride >= n
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    W = torch.zeros((p, rank_stride), dtype=torch.float32, device=device)
    G = torch.zeros((p, rank_stride), dtype=torch.float32, device=device)
    M = torch.zeros((p, rank_stride), dtype=torch.float32, device=device)
    scale_vec = None
    if seg_offsets is not None and seg_scales is not None:
        reps = torch.as_tensor(np.diff(np.asarray(seg_offsets)), device=device)
        scale_vec = torch.repeat_interleave(
            torch.as_tensor(np.asarray(seg_scales), dtype=torch.float32, device=device), reps)
    for j in range(p):
        if identical_ranks and j > 0:
            W[j, :n] = W[0, :n]
            G[j, :n] = G[0, :n]
            continue
        W[j, :n].normal_(0.0, w_std, generator=gen)
        G[j, :n].normal_(0.0, g_std, generator=gen)
        if scale_vec is not None:
            G[j, :n] *= scale_vec
    return W, G, M


def make_indices(n_total, device="cpu"):
    """Sample ids 0..n-1 in order (block-partitioned by the caller)."""
    return torch.arange(n_total, dtype=torch.int32, device=device)


def block_offsets(n_total, p):
    """Block partition: rank j holds floor(n/p) + (j < n mod p) consecutive slots."""
    base, extra = divmod(n_total, p)
    off = np.zeros(p + 1, dtype=np.int64)
    for j in range(p):
        off[j + 1] = off[j] + base + (1 if j < extra else 0)
    return off


def sample_windows(n, num_random=256, width=1024, seed=0, boundary=64 * 1024 * 1024):
    """Index windows [lo, hi) for slice checks of the largest shapes: the first
    and last 4096 elements, a window across every `boundary`-element multiple,
    and `num_random` random windows of `width` elements."""
    wins = [(0, min(4096, n)), (max(0, n - 4096), n)]
    b = boundary
    while b < n:
        wins.append((max(0, b - width // 2), min(n, b + width // 2)))
        b += boundary
    rng = np.random.default_rng(seed)
    for s in rng.integers(0, max(1, n - width), size=num_random):
        wins.append((int(s), min(n, int(s) + width)))
    return wins
