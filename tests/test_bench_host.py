"""Host-side pieces of bench.py that need no GPU."""
import subprocess
import sys
import os

import numpy as np

import bench
import gg_synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_buckets_tile_the_buffer_in_backprop_order():
    for n, nseg in [(gg_synth.RESNET50_PARAMS, 161), (1_048_576, 161), (100_003, 7), (1000, 3)]:
        seg, _ = gg_synth.segment_layout(n, nseg, seed=0, lo=1, hi=max(2, n // 4))
        buckets = bench.make_buckets(seg, n, n // 24)
        assert buckets[0][1] == n and buckets[-1][0] == 0
        for (lo, hi), (lo2, hi2) in zip(buckets, buckets[1:]):
            assert hi2 == lo and lo < hi                     # descending, contiguous, non-empty
        assert all(lo % 64 == 0 for lo, _ in buckets)
        assert sum(hi - lo for lo, hi in buckets) == n


def test_segment_layout_matches_its_recipe():
    off, scales = gg_synth.segment_layout(gg_synth.RESNET50_PARAMS, 161, seed=0)
    sizes = np.diff(off)
    assert off[0] == 0 and off[-1] == gg_synth.RESNET50_PARAMS and len(sizes) == 161 and (sizes >= 1).all()
    assert (scales >= 0.1).all() and (scales <= 10.0).all()
    ratio = sizes.max() / sizes.min()
    assert 1e2 < ratio < 2_359_296 / 64 * 4                  # log-uniform spread survives the rescaling
    off2, _ = gg_synth.segment_layout(gg_synth.RESNET50_PARAMS, 161, seed=0)
    assert np.array_equal(off, off2)                         # seeded


def test_more_than_one_gpu_is_refused_with_a_message():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert res.returncode != 0 and "one GPU" in res.stderr and not res.stdout.strip()
