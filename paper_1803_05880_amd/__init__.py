"""GossipGraD hot path for one MI355X: thin Python face of the C-ABI library.

The package holds the HIP sources (csrc/), the build step (build.py) and the
ctypes binding (binding.py).  There is no fallback implementation.
"""
from .binding import (  # noqa: F401
    AVG_GRAD, AVG_MODEL, AVG_NONE, Context, GGConfig, GGError, LIB_PATH, MAX_RANKS, SHUF_PARTNER_SWAP,
    SHUF_RING, TOPO_DISSEMINATION, TOPO_HYPERCUBE, TUNE_BLOCKS_PER_CU, TUNE_CHUNKS, TUNE_HOP_GROUP, TUNE_NONTEMPORAL,
    TUNE_THREADS, TUNE_WALK_AHEAD, TUNE_WALK_STRIDED, TUNE_WALK_TILES, aligned_stride, busy_probe, copy_probe, lib,
)
