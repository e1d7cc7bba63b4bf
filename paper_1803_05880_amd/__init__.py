"""GossipGraD hot path for one MI355X: thin Python face of the C-ABI library.

The package holds the HIP sources (csrc/), the build step (build.py) and the
ctypes binding (binding.py).  There is no fallback implementation.
"""
from .binding import (  # noqa: F401
    AVG_GRAD, AVG_MODEL, AVG_NONE, Context, GGConfig, GGError, LIB_PATH, MAX_RANKS, SHUF_PARTNER_SWAP,
    SHUF_RING, TOPO_DISSEMINATION, TOPO_HYPERCUBE, TUNE_BLOCKS_PER_CU, TUNE_CHUNKS, TUNE_NONTEMPORAL,
    TUNE_THREADS, TUNE_WALK_BARRIER, TUNE_WALK_CHUNKS, TUNE_WALK_GROUP_LOG2, TUNE_WALK_STEP, TUNE_WALK_WAVES, TUNE_WALK_WG_PER_CU,
    aligned_stride, build_id, busy_probe, copy_probe, ensure_current, lib, stream_probe,
)
