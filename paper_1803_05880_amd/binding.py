"""ctypes binding of libgg.so: argument marshalling only.

Every step of the path runs in the library's HIP kernels; there is no CPU or
PyTorch fallback.  Importing this module fails loudly when libgg.so has not
been built and cannot be built (python -m paper_1803_05880_amd.build).  Tensors are torch CUDA
tensors used as device memory; the stream is torch's current stream unless
one is given.
"""
import ctypes
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgg.so")

GG_OK = 0
GG_ERR_ARG, GG_ERR_NOT_POW2, GG_ERR_ALIGN, GG_ERR_HIP, GG_ERR_NOMEM, GG_ERR_UNSUPPORTED, GG_ERR_LIMIT = -1, -2, -3, -4, -5, -6, -7
NOALLOC_MAX_INDICES, NOALLOC_MAX_TILE_COUNTS = 2_097_152, 65_536
TOPO_HYPERCUBE, TOPO_DISSEMINATION = 0, 1
AVG_MODEL, AVG_GRAD, AVG_NONE = 0, 1, 2
SHUF_PARTNER_SWAP, SHUF_RING = 0, 1
MAX_RANKS = 1024
TUNE_THREADS, TUNE_CHUNKS, TUNE_BLOCKS_PER_CU, TUNE_NONTEMPORAL = 0, 1, 2, 3
TUNE_WALK_CHUNKS, TUNE_WALK_WAVES, TUNE_WALK_STEP, TUNE_WALK_WG_PER_CU, TUNE_WALK_BARRIER = 4, 5, 6, 7, 8
TUNE_WALK_GROUP_LOG2 = 9


def aligned_stride(n, elements=1024):
    """Smallest rank_stride >= n whose rows start on 4096-byte boundaries (the layout
    the kernels reach full bandwidth with; see include/gg.h)."""
    return (int(n) + elements - 1) // elements * elements


class GGConfig(ctypes.Structure):
    _fields_ = [
        ("p", ctypes.c_int32),
        ("topology", ctypes.c_int32),
        ("n", ctypes.c_int64),
        ("rank_stride", ctypes.c_int64),
        ("num_comms", ctypes.c_int32),
        ("avg_mode", ctypes.c_int32),
        ("staleness", ctypes.c_int32),
        ("reserved", ctypes.c_int32),
        ("seed", ctypes.c_uint64),
        ("lr", ctypes.c_float),
        ("momentum", ctypes.c_float),
    ]


class GGError(RuntimeError):
    def __init__(self, code, what):
        self.code = code
        super().__init__("%s failed: %s (%d)" % (what, lib().gg_strerror(code).decode(), code))


_lib = None


def lib():
    """Load libgg.so once; raise if it is missing (no fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            # nothing built yet: compile once (hipcc cross-compiles without a GPU); there is
            # no other implementation to fall back to, so a failed build is fatal
            try:
                from .build import build_library
                build_library()
            except Exception as exc:
                raise ImportError("libgg.so is not built and building it failed (%s): run "
                                  "`python -m paper_1803_05880_amd.build`" % exc)
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
        L.gg_init.argtypes = [ctypes.POINTER(GGConfig), ctypes.POINTER(vp)]
        L.gg_destroy.argtypes = [vp]
        L.gg_set_hyper.argtypes = [vp, ctypes.c_float, ctypes.c_float]
        L.gg_partner.argtypes = [vp, i64, vp, vp]
        L.gg_gossip_step.argtypes = [vp, i64, vp, vp, vp, vp, vp, i32, vp]
        L.gg_sgd_step.argtypes = [vp, vp, vp, vp, vp]
        L.gg_allreduce_baseline.argtypes = [vp, vp, i32, vp]
        L.gg_allreduce_onepass.argtypes = [vp, vp, i32, vp]
        L.gg_shuffle.argtypes = [vp, i64, i32, vp, vp, i32, vp]
        L.gg_shuffle_noalloc.argtypes = [vp, i64, i32, vp, vp, i32, vp]
        L.gg_shuffle_payload.argtypes = [vp, i64, vp, i64, vp, i32, vp]
        L.gg_copy_probe.argtypes = [vp, vp, i64, vp]
        L.gg_busy_probe.argtypes = [i64, i32, vp, vp]
        L.gg_stream_probe.argtypes = [i64, i32, vp, i64, vp]
        L.gg_set_tuning.argtypes = [vp, i32, i32]
        L.gg_strerror.argtypes = [ctypes.c_int]
        L.gg_strerror.restype = ctypes.c_char_p
        L.gg_build_id.argtypes = []
        L.gg_build_id.restype = ctypes.c_char_p
        for name in ("gg_init", "gg_destroy", "gg_set_hyper", "gg_partner", "gg_gossip_step", "gg_sgd_step",
                     "gg_allreduce_baseline", "gg_allreduce_onepass", "gg_shuffle", "gg_shuffle_noalloc", "gg_shuffle_payload", "gg_copy_probe",
                     "gg_busy_probe", "gg_stream_probe", "gg_set_tuning"):
            getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def _check(code, what):
    if code != GG_OK:
        raise GGError(code, what)


def _dev_ptr(t, dtype, name):
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError("%s must be a CUDA tensor" % name)
    if t.dtype != dtype or not t.is_contiguous():
        raise TypeError("%s must be contiguous %s" % (name, dtype))
    return ctypes.c_void_p(t.data_ptr())


def _stream_ptr(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


class Context:
    """Owns one gg_ctx.  Method names mirror the C entry points."""

    def __init__(self, p, n, rank_stride=None, topology=TOPO_HYPERCUBE, num_comms=0, seed=0, lr=0.1,
                 momentum=0.9, avg_mode=AVG_MODEL, staleness=0):
        self._h = ctypes.c_void_p()
        self.p, self.n = int(p), int(n)
        self.rank_stride = int(n if rank_stride is None else rank_stride)
        cfg = GGConfig(p=p, topology=topology, n=n, rank_stride=self.rank_stride, num_comms=num_comms,
                       avg_mode=avg_mode, staleness=staleness, reserved=0, seed=seed, lr=lr, momentum=momentum)
        _check(lib().gg_init(ctypes.byref(cfg), ctypes.byref(self._h)), "gg_init")

    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            code = lib().gg_destroy(self._h)
            self._h = ctypes.c_void_p()
            _check(code, "gg_destroy")

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def set_hyper(self, lr, momentum):
        _check(lib().gg_set_hyper(self._h, lr, momentum), "gg_set_hyper")

    def partner(self, step):
        """gg_partner: (send_to, recv_from) as int32 numpy arrays."""
        send = np.empty(self.p, dtype=np.int32)
        recv = np.empty(self.p, dtype=np.int32)
        _check(lib().gg_partner(self._h, step, send.ctypes.data_as(ctypes.c_void_p),
                                recv.ctypes.data_as(ctypes.c_void_p)), "gg_partner")
        return send, recv

    def gossip_step(self, step, w, g, m, w_next=None, seg_offsets=None, stream=None):
        seg_ptr, nseg = None, 0
        if seg_offsets is not None:
            seg = np.ascontiguousarray(seg_offsets, dtype=np.int64)
            seg_ptr, nseg = seg.ctypes.data_as(ctypes.c_void_p), len(seg) - 1
        f32 = torch.float32
        _check(lib().gg_gossip_step(self._h, step, _dev_ptr(w, f32, "w"), _dev_ptr(g, f32, "g"),
                                    _dev_ptr(m, f32, "m"), _dev_ptr(w_next, f32, "w_next"), seg_ptr, nseg,
                                    _stream_ptr(stream)), "gg_gossip_step")

    def sgd_step(self, w, g, m, stream=None):
        f32 = torch.float32
        _check(lib().gg_sgd_step(self._h, _dev_ptr(w, f32, "w"), _dev_ptr(g, f32, "g"), _dev_ptr(m, f32, "m"),
                                 _stream_ptr(stream)), "gg_sgd_step")

    def allreduce_baseline(self, g, average=True, stream=None):
        _check(lib().gg_allreduce_baseline(self._h, _dev_ptr(g, torch.float32, "g"), int(bool(average)),
                                           _stream_ptr(stream)), "gg_allreduce_baseline")

    def allreduce_onepass(self, g, average=True, stream=None):
        _check(lib().gg_allreduce_onepass(self._h, _dev_ptr(g, torch.float32, "g"), int(bool(average)),
                                          _stream_ptr(stream)), "gg_allreduce_onepass")

    def shuffle(self, step, mode, idx, rank_offsets, batch=0, stream=None):
        off = np.ascontiguousarray(rank_offsets, dtype=np.int64)
        if off.shape != (self.p + 1,):
            raise ValueError("rank_offsets must have p+1 entries")
        _check(lib().gg_shuffle(self._h, step, mode, _dev_ptr(idx, torch.int32, "idx"),
                                off.ctypes.data_as(ctypes.c_void_p), batch, _stream_ptr(stream)), "gg_shuffle")

    def shuffle_noalloc(self, step, mode, idx, rank_offsets, batch=0, stream=None):
        """gg_shuffle_noalloc: gg_shuffle on the library's fixed scratch (allocates nothing)."""
        off = np.ascontiguousarray(rank_offsets, dtype=np.int64)
        if off.shape != (self.p + 1,):
            raise ValueError("rank_offsets must have p+1 entries")
        _check(lib().gg_shuffle_noalloc(self._h, step, mode, _dev_ptr(idx, torch.int32, "idx"),
                                        off.ctypes.data_as(ctypes.c_void_p), batch, _stream_ptr(stream)),
               "gg_shuffle_noalloc")

    def shuffle_payload(self, step, payload, rank_offsets, batch, stream=None):
        """gg_shuffle_payload: payload is a 2-D CUDA tensor [n_total][sample elements]."""
        off = np.ascontiguousarray(rank_offsets, dtype=np.int64)
        if off.shape != (self.p + 1,) or payload.dim() != 2 or not payload.is_cuda or not payload.is_contiguous():
            raise ValueError("payload must be a contiguous CUDA tensor [n_total][sample] and rank_offsets p+1 long")
        sample_bytes = payload.shape[1] * payload.element_size()
        _check(lib().gg_shuffle_payload(self._h, step, ctypes.c_void_p(payload.data_ptr()), sample_bytes,
                                        off.ctypes.data_as(ctypes.c_void_p), batch, _stream_ptr(stream)),
               "gg_shuffle_payload")

    def set_tuning(self, key, value):
        _check(lib().gg_set_tuning(self._h, key, value), "gg_set_tuning")


def copy_probe(dst, src, stream=None):
    """gg_copy_probe: plain device copy kernel for bandwidth calibration."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise ValueError("size mismatch")
    _check(lib().gg_copy_probe(ctypes.c_void_p(dst.data_ptr()), ctypes.c_void_p(src.data_ptr()), nbytes,
                               _stream_ptr(stream)), "gg_copy_probe")


def busy_probe(iters, blocks, sink, stream=None):
    """gg_busy_probe: arithmetic-only stand-in for forward/backward computation."""
    _check(lib().gg_busy_probe(int(iters), int(blocks), _dev_ptr(sink, torch.float32, "sink"), _stream_ptr(stream)),
           "gg_busy_probe")


def stream_probe(iters, blocks, buf, stream=None):
    """gg_stream_probe: stand-in for forward/backward computation that also streams memory."""
    _check(lib().gg_stream_probe(int(iters), int(blocks), ctypes.c_void_p(buf.data_ptr()),
                                 buf.numel() * buf.element_size(), _stream_ptr(stream)), "gg_stream_probe")


def build_id():
    """gg_build_id: digest of the sources the loaded library was built from."""
    return lib().gg_build_id().decode()


def ensure_current():
    """Make sure the library that gets loaded was built from the sources in this tree: a
    library on disk with another (or no) digest is rebuilt first, as long as it has not been
    loaded yet.  Returns the digest; raises when the loaded library does not match it."""
    from .build import DIGEST_PATH, build_library, source_digest
    digest = source_digest()
    try:
        on_disk = open(DIGEST_PATH).read().strip()
    except OSError:
        on_disk = None
    if _lib is None and (on_disk != digest or not os.path.exists(LIB_PATH)):
        build_library()
    if build_id() != digest:
        raise RuntimeError("libgg.so was built from other sources (%s...) than the ones beside it (%s...): run "
                           "`python -m paper_1803_05880_amd.build`" % (build_id()[:12], digest[:12]))
    return digest
