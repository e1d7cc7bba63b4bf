/*
 * gg_probe.h -- measurement aids of the GossipGraD library.  Not part of the
 * method: nothing here computes a step of the hot path, and no result of gg.h's
 * entry points depends on any of it.  Kept apart so that gg.h stays the boundary.
 *
 * Same conventions as gg.h (status codes, device pointers, streams).
 */
#ifndef GG_PROBE_H_
#define GG_PROBE_H_

#include <stdint.h>

#include "gg.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Digest (sha256, hex) of the sources and compiler flags this library was built from,
 * as the build step computed it; "unknown" for a build that did not pass one.  Lets a
 * benchmark refuse to time a library that is older than the sources beside it.  Static. */
const char* gg_build_id(void);

/* Plain device-to-device copy kernel (16-byte non-temporal loads/stores) used to
 * calibrate achievable memory bandwidth next to the gossip kernel, and as the
 * known-size reference that scales the profiler's byte counters.  dst, src:
 * device, 16-byte aligned, nbytes a multiple of 16. */
int gg_copy_probe(void* dst, const void* src, int64_t nbytes, void* stream);

/* An arithmetic-only kernel (no memory traffic) that stands in for the
 * forward/backward computation when the overlap of the layer-wise exchange with
 * computation (Sec. 5, Sec. 5.1) is measured.  Runs `blocks` workgroups of 256
 * threads, each thread a dependent chain of `iters` multiply-adds.  sink: device
 * float[1], written only if the chain ends on an impossible value (keeps the loop
 * alive).  1 <= blocks <= 65536, iters >= 0. */
int gg_busy_probe(int64_t iters, int32_t blocks, float* sink, void* stream);

/* The same stand-in with memory traffic: `blocks` workgroups of 256 threads stride once
 * over buf; a thread reads four 16-byte chunks, runs a dependent chain of `iters`
 * multiply-adds on each and writes them back in place, so the computation competes with
 * the exchange for memory bandwidth the way a forward/backward pass does while leaving
 * it wavefront slots.  Its share of the bandwidth is 2 * nbytes over its duration, which
 * iters sets (more arithmetic per byte = lower share); the caller measures it.  buf:
 * device, 16-byte aligned, nbytes a multiple of 16; what is written is finite but
 * otherwise meaningless.  1 <= blocks <= 65536, iters >= 0. */
int gg_stream_probe(int64_t iters, int32_t blocks, void* buf, int64_t nbytes, void* stream);

/* Launch-shape knobs for bandwidth sweeps (never change results). */
enum {
  GG_TUNE_THREADS = 0,       /* threads per workgroup of the general kernels: 64, 128, 256 (default 64) */
  GG_TUNE_CHUNKS = 1,        /* 16-byte chunks per thread per tile: 1, 2, 4, 8 (default 1)              */
  GG_TUNE_BLOCKS_PER_CU = 2, /* cap on resident workgroups per CU, enforced by reserving LDS: 0 = none,
                                3..64 (default 7: few wavefronts in flight keep the set of open DRAM
                                rows small, which is what the streaming kernels want)                   */
  GG_TUNE_NONTEMPORAL = 3,   /* non-temporal loads/stores: 0, 1 (default 1)                             */
  /* kernels that walk over many ranks (dissemination cycles, one-pass all-reduce, payload ring); a key
     that was never set keeps each kernel's own default, given as cycles / all-reduce / ring: */
  GG_TUNE_WALK_CHUNKS = 4,   /* chunks per thread: 1, 2, 4, 8 (1 / 1 / 1); 0 = the kernel's general form      */
  GG_TUNE_WALK_WAVES = 5,    /* wavefronts per workgroup: 1, 2, 4, 8 (4 / 4 / 8); chunks * waves <= 8         */
  GG_TUNE_WALK_STEP = 6,     /* tiles (1 KB) between two tiles of one workgroup: 1..65536 (32)                */
  GG_TUNE_WALK_WG_PER_CU = 7,/* cap on resident workgroups per CU: 0 = none, 3..64 (3 / 3 / 0)                */
  GG_TUNE_WALK_BARRIER = 8,  /* barrier after every hop: 0, 1 (1)                                             */
  GG_TUNE_WALK_GROUP_LOG2 = 9/* all-reduce, ring: 2^this ranks between two barriers: 0..3 (- / 2 / 1)         */
};
int gg_set_tuning(gg_ctx* ctx, int32_t key, int32_t value);

#ifdef __cplusplus
}
#endif
#endif /* GG_PROBE_H_ */
