/*
 * gg.h -- C ABI of the GossipGraD hot path for one MI355X (gfx950).
 *
 * GossipGraD (arXiv 1803.05880) replaces the all-reduce of data-parallel SGD by
 * one exchange per step with a single, rotating partner.  This library runs
 * that step for p *virtual* ranks whose flat fp32 weight / gradient / momentum
 * buffers all live in the memory of one GPU:
 *
 *   - partner schedule: hypercube or dissemination virtual topology laid over
 *     one of R shuffled communicators, the next communicator taken after every
 *     log2(p) steps                                   (Sec. 4.3, 4.4, 4.5.1)
 *   - local momentum-SGD update followed by the average with the partner's
 *     post-update weights                             (Eq. 1-2, Sec. 6)
 *   - rotation of sample indices                      (Sec. 4.5.2, Lemma 1)
 *   - recursive-doubling all-reduce over the same ranks, the Theta(log p)
 *     method the paper compares with                  (Sec. 3.1, Sec. 4.1)
 *
 * Conventions
 *   - Every call returns GG_OK (0) or a negative gg_status.  Nothing is written
 *     and nothing is enqueued when a call fails argument validation.
 *   - "host" pointers are ordinary process memory, read or written before the
 *     call returns.  "device" pointers are HIP device memory of the GPU that was
 *     current at gg_init; they are owned, allocated and freed by the caller.
 *   - Device work is enqueued on `stream` (a hipStream_t passed as void*; NULL is
 *     the default stream) and the call returns without waiting.
 *   - The library keeps no step counter: `step` is an argument, so any step can
 *     be replayed.
 *   - A context is not thread-safe: call it from one host thread at a time.  Calls
 *     may target different streams; work that shares the context's scratch
 *     (two gg_shuffle calls) must be ordered by the caller.
 *   - All [p][.] buffers share one layout: rank j starts at element
 *     j * rank_stride, its n parameters are contiguous, rank_stride >= n.
 *     Buffers whose base address and rank_stride*4 are multiples of 16 bytes take
 *     the vector path; anything 4-byte aligned is accepted.  For full bandwidth make
 *     base addresses and rank_stride*4 multiples of 4096 bytes (rank_stride a
 *     multiple of 1024): measured on p = 64 ResNet50-sized rows, rows aligned to
 *     32 / 64 / 128 / 4096 bytes run at 6.1 / 6.4 / 6.5 / 6.57 TB/s.
 *   - fp32 arithmetic, every multiply/add/subtract rounded on its own (no fused
 *     multiply-add), denormals kept.
 */
#ifndef GG_H_
#define GG_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  GG_OK = 0,
  GG_ERR_ARG = -1,      /* null pointer, out-of-range value, inconsistent sizes     */
  GG_ERR_NOT_POW2 = -2, /* hypercube / all-reduce / partner-swap need p = 2^L       */
  GG_ERR_ALIGN = -3,    /* a device pointer is not 4-byte aligned                   */
  GG_ERR_HIP = -4,      /* a HIP runtime call failed (launch, copy)                 */
  GG_ERR_NOMEM = -5,    /* host or device allocation failed                         */
  GG_ERR_UNSUPPORTED = -6, /* valid request this build does not implement           */
  GG_ERR_LIMIT = -7     /* sizes beyond the fixed scratch of gg_shuffle_noalloc     */
} gg_status;

enum { GG_TOPO_HYPERCUBE = 0, GG_TOPO_DISSEMINATION = 1 };
enum { GG_AVG_MODEL = 0, GG_AVG_GRAD = 1, GG_AVG_NONE = 2 };
enum { GG_SHUF_PARTNER_SWAP = 0, GG_SHUF_RING = 1 };

#define GG_MAX_RANKS 1024

typedef struct gg_ctx gg_ctx; /* opaque; owns only its schedule tables and the shuffle's scratch */

typedef struct {
  int32_t p;           /* virtual ranks, 2 .. GG_MAX_RANKS; power of two for hypercube     */
  int32_t topology;    /* GG_TOPO_*                                                        */
  int64_t n;           /* fp32 parameters per rank, >= 0                                   */
  int64_t rank_stride; /* elements between consecutive ranks in every [p][.] buffer, >= n  */
  int32_t num_comms;   /* R, shuffled communicators: 1 = no rotation, 0 = p (Sec. 4.5.1);
                          at most 4096                                                     */
  int32_t avg_mode;    /* GG_AVG_*: what is averaged with the partner                      */
  int32_t staleness;   /* 0: partner's post-update weights of this step (Sec. 6);
                          1: partner's weights as they stood on entry to this step
                             (asynchronous variant; GG_AVG_MODEL only)                     */
  int32_t reserved;    /* must be 0                                                        */
  uint64_t seed;       /* key of every random draw (communicators, shuffle flags)          */
  float lr;            /* learning rate (lambda of Eq. 1-2)                                */
  float momentum;      /* mu                                                               */
} gg_config;

/* Build a context on the current HIP device: validates cfg, draws the R
 * communicators (communicator 0 is the original one, r >= 1 a Fisher-Yates
 * shuffle driven by Philox4x32-10 keyed by seed; Sec. 4.5.1 creates them once at
 * start-up) and uploads them.  *out is written only on success.  Host pointers. */
int gg_init(const gg_config* cfg, gg_ctx** out);

/* Change the learning rate and momentum used by later calls (the paper's runs
 * lower the learning rate on a schedule, Sec. 7.3).  Takes effect for calls
 * enqueued after it returns; NaN is rejected. */
int gg_set_hyper(gg_ctx* ctx, float lr, float momentum);

/* Free the context's tables and scratch (waits for the device first). */
int gg_destroy(gg_ctx* ctx);

/* Partner schedule of one step (Sec. 4.3, 4.4.1, 4.4.2, 4.5.1).  Pure function of
 * (ctx, step): phase k = step mod L, communicator r = (step div L) mod R,
 * L = ceil(log2 p).  Hypercube: send_to[j] = recv_from[j] = the rank whose virtual
 * id differs from j's in bit k.  Dissemination: virtual rank i sends to
 * (i + 2^k) mod p and receives from (i + p - 2^k) mod p.
 * send_to: host int32[p], required.  recv_from: host int32[p] or NULL.  step >= 0. */
int gg_partner(const gg_ctx* ctx, int64_t step, int32_t* send_to, int32_t* recv_from);

/* One GossipGraD step for all p ranks (Eq. 1-2 + Sec. 6), update and average fused in
 * one launch (plus one scalar launch for a ragged or unaligned remainder); allocates
 * nothing and never synchronises:
 *     v = mu*m + lr*g ;  m <- v ;  T = w - v ;  w_new[j] = (T[j] + X[c(j)]) / 2
 * with c = the step's partner map (hypercube: the pair partner; dissemination:
 * the rank j receives from), X = T (staleness 0) or the entry weights w
 * (staleness 1).  GG_AVG_GRAD averages the two gradients before the update
 * instead; GG_AVG_NONE is the local update alone.  g is never written.
 *   w, m   device float [p][rank_stride], updated in place
 *   g      device float [p][rank_stride], read only
 *   w_next device float [p][rank_stride] or NULL.  When given, the new weights go
 *          there and w is left untouched (double buffer of the asynchronous
 *          variant); every topology also works in place with NULL.
 *   seg_offsets / nseg   host int64[nseg+1] ascending offsets within [0, n]
 *          (per-layer segments, Sec. 5), or NULL / 0 for the whole buffer.  Only
 *          parameters in [seg_offsets[0], seg_offsets[nseg]) are touched; the
 *          result does not depend on how that range is cut into segments.
 * Buffers must not overlap one another. */
int gg_gossip_step(gg_ctx* ctx, int64_t step, float* w, const float* g, float* m,
                   float* w_next, const int64_t* seg_offsets, int32_t nseg, void* stream);

/* Local momentum-SGD update alone on every rank (Eq. 1-2; Sec. 4.1's
 * no-communication case), used after gg_allreduce_baseline.  In place on w, m. */
int gg_sgd_step(gg_ctx* ctx, float* w, const float* g, float* m, void* stream);

/* Recursive-doubling all-reduce of g over the p ranks (Sec. 3.1: the log p
 * reduction of the baseline): round k adds the buffer of rank j XOR 2^k, L rounds,
 * then (average != 0) multiplies by 1/p.  In place; every rank ends with the same
 * bits.  p must be a power of two.  g: device float [p][rank_stride]. */
int gg_allreduce_baseline(gg_ctx* ctx, float* g, int32_t average, void* stream);

/* The same sum in one pass: each element's p values are read once, added in the
 * order of the recursive-doubling tree (bit-identical result) and written back to
 * every rank -- the bandwidth-optimal form available when all ranks share one
 * memory.  Same arguments as gg_allreduce_baseline.  Above p = 128 it runs the
 * rounds of gg_allreduce_baseline instead (same result). */
int gg_allreduce_onepass(gg_ctx* ctx, float* g, int32_t average, void* stream);

/* Rotation of sample indices (Sec. 4.5.2).  idx: device int32[rank_offsets[p]],
 * rank j owns slots rank_offsets[j] .. rank_offsets[j+1]-1 (host int64[p+1],
 * ascending from 0).  In place.
 *   GG_SHUF_RING          each rank's slots are a full circular FIFO with head
 *                         (step*batch) mod n_j; the `batch` slots at the head (the
 *                         batch just used) go to rank (j+1) mod p and are replaced
 *                         by the batch of rank (j-1) mod p.  0 <= batch <= min n_j.
 *   GG_SHUF_PARTNER_SWAP  slot i of rank j is flagged when the top 3 bits of word
 *                         i%4 of Philox4x32-10(key = seed, counter = (i/4, j,
 *                         step mod 2^32, 2)) are zero; the r-th flagged slot of j
 *                         swaps with the r-th flagged slot of its hypercube
 *                         partner, r < min of the two counts.  `batch` ignored.
 * The context grows its scratch (one word per index plus per-tile counts) on first
 * use and keeps a device copy of rank_offsets; either may allocate or copy and
 * therefore synchronise the device on the first call or when the offsets change. */
int gg_shuffle(gg_ctx* ctx, int64_t step, int32_t mode, int32_t* idx,
               const int64_t* rank_offsets, int32_t batch, void* stream);

/* gg_shuffle for callers that cannot allocate: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, same result, same
 * kernels, but the scratch (rank offsets, flagged-slot lists, per-tile counts, staged
 * ring batches) is a fixed array that is part of the library image -- one copy per GPU,
 * about 8.3 MiB, held until the process ends -- and the rank offsets reach the device
 * in kernel arguments.  The call allocates nothing, frees nothing, copies nothing and
 * never synchronises.  Limits: rank_offsets[p] <= GG_NOALLOC_MAX_INDICES and
 * p * ceil(max n_j / 4096) <= GG_NOALLOC_MAX_TILE_COUNTS, else GG_ERR_LIMIT (nothing
 * enqueued).  Every call on a GPU, from any context, uses that GPU's one array and
 * overwrites what the last call left: calls that overlap on one GPU race, so order
 * them (one stream, or events).  Nothing in the array has to be cleared between calls. */
#define GG_NOALLOC_MAX_INDICES 2097152
#define GG_NOALLOC_MAX_TILE_COUNTS 65536
int gg_shuffle_noalloc(gg_ctx* ctx, int64_t step, int32_t mode, int32_t* idx,
                       const int64_t* rank_offsets, int32_t batch, void* stream);

/* The ring rotation of gg_shuffle(GG_SHUF_RING) applied to the samples themselves
 * (Sec. 4.5.2: a rank sends the batch it has just used to its ring neighbour;
 * Table 5 gives the sample sizes): slot s of rank j is the sample_bytes bytes at
 * payload + (rank_offsets[j] + s) * sample_bytes, and the slots move exactly as the
 * indices do, so an index array and a payload array rotated with the same
 * (step, batch) stay in correspondence.  In place, every byte read once and written
 * once.  payload: device, 4-byte aligned (16-byte aligned with sample_bytes % 16 == 0
 * for the vector path); sample_bytes > 0, multiple of 4; 0 <= batch <= min n_j. */
int gg_shuffle_payload(gg_ctx* ctx, int64_t step, void* payload, int64_t sample_bytes,
                       const int64_t* rank_offsets, int32_t batch, void* stream);

/* Static, never NULL. */
const char* gg_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* GG_H_ */
