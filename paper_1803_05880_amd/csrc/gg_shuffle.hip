// Rotation of sample indices (Sec. 4.5.2, Lemma 1): the ring of used batches and
// the partner-swap variant.  Integer work only; results are bit-exact.
#include <string.h>

#include <mutex>

#include "gg_internal.h"

// ---- scratch that is never allocated: gg_shuffle_noalloc
// One array per GPU, part of the loaded code object, kept until the process ends.  In host
// code the array's name is only a stand-in for the symbol: its device address on each GPU
// comes from hipGetSymbolAddress with that GPU current, and only that address is ever
// handed to a kernel.  Layout: rank offsets int64[GG_MAX_RANKS + 1] (padded to 256-byte
// multiple), then the int32 words of check_shuffle's layout.
enum {
  NOALLOC_OFF_BYTES = ((GG_MAX_RANKS + 1) * 8 + 255) / 256 * 256,
  NOALLOC_WORDS = GG_NOALLOC_MAX_INDICES + GG_NOALLOC_MAX_TILE_COUNTS + 4,
  NOALLOC_MAX_DEVICES = 64,
  OFFSETS_PER_LAUNCH = 256
};
static __device__ __align__(256) unsigned char scratch[NOALLOC_OFF_BYTES + (size_t)NOALLOC_WORDS * 4];

namespace {

enum { SWAP_THREADS = 1024, SWAP_WAVES = SWAP_THREADS / 64, SLOTS_PER_THREAD = 4 };

struct swap_args {
  int32_t* idx;
  int32_t* sel;            // scratch int32[n_total]: flagged slot numbers, per rank, ascending
  const int64_t* off;      // device int64[p+1]
  const uint16_t* sigma;   // communicator row
  int32_t shift;
  uint32_t step32;
  uint32_t k0, k1;
};

// Inclusive prefix sum of one value per lane across the 64-lane wavefront.
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t x, uint32_t lane) {
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const uint32_t y = __shfl_up(x, d, 64);
    if (lane >= (uint32_t)d) x += y;
  }
  return x;
}

// Flags of the 4 consecutive slots a thread owns in the tile that starts at tile0
// (one Philox block); slots beyond the rank's end are never flagged.
__device__ __forceinline__ uint32_t tile_flags(const swap_args& a, uint32_t rank, int64_t n_r, int64_t tile0,
                                               uint32_t f[4]) {
  const int64_t slot0 = tile0 + (int64_t)threadIdx.x * SLOTS_PER_THREAD;
  f[0] = f[1] = f[2] = f[3] = 0;
  if (slot0 < n_r) {
    const gg_u32x4 o = gg_philox4x32_10((uint32_t)(slot0 >> 2), rank, a.step32, (uint32_t)GG_TAG_SHUF, a.k0, a.k1);
    f[0] = (o.x >> 29) == 0;
    f[1] = (o.y >> 29) == 0 && slot0 + 1 < n_r;
    f[2] = (o.z >> 29) == 0 && slot0 + 2 < n_r;
    f[3] = (o.w >> 29) == 0 && slot0 + 3 < n_r;
  }
  return f[0] + f[1] + f[2] + f[3];
}

// Exclusive prefix of one count per thread over the 1024-thread workgroup
// (wavefront prefix, then a prefix over the 16 wave totals in LDS).  Returns the
// thread's offset and the workgroup total; ends with a barrier so the LDS words can
// be reused at once.
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t cnt, uint32_t* s_wave, uint32_t* s_total,
                                                         uint32_t* total) {
  const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
  const uint32_t incl = wave_inclusive_scan(cnt, lane);
  if (lane == 63) s_wave[wave] = incl;
  __syncthreads();
  if (wave == 0) {
    const uint32_t t = lane < SWAP_WAVES ? s_wave[lane] : 0u;
    const uint32_t ti = wave_inclusive_scan(t, lane);
    if (lane < SWAP_WAVES) s_wave[lane] = ti - t;  // exclusive offset of each wave
    if (lane == SWAP_WAVES - 1) *s_total = ti;
  }
  __syncthreads();
  const uint32_t offset = s_wave[wave] + (incl - cnt);
  *total = *s_total;
  __syncthreads();
  return offset;
}

// Flag the slots of one rank tile by tile and write the flagged slot numbers to
// sel_r[0 ..] in ascending order (per-thread popcount -> prefix -> ordered
// scatter).  Returns the number of flagged slots (same in every thread).
__device__ uint32_t compact_flagged(const swap_args& a, uint32_t rank, int64_t n_r, int32_t* sel_r,
                                    uint32_t* s_wave, uint32_t* s_total) {
  uint32_t running = 0;
  const int64_t per_tile = (int64_t)SWAP_THREADS * SLOTS_PER_THREAD;
  for (int64_t tile0 = 0; tile0 < n_r; tile0 += per_tile) {
    uint32_t f[4], total;
    const uint32_t cnt = tile_flags(a, rank, n_r, tile0, f);
    uint32_t pos = running + block_exclusive_scan(cnt, s_wave, s_total, &total);
    const int64_t slot0 = tile0 + (int64_t)threadIdx.x * SLOTS_PER_THREAD;
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (f[e]) sel_r[pos++] = (int32_t)(slot0 + e);
    running += total;
  }
  return running;
}

// One workgroup per partner pair (j, c): compact both ranks' flagged slots, then
// swap the r-th flagged slot of j with the r-th flagged slot of c.  Used while a
// rank holds few tiles; beyond that the three kernels below spread the tiles over
// the chip.
__global__ void __launch_bounds__(SWAP_THREADS) partner_swap_kernel(swap_args a) {
  __shared__ uint32_t s_wave[SWAP_WAVES];
  __shared__ uint32_t s_total;
  const int32_t q = blockIdx.x;
  const int32_t low = a.shift - 1;
  const int32_t v0 = ((q & ~low) << 1) | (q & low);
  const uint32_t j = a.sigma[v0];
  const uint32_t c = a.sigma[v0 | a.shift];
  const int64_t off_j = a.off[j], off_c = a.off[c];
  const int64_t n_j = a.off[j + 1] - off_j, n_c = a.off[c + 1] - off_c;
  int32_t* sel_j = a.sel + off_j;
  int32_t* sel_c = a.sel + off_c;
  const uint32_t cnt_j = compact_flagged(a, j, n_j, sel_j, s_wave, &s_total);
  const uint32_t cnt_c = compact_flagged(a, c, n_c, sel_c, s_wave, &s_total);
  __syncthreads();  // the sel lists written above are read by other threads below
  const uint32_t m = cnt_j < cnt_c ? cnt_j : cnt_c;
  for (uint32_t r = threadIdx.x; r < m; r += SWAP_THREADS) {
    int32_t* pa = a.idx + off_j + sel_j[r];
    int32_t* pb = a.idx + off_c + sel_c[r];
    const int32_t va = *pa, vb = *pb;
    *pa = vb;
    *pb = va;
  }
}

// ---- the same shuffle for ranks with many tiles: count, scatter, swap
// tile_counts[rank * max_tiles + tile] = flagged slots in that tile.
__global__ void __launch_bounds__(SWAP_THREADS) swap_count_kernel(swap_args a, uint32_t* tile_counts,
                                                                  int32_t max_tiles) {
  __shared__ uint32_t s_wave[SWAP_WAVES];
  __shared__ uint32_t s_total;
  const uint32_t rank = blockIdx.y, tile = blockIdx.x;
  const int64_t n_r = a.off[rank + 1] - a.off[rank];
  uint32_t f[4], total;
  const uint32_t cnt = tile_flags(a, rank, n_r, (int64_t)tile * SWAP_THREADS * SLOTS_PER_THREAD, f);
  (void)block_exclusive_scan(cnt, s_wave, &s_total, &total);
  if (threadIdx.x == 0) tile_counts[(int64_t)rank * max_tiles + tile] = total;
}

// Sum of counts[0 .. n) by the whole workgroup (n is small: tiles of one rank).
__device__ __forceinline__ uint32_t block_sum(const uint32_t* counts, int32_t n, uint32_t* s_wave, uint32_t* s_total) {
  uint32_t part = 0, total;
  for (int32_t i = threadIdx.x; i < n; i += SWAP_THREADS) part += counts[i];
  (void)block_exclusive_scan(part, s_wave, s_total, &total);
  return total;
}

__global__ void __launch_bounds__(SWAP_THREADS) swap_scatter_kernel(swap_args a, const uint32_t* tile_counts,
                                                                    int32_t max_tiles) {
  __shared__ uint32_t s_wave[SWAP_WAVES];
  __shared__ uint32_t s_total;
  const uint32_t rank = blockIdx.y, tile = blockIdx.x;
  const int64_t n_r = a.off[rank + 1] - a.off[rank];
  const int64_t tile0 = (int64_t)tile * SWAP_THREADS * SLOTS_PER_THREAD;
  if (tile0 >= n_r) return;  // uniform for the workgroup
  const uint32_t base = block_sum(tile_counts + (int64_t)rank * max_tiles, (int32_t)tile, s_wave, &s_total);
  uint32_t f[4], total;
  const uint32_t cnt = tile_flags(a, rank, n_r, tile0, f);
  uint32_t pos = base + block_exclusive_scan(cnt, s_wave, &s_total, &total);
  int32_t* sel_r = a.sel + a.off[rank];
  const int64_t slot0 = tile0 + (int64_t)threadIdx.x * SLOTS_PER_THREAD;
#pragma unroll
  for (int e = 0; e < 4; ++e)
    if (f[e]) sel_r[pos++] = (int32_t)(slot0 + e);
}

__global__ void __launch_bounds__(SWAP_THREADS) swap_apply_kernel(swap_args a, const uint32_t* tile_counts,
                                                                  int32_t max_tiles) {
  __shared__ uint32_t s_wave[SWAP_WAVES];
  __shared__ uint32_t s_total;
  const int32_t q = blockIdx.y;
  const int32_t low = a.shift - 1;
  const int32_t v0 = ((q & ~low) << 1) | (q & low);
  const uint32_t j = a.sigma[v0];
  const uint32_t c = a.sigma[v0 | a.shift];
  const uint32_t cnt_j = block_sum(tile_counts + (int64_t)j * max_tiles, max_tiles, s_wave, &s_total);
  const uint32_t cnt_c = block_sum(tile_counts + (int64_t)c * max_tiles, max_tiles, s_wave, &s_total);
  const uint32_t m = cnt_j < cnt_c ? cnt_j : cnt_c;
  const int64_t off_j = a.off[j], off_c = a.off[c];
  const int32_t* sel_j = a.sel + off_j;
  const int32_t* sel_c = a.sel + off_c;
  for (uint32_t r = blockIdx.x * SWAP_THREADS + threadIdx.x; r < m; r += gridDim.x * SWAP_THREADS) {
    int32_t* pa = a.idx + off_j + sel_j[r];
    int32_t* pb = a.idx + off_c + sel_c[r];
    const int32_t va = *pa, vb = *pb;
    *pa = vb;
    *pb = va;
  }
}

struct ring_args {
  int32_t* idx;
  int32_t* stage;      // scratch int32[p * batch]
  const int64_t* off;  // device int64[p+1]
  int64_t step;
  int32_t batch;
  int32_t p;
};

__device__ __forceinline__ int64_t ring_head(const ring_args& a, int32_t j) {
  const int64_t n_j = a.off[j + 1] - a.off[j];
  return ((a.step % n_j) * ((int64_t)a.batch % n_j)) % n_j;  // (step*batch) mod n_j
}

__device__ __forceinline__ int64_t ring_slot(const ring_args& a, int32_t j, int32_t r) {
  const int64_t n_j = a.off[j + 1] - a.off[j];
  return a.off[j] + (ring_head(a, j) + r) % n_j;
}

// Phase 1: every rank's batch at the head of its queue is copied out.
__global__ void __launch_bounds__(256) ring_gather_kernel(ring_args a) {
  const int32_t j = blockIdx.y;
  for (int32_t r = blockIdx.x * blockDim.x + threadIdx.x; r < a.batch; r += gridDim.x * blockDim.x)
    a.stage[(int64_t)j * a.batch + r] = a.idx[ring_slot(a, j, r)];
}
// Phase 2: rank j's freed slots take the batch of rank j-1, in order.
__global__ void __launch_bounds__(256) ring_scatter_kernel(ring_args a) {
  const int32_t j = blockIdx.y;
  const int32_t src = j == 0 ? a.p - 1 : j - 1;
  for (int32_t r = blockIdx.x * blockDim.x + threadIdx.x; r < a.batch; r += gridDim.x * blockDim.x)
    a.idx[ring_slot(a, j, r)] = a.stage[(int64_t)src * a.batch + r];
}

// Ring rotation of the sample payload itself: the same slot movement as the index
// ring, on rows of `words` W-sized words.  One thread owns word x of batch entry r
// for ALL ranks and walks the ring once (hold rank p-1's word, then for j = 0..p-1
// swap the held word into rank j's slot), so every byte is read once and written
// once, in place, without staging.  General form (4-byte words, any alignment).
template <typename Wd>
__global__ void __launch_bounds__(256) ring_payload_kernel(ring_args a, Wd* payload, int64_t words) {
  const int64_t total = (int64_t)a.batch * words;
  for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (int64_t)gridDim.x * blockDim.x) {
    const int32_t r = (int32_t)(t / words);
    const int64_t x = t - (int64_t)r * words;
    Wd held = __builtin_nontemporal_load(payload + ring_slot(a, a.p - 1, r) * words + x);
    Wd cur = __builtin_nontemporal_load(payload + ring_slot(a, 0, r) * words + x);
    for (int32_t j = 0; j < a.p; ++j) {
      Wd* dst = payload + ring_slot(a, j, r) * words + x;
      Wd nxt = cur;
      if (j + 1 < a.p) nxt = __builtin_nontemporal_load(payload + ring_slot(a, j + 1, r) * words + x);
      __builtin_nontemporal_store(held, dst);
      held = cur;
      cur = nxt;
    }
  }
}

// Default form for 16-byte words: the same walk with the chip in step.  A workgroup of
// W wavefronts owns W*U tiles (64 words = 1 KB each) `step` tiles apart -- 32 KB apart
// in memory wherever they fall into one sample, i.e. in the same DRAM channel.  It takes
// the ranks D at a time: D loads per word in flight, then the D stores (every store
// follows the load of the same address in program order), then a barrier, so that
// only D ranks' batches are streamed at a time instead of all p.  The queue heads
// ((step*batch) mod n_j: three 64-bit divisions) are worked out once per workgroup into
// LDS, so a hop costs no division.
struct ring_walk_shape {
  int32_t step;
  int32_t barrier;
};

template <int U, int D>
__global__ void __launch_bounds__(512 / U) ring_payload_walk_kernel(ring_args a, v4f* payload, int64_t words,
                                                                     ring_walk_shape ws) {
  const int64_t total = (int64_t)a.batch * words;
  int32_t r[U];
  int64_t x[U];
  bool on[U];
  {
    const int64_t bx = blockIdx.x, step = ws.step;
    const int64_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63, W = blockDim.x >> 6;
    const int64_t tile0 = (bx / step) * (step * W * U) + bx % step + wave * U * step;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t t = (tile0 + u * step) * 64 + lane;
      on[u] = t < total;
      r[u] = on[u] ? (int32_t)(t / words) : 0;
      x[u] = t - (int64_t)r[u] * words;
    }
  }
  __shared__ int64_t s_head[GG_MAX_RANKS];
  for (int32_t j = threadIdx.x; j < a.p; j += blockDim.x) s_head[j] = ring_head(a, j);
  __syncthreads();
  // word of batch entry r[u] in rank j: head + r < 2 n_j, so one conditional subtraction wraps it
  auto word_at = [&](int32_t j, int u) -> v4f* {
    const int64_t off_j = a.off[j], n_j = a.off[j + 1] - off_j;
    int64_t slot = s_head[j] + r[u];
    if (slot >= n_j) slot -= n_j;
    return payload + (off_j + slot) * words + x[u];
  };
  v4f held[U];
#pragma unroll
  for (int u = 0; u < U; ++u)
    if (on[u]) held[u] = __builtin_nontemporal_load(word_at(a.p - 1, u));
  const int32_t last = a.p - 1;  // rank p-1 was read above and is written after the loop
  for (int32_t j0 = 0; j0 < last; j0 += D) {
    v4f cur[D][U];
    v4f* ptr[D][U];
#pragma unroll
    for (int d = 0; d < D; ++d) {
      if (j0 + d < last) {  // uniform
#pragma unroll
        for (int u = 0; u < U; ++u) {
          ptr[d][u] = word_at(j0 + d, u);
          if (on[u]) cur[d][u] = __builtin_nontemporal_load(ptr[d][u]);
        }
      }
    }
#pragma unroll
    for (int d = 0; d < D; ++d) {
      if (j0 + d < last) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
          if (on[u]) __builtin_nontemporal_store(held[u], ptr[d][u]);
          held[u] = cur[d][u];
        }
      }
    }
    if (ws.barrier) __syncthreads();  // uniform trip count: every wavefront walks all p ranks
  }
#pragma unroll
  for (int u = 0; u < U; ++u)
    if (on[u]) __builtin_nontemporal_store(held[u], word_at(last, u));
}

// Make the device copy of rank_offsets current and the scratch large enough.
int prepare(gg_ctx* ctx, const int64_t* off, hipStream_t s, int64_t scratch_words) {
  const int32_t p = ctx->cfg.p;
  if (!ctx->d_offsets) {
    if (hipMalloc((void**)&ctx->d_offsets, (size_t)(p + 1) * sizeof(int64_t)) != hipSuccess ||
        hipHostMalloc((void**)&ctx->h_offsets_pinned, (size_t)(p + 1) * sizeof(int64_t), hipHostMallocDefault) !=
            hipSuccess) {
      (void)hipGetLastError();
      return GG_ERR_NOMEM;
    }
  }
  if (ctx->offsets_cached.size() != (size_t)(p + 1) ||
      memcmp(ctx->offsets_cached.data(), off, (size_t)(p + 1) * sizeof(int64_t)) != 0) {
    // an earlier upload may still be reading the staging buffer
    GG_HIP_TRY(hipDeviceSynchronize());
    memcpy(ctx->h_offsets_pinned, off, (size_t)(p + 1) * sizeof(int64_t));
    GG_HIP_TRY(hipMemcpyAsync(ctx->d_offsets, ctx->h_offsets_pinned, (size_t)(p + 1) * sizeof(int64_t),
                              hipMemcpyHostToDevice, s));
    ctx->offsets_cached.assign(off, off + p + 1);
  }
  if (scratch_words > ctx->scratch_cap) {
    GG_HIP_TRY(hipDeviceSynchronize());
    if (ctx->d_scratch) (void)hipFree(ctx->d_scratch);
    ctx->d_scratch = nullptr;
    ctx->scratch_cap = 0;
    if (hipMalloc((void**)&ctx->d_scratch, (size_t)scratch_words * sizeof(int32_t)) != hipSuccess) {
      (void)hipGetLastError();
      return GG_ERR_NOMEM;
    }
    ctx->scratch_cap = scratch_words;
  }
  return GG_OK;
}

// Argument checks shared by both index-shuffle entry points; fills the per-call sizes.
struct shuffle_sizes {
  int64_t min_n, max_n, n_total;
  int32_t max_tiles;   // tiles of the largest rank (4096 slots each)
  int64_t counts_at;   // word offset of the per-tile counts behind the flagged-slot lists
  int64_t words;       // scratch words needed in all
};

int check_shuffle(const gg_ctx* ctx, int64_t step, int32_t mode, const int32_t* idx, const int64_t* rank_offsets,
                  int32_t batch, shuffle_sizes* out) {
  if (!ctx || !idx || !rank_offsets || step < 0) return GG_ERR_ARG;
  if (mode != GG_SHUF_PARTNER_SWAP && mode != GG_SHUF_RING) return GG_ERR_ARG;
  if (!gg_aligned(idx, 4)) return GG_ERR_ALIGN;
  const int32_t p = ctx->cfg.p;
  if (rank_offsets[0] != 0) return GG_ERR_ARG;
  int64_t min_n = INT64_MAX, max_n = 0;
  for (int32_t j = 0; j < p; ++j) {
    const int64_t n_j = rank_offsets[j + 1] - rank_offsets[j];
    if (n_j < 0 || n_j > 0x7fffffffLL) return GG_ERR_ARG;
    if (n_j < min_n) min_n = n_j;
    if (n_j > max_n) max_n = n_j;
  }
  if (rank_offsets[p] > (int64_t(1) << 34)) return GG_ERR_ARG;
  if (mode == GG_SHUF_PARTNER_SWAP) {
    if (ctx->cfg.topology != GG_TOPO_HYPERCUBE) return GG_ERR_UNSUPPORTED;  // needs an involution
  } else {
    if (batch < 0 || batch > min_n) return GG_ERR_ARG;
  }
  const int64_t per_tile = (int64_t)SWAP_THREADS * SLOTS_PER_THREAD;
  out->min_n = min_n;
  out->max_n = max_n;
  out->n_total = rank_offsets[p];
  out->max_tiles = (int32_t)((max_n + per_tile - 1) / per_tile);
  // scratch: flagged-slot lists (one word per slot at most; the ring's staged batches fit the
  // same words, p * batch <= n_total), then per-tile counts
  out->counts_at = (rank_offsets[p] + 3) / 4 * 4;
  out->words = out->counts_at + (int64_t)p * (out->max_tiles > 0 ? out->max_tiles : 1);
  return gg_check_ctx_device(ctx);
}

// The launches of one index shuffle; d_off and scratch are ready on stream s.
int enqueue_shuffle(gg_ctx* ctx, int64_t step, int32_t mode, int32_t* idx, int32_t batch, const shuffle_sizes& sz,
                    const int64_t* d_off, int32_t* scratch, hipStream_t s) {
  const int32_t p = ctx->cfg.p;
  if (mode == GG_SHUF_PARTNER_SWAP) {
    const int32_t k = (int32_t)(step % ctx->L);
    const int32_t r = (int32_t)((step / ctx->L) % ctx->R);
    swap_args a;
    a.idx = idx;
    a.sel = scratch;
    a.off = d_off;
    a.sigma = ctx->d_sigma + (size_t)r * p;
    a.shift = int32_t(1) << k;
    a.step32 = (uint32_t)((uint64_t)step & 0xffffffffu);
    a.k0 = (uint32_t)ctx->cfg.seed;
    a.k1 = (uint32_t)(ctx->cfg.seed >> 32);
    if (sz.max_tiles <= 8) {
      // few tiles per rank: one workgroup per pair does everything in one launch
      hipLaunchKernelGGL(partner_swap_kernel, dim3(p / 2), dim3(SWAP_THREADS), 0, s, a);
      GG_HIP_TRY(hipGetLastError());
    } else {
      // every (tile, rank) count is written by swap_count_kernel before it is read: nothing to clear
      uint32_t* counts = reinterpret_cast<uint32_t*>(scratch + sz.counts_at);
      const int32_t max_tiles = sz.max_tiles;
      hipLaunchKernelGGL(swap_count_kernel, dim3(max_tiles, p), dim3(SWAP_THREADS), 0, s, a, counts, max_tiles);
      GG_HIP_TRY(hipGetLastError());
      hipLaunchKernelGGL(swap_scatter_kernel, dim3(max_tiles, p), dim3(SWAP_THREADS), 0, s, a, counts, max_tiles);
      GG_HIP_TRY(hipGetLastError());
      int64_t bx = sz.max_n / (8 * SWAP_THREADS) + 1;  // about one thread per expected swap
      if (bx > 4096) bx = 4096;
      hipLaunchKernelGGL(swap_apply_kernel, dim3((unsigned)bx, p / 2), dim3(SWAP_THREADS), 0, s, a, counts, max_tiles);
      GG_HIP_TRY(hipGetLastError());
    }
  } else {
    if (batch == 0) return GG_OK;
    ring_args a;
    a.idx = idx;
    a.stage = scratch;
      a.off = d_off;
    a.step = step;
    a.batch = batch;
    a.p = p;
    int32_t bx = (batch + 255) / 256;
    if (bx > 1024) bx = 1024;
    hipLaunchKernelGGL(ring_gather_kernel, dim3(bx, p), dim3(256), 0, s, a);
    GG_HIP_TRY(hipGetLastError());
    hipLaunchKernelGGL(ring_scatter_kernel, dim3(bx, p), dim3(256), 0, s, a);
    GG_HIP_TRY(hipGetLastError());
  }
  return GG_OK;
}

std::mutex g_scratch_lock;
unsigned char* g_scratch_ptr[NOALLOC_MAX_DEVICES];  // per device: address of its copy of `scratch`, or null

// Rank offsets travel to the device in the kernel arguments, 256 at a time: no staging
// buffer, no copy engine, nothing to allocate.
struct offsets_block {
  int64_t v[OFFSETS_PER_LAUNCH];
};
__global__ void __launch_bounds__(OFFSETS_PER_LAUNCH) put_offsets_kernel(offsets_block b, int32_t base, int32_t count,
                                                                         int64_t* dst) {
  const int32_t i = threadIdx.x;
  if (i < count) dst[base + i] = b.v[i];
}

}  // namespace

int gg_static_scratch_setup(int device) {
  if (device < 0 || device >= NOALLOC_MAX_DEVICES) return GG_ERR_ARG;
  std::lock_guard<std::mutex> hold(g_scratch_lock);
  if (g_scratch_ptr[device]) return GG_OK;
  void* ptr = nullptr;
  if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
    (void)hipGetLastError();
    return GG_ERR_HIP;
  }
  g_scratch_ptr[device] = static_cast<unsigned char*>(ptr);
  return GG_OK;
}

extern "C" int gg_shuffle(gg_ctx* ctx, int64_t step, int32_t mode, int32_t* idx, const int64_t* rank_offsets,
                          int32_t batch, void* stream) {
  shuffle_sizes sz;
  int rc = check_shuffle(ctx, step, mode, idx, rank_offsets, batch, &sz);
  if (rc != GG_OK) return rc;
  if (sz.n_total == 0) return GG_OK;
  hipStream_t s = (hipStream_t)stream;
  rc = prepare(ctx, rank_offsets, s, sz.words);
  if (rc != GG_OK) return rc;
  return enqueue_shuffle(ctx, step, mode, idx, batch, sz, ctx->d_offsets, ctx->d_scratch, s);
}

extern "C" int gg_shuffle_noalloc(gg_ctx* ctx, int64_t step, int32_t mode, int32_t* idx, const int64_t* rank_offsets,
                                  int32_t batch, void* stream) {
  shuffle_sizes sz;
  int rc = check_shuffle(ctx, step, mode, idx, rank_offsets, batch, &sz);
  if (rc != GG_OK) return rc;
  const int32_t p = ctx->cfg.p;
  if (sz.n_total > GG_NOALLOC_MAX_INDICES) return GG_ERR_LIMIT;
  if ((int64_t)p * sz.max_tiles > GG_NOALLOC_MAX_TILE_COUNTS) return GG_ERR_LIMIT;
  if (sz.n_total == 0) return GG_OK;
  unsigned char* base = ctx->device < NOALLOC_MAX_DEVICES ? g_scratch_ptr[ctx->device] : nullptr;
  if (!base) return GG_ERR_HIP;  // gg_init could not resolve the array on this device
  hipStream_t s = (hipStream_t)stream;
  int64_t* d_off = reinterpret_cast<int64_t*>(base);
  int32_t* words = reinterpret_cast<int32_t*>(base + NOALLOC_OFF_BYTES);
  for (int32_t at = 0; at <= p; at += OFFSETS_PER_LAUNCH) {
    offsets_block b;
    const int32_t count = p + 1 - at < OFFSETS_PER_LAUNCH ? p + 1 - at : OFFSETS_PER_LAUNCH;
    for (int32_t i = 0; i < OFFSETS_PER_LAUNCH; ++i) b.v[i] = i < count ? rank_offsets[at + i] : 0;
    hipLaunchKernelGGL(put_offsets_kernel, dim3(1), dim3(OFFSETS_PER_LAUNCH), 0, s, b, at, count, d_off);
    GG_HIP_TRY(hipGetLastError());
  }
  return enqueue_shuffle(ctx, step, mode, idx, batch, sz, d_off, words, s);
}

extern "C" int gg_shuffle_payload(gg_ctx* ctx, int64_t step, void* payload, int64_t sample_bytes,
                                  const int64_t* rank_offsets, int32_t batch, void* stream) {
  if (!ctx || !payload || !rank_offsets || step < 0 || sample_bytes <= 0 || sample_bytes % 4) return GG_ERR_ARG;
  if (!gg_aligned(payload, 4)) return GG_ERR_ALIGN;
  const int32_t p = ctx->cfg.p;
  if (rank_offsets[0] != 0) return GG_ERR_ARG;
  int64_t min_n = INT64_MAX;
  for (int32_t j = 0; j < p; ++j) {
    const int64_t n_j = rank_offsets[j + 1] - rank_offsets[j];
    if (n_j < 0 || n_j > 0x7fffffffLL) return GG_ERR_ARG;
    if (n_j < min_n) min_n = n_j;
  }
  if (batch < 0 || batch > min_n) return GG_ERR_ARG;
  if (rank_offsets[p] > (int64_t(1) << 34) || sample_bytes > (int64_t(1) << 30)) return GG_ERR_ARG;
  int rc = gg_check_ctx_device(ctx);
  if (rc != GG_OK) return rc;
  if (batch == 0) return GG_OK;
  hipStream_t s = (hipStream_t)stream;
  rc = prepare(ctx, rank_offsets, s, 0);
  if (rc != GG_OK) return rc;
  ring_args a;
  a.idx = nullptr;
  a.stage = nullptr;
  a.off = ctx->d_offsets;
  a.step = step;
  a.batch = batch;
  a.p = p;
  const bool vec = gg_aligned(payload, 16) && sample_bytes % 16 == 0;
  const int64_t words = vec ? sample_bytes / 16 : sample_bytes / 4;
  // measured best for 64 ranks x 32 samples of 192 KB: 8 wavefronts x 1 chunk, 2 ranks per barrier, no cap
  const gg_walk_shape own{1, 8, 32, 0, 1, 1};
  const gg_walk_launch wl = gg_walk_geometry(ctx, own, 4, ((int64_t)batch * words + 63) / 64);
  if (vec && wl.grid_x > 0) {
    ring_walk_shape ws{wl.shape.step, wl.shape.barrier};
    const uint32_t lds = wl.lds_bytes;
    const int U = wl.shape.chunks;
    const dim3 grid((unsigned)wl.grid_x), block(64u * (unsigned)wl.shape.waves);
#define GG_RING_CASE(UU, DD) \
  hipLaunchKernelGGL((ring_payload_walk_kernel<UU, DD>), grid, block, lds, s, a, (v4f*)payload, words, ws)
#define GG_RING_U(DD)             \
  switch (U) {                    \
    case 1: GG_RING_CASE(1, DD); break; \
    case 2: GG_RING_CASE(2, DD); break; \
    default: GG_RING_CASE(4, DD); break; \
  }
    switch (wl.shape.group_log2) {
      case 0: GG_RING_U(1) break;
      case 1: GG_RING_U(2) break;
      case 2: GG_RING_U(4) break;
      default: GG_RING_U(8) break;
    }
#undef GG_RING_U
#undef GG_RING_CASE
  } else {
    int64_t blocks = ((int64_t)batch * words + 255) / 256;
    if (blocks > 0x7fffffffLL) blocks = 0x7fffffffLL;
    if (vec)
      hipLaunchKernelGGL(ring_payload_kernel<v4f>, dim3((unsigned)blocks), dim3(256), 0, s, a, (v4f*)payload, words);
    else
      hipLaunchKernelGGL(ring_payload_kernel<float>, dim3((unsigned)blocks), dim3(256), 0, s, a, (float*)payload, words);
  }
  GG_HIP_TRY(hipGetLastError());
  return GG_OK;
}
