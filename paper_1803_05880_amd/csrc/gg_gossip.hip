// Fused momentum-SGD update + pairwise model average (Eq. 1-2, Sec. 6) for all
// virtual ranks in one launch, and the local update alone (Sec. 4.1).
//
// Memory-bound streaming kernels: per rank and parameter the step must read
// w, g, m (12 B) and write w, m (8 B).  One thread owns the same 16-byte chunk of
// BOTH partners (hypercube) or of a whole partner cycle (dissemination), so the
// partner's post-update weights never travel through memory: 20 B / rank /
// parameter in every mode, in place, race-free by construction.
//
// Arithmetic is fp32 with every operation rounded on its own; contraction into
// fused multiply-add is switched off here and on the command line.
#pragma clang fp contract(off)

#include "gg_internal.h"

namespace {

enum { MODE_SYNC = 0, MODE_STALE = 1, MODE_GRAD = 2 };

struct step_args {
  float* w;
  const float* g;
  float* m;
  float* wn;              // where new weights go (== w when in place)
  int64_t stride;         // elements between consecutive ranks
  gg_range rng;           // work items, in units of the access type V
  int64_t tiles;          // tiles per grid row
  int32_t shift;          // 2^k of the current phase
  int32_t p;
  float lr, mu;
};

// World ranks (j, c) of the step's pairs, one packed entry per grid row q.  Passed
// by value so that a workgroup finds its two ranks with one scalar load from the
// kernel-argument segment, issued together with the other arguments: workgroups
// here live for a microsecond or two and a dependent table lookup in global
// memory would be a visible part of that.
struct pair_table {
  uint32_t jc[GG_MAX_RANKS / 2];  // j | c << 10 | tile shift << 20 (lean kernel only)
};

// Streaming 16-byte store with the write-through scope bits set next to the
// non-temporal hint: measured about 1 % faster than the hint alone for this
// read-modify-write stream (the line just read is never needed again on chip).
// A store of more than 8 bytes reads its data registers after it has issued; a
// vector ALU instruction that overwrites them needs two wait states in between.
// The compiler pads its own stores but cannot see into this one, hence the s_nop.
__device__ __forceinline__ void st_stream(v4f* ptr, v4f val) {
  asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1 nt\n\ts_nop 1" : : "v"(ptr), "v"(val) : "memory");
}

// v = mu*m + lr*g ; returns T = w - v.  Three roundings for v, one for T.
template <typename V>
__device__ __forceinline__ V local_update(V w, V g, V m, float lr, float mu, V& v) {
  const V a = m * mu;
  const V b = g * lr;
  v = a + b;
  return w - v;
}

// ---------------------------------------------------------------- hypercube pairs
// Grid row q is one of the p/2 pairs; the host lists their world ranks (j, c).
template <typename V, int MODE, int U, bool NT, bool GUARD>
__device__ __forceinline__ void pair_tile(const step_args& a, int64_t x0, const V* wj, const V* gj, V* mj,
                                          const V* wc, const V* gc, V* mc, V* nj, V* nc) {
  V Wj[U], Gj[U], Mj[U], Wc[U], Gc[U], Mc[U];
  int64_t idx[U];
  bool on[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int64_t x = x0 + (int64_t)u * blockDim.x;
    on[u] = !GUARD || x < a.rng.count;
    idx[u] = gg_item_index(a.rng, x);
    if (on[u]) {
      Wj[u] = gg_ld<NT>(wj + idx[u]);
      Wc[u] = gg_ld<NT>(wc + idx[u]);
      Gj[u] = gg_ld<NT>(gj + idx[u]);
      Gc[u] = gg_ld<NT>(gc + idx[u]);
      Mj[u] = gg_ld<NT>(mj + idx[u]);
      Mc[u] = gg_ld<NT>(mc + idx[u]);
    }
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    if (!on[u]) continue;
    V vj, vc, outj, outc;
    if (MODE == MODE_GRAD) {
      const V gbar = (Gj[u] + Gc[u]) * 0.5f;  // addition commutes: both sides see the same bits
      outj = local_update(Wj[u], gbar, Mj[u], a.lr, a.mu, vj);
      outc = local_update(Wc[u], gbar, Mc[u], a.lr, a.mu, vc);
    } else {
      const V Tj = local_update(Wj[u], Gj[u], Mj[u], a.lr, a.mu, vj);
      const V Tc = local_update(Wc[u], Gc[u], Mc[u], a.lr, a.mu, vc);
      if (MODE == MODE_SYNC) {
        outj = (Tj + Tc) * 0.5f;
        outc = outj;
      } else {  // staleness 1: the partner contributes the weights it held on entry
        outj = (Tj + Wc[u]) * 0.5f;
        outc = (Tc + Wj[u]) * 0.5f;
      }
    }
    gg_st<NT>(nj + idx[u], outj);
    gg_st<NT>(nc + idx[u], outc);
    gg_st<NT>(mj + idx[u], vj);
    gg_st<NT>(mc + idx[u], vc);
  }
}

template <typename V, int MODE, int U, bool NT>
__global__ void __launch_bounds__(256) gossip_pair_kernel(step_args a, pair_table pt) {
  const uint32_t jc = pt.jc[blockIdx.y];
  const int64_t j = jc & 0x3ffu;
  const int64_t c = (jc >> 10) & 0x3ffu;
  const V* wj = reinterpret_cast<const V*>(a.w + j * a.stride);
  const V* wc = reinterpret_cast<const V*>(a.w + c * a.stride);
  const V* gj = reinterpret_cast<const V*>(a.g + j * a.stride);
  const V* gc = reinterpret_cast<const V*>(a.g + c * a.stride);
  V* mj = reinterpret_cast<V*>(a.m + j * a.stride);
  V* mc = reinterpret_cast<V*>(a.m + c * a.stride);
  V* nj = reinterpret_cast<V*>(a.wn + j * a.stride);
  V* nc = reinterpret_cast<V*>(a.wn + c * a.stride);
  const int64_t per_tile = (int64_t)blockDim.x * U;
  int64_t tile = blockIdx.x;  // the grid never has more columns than tiles
  do {
    const int64_t x0 = tile * per_tile + threadIdx.x;
    if ((tile + 1) * per_tile <= a.rng.count)
      pair_tile<V, MODE, U, NT, false>(a, x0, wj, gj, mj, wc, gc, mc, nj, nc);
    else
      pair_tile<V, MODE, U, NT, true>(a, x0, wj, gj, mj, wc, gc, mc, nj, nc);
    tile += gridDim.x;
  } while (tile < a.tiles);
}

// Lean form of the same kernel for the default launch shape: one wavefront per
// workgroup, one 16-byte chunk per thread, one tile per workgroup, no ragged
// range.  Workgroups live for about a microsecond, so everything that delays the
// first load (extra argument fetches, loop set-up) shows up in the bandwidth.
template <int MODE, bool NT>
__global__ void __launch_bounds__(64) gossip_pair_lean_kernel(step_args a, pair_table pt) {
  const uint32_t jc = pt.jc[blockIdx.y];
  const int64_t j = jc & 0x3ffu;
  const int64_t c = (jc >> 10) & 0x3ffu;
  // Tiles are laid so that rank j's 1 KB wavefront accesses start on 1 KB boundaries even
  // when the rows themselves do not (the host passes the shift, 0 for aligned layouts).
  const int64_t i = a.rng.lo + (int64_t)blockIdx.x * 64 + threadIdx.x - (int64_t)(jc >> 20);
  if (i < a.rng.lo || i >= a.rng.lo + a.rng.count) return;
  const v4f* wj = reinterpret_cast<const v4f*>(a.w + j * a.stride) + i;
  const v4f* wc = reinterpret_cast<const v4f*>(a.w + c * a.stride) + i;
  const v4f* gj = reinterpret_cast<const v4f*>(a.g + j * a.stride) + i;
  const v4f* gc = reinterpret_cast<const v4f*>(a.g + c * a.stride) + i;
  v4f* mj = reinterpret_cast<v4f*>(a.m + j * a.stride) + i;
  v4f* mc = reinterpret_cast<v4f*>(a.m + c * a.stride) + i;
  v4f* nj = reinterpret_cast<v4f*>(a.wn + j * a.stride) + i;
  v4f* nc = reinterpret_cast<v4f*>(a.wn + c * a.stride) + i;
  const v4f Wj = gg_ld<NT>(wj), Wc = gg_ld<NT>(wc), Gj = gg_ld<NT>(gj), Gc = gg_ld<NT>(gc), Mj = gg_ld<NT>(mj), Mc = gg_ld<NT>(mc);
  v4f vj, vc, outj, outc;
  if (MODE == MODE_GRAD) {
    const v4f gbar = (Gj + Gc) * 0.5f;
    outj = local_update(Wj, gbar, Mj, a.lr, a.mu, vj);
    outc = local_update(Wc, gbar, Mc, a.lr, a.mu, vc);
  } else {
    const v4f Tj = local_update(Wj, Gj, Mj, a.lr, a.mu, vj);
    const v4f Tc = local_update(Wc, Gc, Mc, a.lr, a.mu, vc);
    if (MODE == MODE_SYNC) {
      outj = (Tj + Tc) * 0.5f;
      outc = outj;
    } else {
      outj = (Tj + Wc) * 0.5f;
      outc = (Tc + Wj) * 0.5f;
    }
  }
  if (NT) {
    st_stream(nj, outj);
    st_stream(nc, outc);
    st_stream(mj, vj);
    st_stream(mc, vc);
  } else {
    gg_st<false>(nj, outj);
    gg_st<false>(nc, outc);
    gg_st<false>(mj, vj);
    gg_st<false>(mc, vc);
  }
}

// ------------------------------------------------------------ dissemination cycles
// At phase k virtual rank v receives from v - 2^k (mod p).  The map splits the
// ranks into gcd(p, 2^k) cycles v0, v0+2^k, v0+2*2^k, ...; grid row = cycle.  One
// thread walks its cycle for one chunk and carries the previous rank's
// contribution in registers, so each rank's w, g, m are read once and written
// once, in place.
//
// Communicator row (virtual -> world rank) for the cycle walk, two ranks per word,
// passed by value like pair_table: a hop's rank comes from one scalar load in the
// kernel-argument segment instead of an LDS copy that every short-lived workgroup
// would first have to fill behind a barrier.
struct rank_table {
  uint32_t r2[GG_MAX_RANKS / 2];
};

// General form (any launch shape, scalar instantiation for unaligned buffers): one
// thread walks its cycle for U chunks with two ranks of look-ahead.
template <typename V, int MODE, int U, bool NT>
__global__ void __launch_bounds__(256) gossip_cycle_kernel(step_args a, int32_t cycle_len, rank_table rt) {
  const int32_t v0 = blockIdx.y;
  // world rank at hop t of this cycle: virtual rank (v0 + t*shift) mod p
  auto rank_at = [&](int32_t t) -> int64_t {
    const uint32_t v = (uint32_t)((v0 + t * a.shift) % a.p);
    return (rt.r2[v >> 1] >> ((v & 1u) * 16u)) & 0xffffu;
  };
  const int64_t per_tile = (int64_t)blockDim.x * U;
  for (int64_t tile = blockIdx.x; tile < a.tiles; tile += gridDim.x) {
    int64_t idx[U];
    bool on[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t x = tile * per_tile + (int64_t)u * blockDim.x + threadIdx.x;
      on[u] = x < a.rng.count;
      idx[u] = gg_item_index(a.rng, x);
    }
    auto load = [&](int64_t rank, V* w, V* g, V* m) {
      const V* pw = reinterpret_cast<const V*>(a.w + rank * a.stride);
      const V* pg = reinterpret_cast<const V*>(a.g + rank * a.stride);
      const V* pm = reinterpret_cast<const V*>(a.m + rank * a.stride);
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (on[u]) {
          w[u] = gg_ld<NT>(pw + idx[u]);
          g[u] = gg_ld<NT>(pg + idx[u]);
          m[u] = gg_ld<NT>(pm + idx[u]);
        }
    };
    auto store_one = [&](float* base, int64_t row, const V* val) {
      V* ptr = reinterpret_cast<V*>(base + row * a.stride);
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (on[u]) gg_st<NT>(ptr + idx[u], val[u]);
    };

    // first rank of the cycle: its new weights need the LAST rank's contribution
    V fw[U], fg[U], fm[U], fT[U];
    V carry[U];  // what the previous rank on the walk contributes to the next one
    const int64_t rank0 = rank_at(0);
    load(rank0, fw, fg, fm);
    if (MODE == MODE_GRAD) {
#pragma unroll
      for (int u = 0; u < U; ++u) carry[u] = fg[u];
    } else {
      V v[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        fT[u] = local_update(fw[u], fg[u], fm[u], a.lr, a.mu, v[u]);
        carry[u] = (MODE == MODE_SYNC) ? fT[u] : fw[u];
      }
      store_one(a.m, rank0, v);
    }

    int64_t rank = rank_at(1);
    int64_t rank_1 = rank_at(2);
    V cw[U], cg[U], cm[U];
    V n1w[U], n1g[U], n1m[U];
    if (1 < cycle_len) load(rank, cw, cg, cm);
    if (2 < cycle_len) load(rank_1, n1w, n1g, n1m);
    for (int32_t t = 1; t < cycle_len; ++t) {
      const int64_t rank_2 = rank_at(t + 2);
      V n2w[U], n2g[U], n2m[U];
      if (t + 2 < cycle_len) load(rank_2, n2w, n2g, n2m);
      V v[U], out[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (MODE == MODE_GRAD) {
          const V gbar = (cg[u] + carry[u]) * 0.5f;
          out[u] = local_update(cw[u], gbar, cm[u], a.lr, a.mu, v[u]);
          carry[u] = cg[u];
        } else {
          const V T = local_update(cw[u], cg[u], cm[u], a.lr, a.mu, v[u]);
          out[u] = (T + carry[u]) * 0.5f;
          carry[u] = (MODE == MODE_SYNC) ? T : cw[u];
        }
      }
      store_one(a.m, rank, v);
      store_one(a.wn, rank, out);
#pragma unroll
      for (int u = 0; u < U; ++u) {
        cw[u] = n1w[u];
        cg[u] = n1g[u];
        cm[u] = n1m[u];
        n1w[u] = n2w[u];
        n1g[u] = n2g[u];
        n1m[u] = n2m[u];
      }
      rank = rank_1;
      rank_1 = rank_2;
    }
    // close the cycle
    V out[U];
    if (MODE == MODE_GRAD) {
      V v[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const V gbar = (fg[u] + carry[u]) * 0.5f;
        out[u] = local_update(fw[u], gbar, fm[u], a.lr, a.mu, v[u]);
      }
      store_one(a.m, rank0, v);
    } else {
#pragma unroll
      for (int u = 0; u < U; ++u) out[u] = (fT[u] + carry[u]) * 0.5f;
    }
    store_one(a.wn, rank0, out);
  }
}

// Default form for 16-byte aligned buffers.  Three things, each measured, set it apart:
//  * One wavefront walks the cycle once for U tiles, a workgroup of W wavefronts for
//    W*U tiles (default 4 x 1), and a barrier after every hop keeps the workgroup on the
//    same rank.
//  * The workgroup's tiles are `step` tiles apart (32 = 32 KB by default).  Device
//    memory interleaves consecutive 128-byte pieces over its channels, so addresses
//    32 KB apart fall into the same channel and, eight of them, into one DRAM row: the
//    workgroup touches every row it opens W*U times at once instead of once.  Workgroup
//    bx handles tiles (bx / step) * step*W*U + bx % step + i * step, i < W*U, so that
//    consecutive workgroups still take consecutive tiles.
//  * Few workgroups are resident per CU (the launch reserves LDS it never touches).
// A cycle through all 64 ranks then streams at 0.96 of the pair kernel's rate, where
// one tile per wavefront gave 0.78 (every rank of the cycle open somewhere on the chip,
// each DRAM row opened for one 128-byte piece at a time).
struct walk_args {
  int32_t cycle_len;
  int32_t hop_barrier;
  int32_t step;  // tiles between two tiles of one workgroup
};

template <int MODE, int U>
__global__ void __launch_bounds__(512 / U) gossip_cycle_walk_kernel(step_args a, walk_args wa, rank_table rt) {
  const int32_t v0 = blockIdx.y;
  auto rank_at = [&](int32_t t) -> int64_t {
    const uint32_t v = (uint32_t)((v0 + t * a.shift) % a.p);
    return (rt.r2[v >> 1] >> ((v & 1u) * 16u)) & 0xffffu;
  };
  int64_t idx[U];
  bool on[U];
  {
    const int64_t bx = blockIdx.x, step = wa.step;
    const int64_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63, W = blockDim.x >> 6;
    const int64_t tile0 = (bx / step) * (step * W * U) + bx % step + wave * U * step;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t x = (tile0 + u * step) * 64 + lane;
      on[u] = x < a.rng.count;
      idx[u] = a.rng.lo + x;
    }
  }
  auto load = [&](int64_t rank, v4f* w, v4f* g, v4f* m) {
    const v4f* pw = reinterpret_cast<const v4f*>(a.w + rank * a.stride);
    const v4f* pg = reinterpret_cast<const v4f*>(a.g + rank * a.stride);
    const v4f* pm = reinterpret_cast<const v4f*>(a.m + rank * a.stride);
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (on[u]) {
        w[u] = gg_ld<true>(pw + idx[u]);
        g[u] = gg_ld<true>(pg + idx[u]);
        m[u] = gg_ld<true>(pm + idx[u]);
      }
  };
  auto store_one = [&](float* base, int64_t row, const v4f* val) {
    v4f* ptr = reinterpret_cast<v4f*>(base + row * a.stride);
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (on[u]) st_stream(ptr + idx[u], val[u]);
  };

  // first rank of the cycle: its new weights need the LAST rank's contribution, so what
  // closes the cycle stays in registers until the walk comes round
  v4f first[U];      // SYNC/STALE: T of the first rank; GRAD: its gradient
  v4f fw[U], fm[U];  // GRAD only: the first rank's weights and momentum
  v4f carry[U];      // what the previous rank on the walk contributes to the next one
  const int64_t rank0 = rank_at(0);
  {
    v4f w0[U], g0[U], m0[U], v[U];
    load(rank0, w0, g0, m0);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (MODE == MODE_GRAD) {
        first[u] = g0[u];
        fw[u] = w0[u];
        fm[u] = m0[u];
        carry[u] = g0[u];
      } else {
        first[u] = local_update(w0[u], g0[u], m0[u], a.lr, a.mu, v[u]);
        carry[u] = (MODE == MODE_SYNC) ? first[u] : w0[u];
      }
    }
    if (MODE != MODE_GRAD) store_one(a.m, rank0, v);
  }
  for (int32_t t = 1; t < wa.cycle_len; ++t) {
    // every wavefront of the workgroup takes this branch the same number of times
    if (wa.hop_barrier) __syncthreads();
    const int64_t rank = rank_at(t);
    v4f cw[U], cg[U], cm[U], v[U], out[U];
    load(rank, cw, cg, cm);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (MODE == MODE_GRAD) {
        const v4f gbar = (cg[u] + carry[u]) * 0.5f;
        out[u] = local_update(cw[u], gbar, cm[u], a.lr, a.mu, v[u]);
        carry[u] = cg[u];
      } else {
        const v4f T = local_update(cw[u], cg[u], cm[u], a.lr, a.mu, v[u]);
        out[u] = (T + carry[u]) * 0.5f;
        carry[u] = (MODE == MODE_SYNC) ? T : cw[u];
      }
    }
    store_one(a.m, rank, v);
    store_one(a.wn, rank, out);
  }
  // close the cycle
  v4f out[U];
  if (MODE == MODE_GRAD) {
    v4f v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const v4f gbar = (first[u] + carry[u]) * 0.5f;
      out[u] = local_update(fw[u], gbar, fm[u], a.lr, a.mu, v[u]);
    }
    store_one(a.m, rank0, v);
  } else {
#pragma unroll
    for (int u = 0; u < U; ++u) out[u] = (first[u] + carry[u]) * 0.5f;
  }
  store_one(a.wn, rank0, out);
}

// ------------------------------------------------------------------- local update
template <typename V, int U, bool NT, bool GUARD>
__device__ __forceinline__ void sgd_tile(const step_args& a, int64_t x0, const V* w, const V* g, V* m, V* n) {
  V Wr[U], Gr[U], Mr[U];
  int64_t idx[U];
  bool on[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int64_t x = x0 + (int64_t)u * blockDim.x;
    on[u] = !GUARD || x < a.rng.count;
    idx[u] = gg_item_index(a.rng, x);
    if (on[u]) {
      Wr[u] = gg_ld<NT>(w + idx[u]);
      Gr[u] = gg_ld<NT>(g + idx[u]);
      Mr[u] = gg_ld<NT>(m + idx[u]);
    }
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    if (!on[u]) continue;
    V v;
    const V T = local_update(Wr[u], Gr[u], Mr[u], a.lr, a.mu, v);
    gg_st<NT>(n + idx[u], T);
    gg_st<NT>(m + idx[u], v);
  }
}

template <typename V, int U, bool NT>
__global__ void __launch_bounds__(256) sgd_kernel(step_args a) {
  const int64_t j = blockIdx.y;
  const V* w = reinterpret_cast<const V*>(a.w + j * a.stride);
  const V* g = reinterpret_cast<const V*>(a.g + j * a.stride);
  V* m = reinterpret_cast<V*>(a.m + j * a.stride);
  V* n = reinterpret_cast<V*>(a.wn + j * a.stride);
  const int64_t per_tile = (int64_t)blockDim.x * U;
  for (int64_t tile = blockIdx.x; tile < a.tiles; tile += gridDim.x) {
    const int64_t x0 = tile * per_tile + threadIdx.x;
    if ((tile + 1) * per_tile <= a.rng.count)
      sgd_tile<V, U, NT, false>(a, x0, w, g, m, n);
    else
      sgd_tile<V, U, NT, true>(a, x0, w, g, m, n);
  }
}

// Lean form for the default launch shape (see gossip_pair_lean_kernel).
template <bool NT>
__global__ void __launch_bounds__(64) sgd_lean_kernel(step_args a) {
  const int64_t j = blockIdx.y;
  // tiles start on 1 KB boundaries of this rank's row even when the row itself does not
  const int64_t sh = (int64_t)(((uint64_t)(uintptr_t)(a.w + j * a.stride) / 16 + (uint64_t)a.rng.lo) % 64);
  const int64_t i = a.rng.lo + (int64_t)blockIdx.x * 64 + threadIdx.x - sh;
  if (i < a.rng.lo || i >= a.rng.lo + a.rng.count) return;
  const v4f* w = reinterpret_cast<const v4f*>(a.w + j * a.stride) + i;
  const v4f* g = reinterpret_cast<const v4f*>(a.g + j * a.stride) + i;
  v4f* m = reinterpret_cast<v4f*>(a.m + j * a.stride) + i;
  v4f* n = reinterpret_cast<v4f*>(a.wn + j * a.stride) + i;
  const v4f Wr = gg_ld<NT>(w), Gr = gg_ld<NT>(g), Mr = gg_ld<NT>(m);
  v4f v;
  const v4f T = local_update(Wr, Gr, Mr, a.lr, a.mu, v);
  if (NT) {
    st_stream(n, T);
    st_stream(m, v);
  } else {
    gg_st<false>(n, T);
    gg_st<false>(m, v);
  }
}

// ------------------------------------------------------------------------ dispatch
enum { KIND_PAIR = 0, KIND_CYCLE = 1, KIND_SGD = 2 };

struct launch_ctx {
  gg_grid gd;
  hipStream_t s;
  const pair_table* pt;
  const rank_table* rt;
  int32_t cycle_len;
};

// The lean kernels serve the default launch shape: 16-byte accesses, one chunk per
// thread, one wavefront per workgroup, one tile per workgroup.
template <typename V, int U>
bool lean_shape(const gg_grid& gd, const step_args& a) {
  return sizeof(V) == sizeof(v4f) && U == 1 && gd.block.x == 64 && (int64_t)gd.grid.x == a.tiles &&
         a.tiles < 0x7fffffffLL;
}

// First 16-byte chunk of the range in rank j's row, counted from address 0: its
// remainder mod 64 is how far the row's tiles sit above a 1 KB boundary.
inline uint64_t first_chunk(const step_args& a, uint64_t j) {
  return (uint64_t)(uintptr_t)(a.w + j * a.stride) / 16 + (uint64_t)a.rng.lo;
}

template <typename V, int MODE, int U, bool NT>
void launch_pair(const launch_ctx& lc, const step_args& a) {
  const gg_grid& gd = lc.gd;
  if (!lean_shape<V, U>(gd, a)) {
    hipLaunchKernelGGL((gossip_pair_kernel<V, MODE, U, NT>), gd.grid, gd.block, gd.lds_bytes, lc.s, a, *lc.pt);
    return;
  }
  // per-pair tile shift; one extra (partial) tile column when any row is off a 1 KB boundary
  pair_table pt = *lc.pt;
  bool shifted = false;
  for (int32_t q = 0; q < a.p / 2; ++q) {
    const uint32_t sh = (uint32_t)(first_chunk(a, pt.jc[q] & 0x3ffu) % 64);
    pt.jc[q] |= sh << 20;
    shifted = shifted || sh != 0;
  }
  dim3 grid = gd.grid;
  if (shifted) grid.x += 1;
  hipLaunchKernelGGL((gossip_pair_lean_kernel<MODE, NT>), grid, gd.block, gd.lds_bytes, lc.s, a, pt);
}

template <typename V, int MODE, int U, bool NT>
void launch_cycle(const launch_ctx& lc, const step_args& a) {
  const gg_grid& gd = lc.gd;
  constexpr int UC = U > 2 ? 2 : U;  // the walk keeps three ranks in registers: two chunks at most
  hipLaunchKernelGGL((gossip_cycle_kernel<V, MODE, UC, NT>), gd.grid, gd.block, gd.lds_bytes, lc.s, a, lc.cycle_len,
                     *lc.rt);
}

template <int MODE>
void launch_walk(int U, dim3 grid, dim3 block, uint32_t lds, hipStream_t s, const step_args& a, const walk_args& wa,
                 const rank_table& rt) {
  switch (U) {
    case 1: hipLaunchKernelGGL((gossip_cycle_walk_kernel<MODE, 1>), grid, block, lds, s, a, wa, rt); break;
    case 2: hipLaunchKernelGGL((gossip_cycle_walk_kernel<MODE, 2>), grid, block, lds, s, a, wa, rt); break;
    case 4: hipLaunchKernelGGL((gossip_cycle_walk_kernel<MODE, 4>), grid, block, lds, s, a, wa, rt); break;
    default: hipLaunchKernelGGL((gossip_cycle_walk_kernel<MODE, 8>), grid, block, lds, s, a, wa, rt); break;
  }
}

template <typename V, int U, bool NT>
void launch_sgd(const launch_ctx& lc, const step_args& a) {
  const gg_grid& gd = lc.gd;
  if (!lean_shape<V, U>(gd, a)) {
    hipLaunchKernelGGL((sgd_kernel<V, U, NT>), gd.grid, gd.block, gd.lds_bytes, lc.s, a);
    return;
  }
  dim3 grid = gd.grid;
  const bool on_boundaries = first_chunk(a, 0) % 64 == 0 && a.stride % 256 == 0;
  if (!on_boundaries) grid.x += 1;  // shifted tile grids need one more (partial) column
  hipLaunchKernelGGL((sgd_lean_kernel<NT>), grid, gd.block, gd.lds_bytes, lc.s, a);
}

template <typename V, int MODE, int U, bool NT>
void launch_one(int kind, const launch_ctx& lc, const step_args& a) {
  if (kind == KIND_PAIR)
    launch_pair<V, MODE, U, NT>(lc, a);
  else if (kind == KIND_CYCLE)
    launch_cycle<V, MODE, U, NT>(lc, a);
  else
    launch_sgd<V, U, NT>(lc, a);
}

template <typename V, int MODE>
void launch_mode(int kind, int U, bool nt, const launch_ctx& lc, const step_args& a) {
#define GG_CASE(UU)                                              \
  case UU:                                                       \
    if (nt)                                                      \
      launch_one<V, MODE, UU, true>(kind, lc, a);                \
    else                                                         \
      launch_one<V, MODE, UU, false>(kind, lc, a);               \
    break;
  switch (U) {
    GG_CASE(1)
    GG_CASE(2)
    GG_CASE(4)
    default:
      GG_CASE(8)
  }
#undef GG_CASE
}

template <typename V>
void launch_any(int kind, int mode, int U, bool nt, const launch_ctx& lc, const step_args& a) {
  if (mode == MODE_SYNC)
    launch_mode<V, MODE_SYNC>(kind, U, nt, lc, a);
  else if (mode == MODE_STALE)
    launch_mode<V, MODE_STALE>(kind, U, nt, lc, a);
  else
    launch_mode<V, MODE_GRAD>(kind, U, nt, lc, a);
}

int32_t gcd32(int32_t x, int32_t y) {
  while (y) {
    const int32_t t = x % y;
    x = y;
    y = t;
  }
  return x;
}

// The lockstep walk of the dissemination cycles over the aligned body.  Returns false
// (nothing enqueued) when the walking form does not apply.
bool enqueue_walk(const gg_ctx* ctx, int mode, step_args& a, int32_t cycle_len, int64_t cycles,
                  const rank_table& rt, hipStream_t s) {
  // measured best at 25.6 M parameters per rank for p = 16 ... 128 and every cycle length: 4 wavefronts x 1
  // chunk, tiles 32 KB apart, 3 workgroups per CU
  const gg_walk_shape own{1, 4, 32, 3, 1, 0};
  const gg_walk_launch wl = gg_walk_geometry(ctx, own, 8, (a.rng.count + 63) / 64);
  if (wl.grid_x == 0) return false;
  walk_args wa;
  wa.cycle_len = cycle_len;
  wa.hop_barrier = wl.shape.barrier;
  wa.step = wl.shape.step;
  const dim3 grid((unsigned)wl.grid_x, (unsigned)cycles, 1), block(64u * (unsigned)wl.shape.waves);
  if (mode == MODE_SYNC)
    launch_walk<MODE_SYNC>(wl.shape.chunks, grid, block, wl.lds_bytes, s, a, wa, rt);
  else if (mode == MODE_STALE)
    launch_walk<MODE_STALE>(wl.shape.chunks, grid, block, wl.lds_bytes, s, a, wa, rt);
  else
    launch_walk<MODE_GRAD>(wl.shape.chunks, grid, block, wl.lds_bytes, s, a, wa, rt);
  return true;
}

// Enqueue one kind of step over the element range [e_lo, e_hi) of every rank: a
// 16-byte vector launch for the aligned body and, when the range is ragged or the
// buffers are not 16-byte aligned, one scalar launch for what is left.
int enqueue_step(gg_ctx* ctx, int kind, int mode, step_args a, const uint16_t* sigma_host, int64_t e_lo,
                 int64_t e_hi, hipStream_t s) {
  if (e_hi <= e_lo) return GG_OK;
  const int32_t p = ctx->cfg.p;
  int64_t rows = p;
  int32_t cycle_len = 1;
  pair_table pt;
  if (kind == KIND_PAIR) {
    rows = p / 2;
    // virtual pairs (v, v | shift) with bit k of v clear, mapped through the communicator
    const int32_t low = a.shift - 1;
    for (int32_t q = 0; q < p / 2; ++q) {
      const int32_t v0 = ((q & ~low) << 1) | (q & low);
      pt.jc[q] = (uint32_t)sigma_host[v0] | ((uint32_t)sigma_host[v0 | a.shift] << 10);
    }
    for (int32_t q = p / 2; q < GG_MAX_RANKS / 2; ++q) pt.jc[q] = 0;
  }
  rank_table rt;
  if (kind == KIND_CYCLE) {
    rows = gcd32(p, a.shift);
    cycle_len = p / (int32_t)rows;
    for (int32_t v = 0; v < GG_MAX_RANKS; v += 2) {
      const uint32_t r0 = v < p ? sigma_host[v] : 0u, r1 = v + 1 < p ? sigma_host[v + 1] : 0u;
      rt.r2[v >> 1] = r0 | (r1 << 16);
    }
  }
  const bool vec_ok = gg_aligned(a.w, 16) && gg_aligned(a.g, 16) && gg_aligned(a.m, 16) &&
                      gg_aligned(a.wn, 16) && (a.stride % 4 == 0);
  int64_t body_lo = e_lo, body_hi = e_lo;  // empty body unless the vector path applies
  if (vec_ok) {
    body_lo = (e_lo + 3) / 4 * 4;
    body_hi = e_hi / 4 * 4;
    if (body_hi < body_lo) body_hi = body_lo = e_lo;
  }
  const bool nt = ctx->tune.nontemporal != 0;
  const int64_t edge = (body_lo - e_lo) + (e_hi - body_hi);
  const int loads = kind == KIND_SGD ? 3 : (kind == KIND_CYCLE ? 5 : 6);

  if (body_hi > body_lo) {
    a.rng = gg_range{body_lo / 4, (body_hi - body_lo) / 4, INT64_MAX, 0};
    bool done = false;
    if (kind == KIND_CYCLE) done = enqueue_walk(ctx, mode, a, cycle_len, rows, rt, s);
    if (!done) {
      int U = ctx->tune.chunks;
      if (kind == KIND_CYCLE && U > 2) U = 2;
      launch_ctx lc{gg_make_grid(ctx, a.rng.count, U, rows, loads), s, &pt, &rt, cycle_len};
      a.tiles = lc.gd.tiles;
      launch_any<v4f>(kind, mode, U, nt, lc, a);
    }
    GG_HIP_TRY(hipGetLastError());
  }
  if (edge > 0) {
    a.rng = gg_range{e_lo, edge, body_lo, body_hi - body_lo};
    launch_ctx lc{gg_make_grid(ctx, a.rng.count, 1, rows, loads), s, &pt, &rt, cycle_len};
    a.tiles = lc.gd.tiles;
    launch_any<float>(kind, mode, 1, nt, lc, a);
    GG_HIP_TRY(hipGetLastError());
  }
  return GG_OK;
}

int check_buffers(const gg_ctx* ctx, const float* w, const float* g, const float* m, const float* wn) {
  if (!ctx || !w || !g || !m) return GG_ERR_ARG;
  if (!gg_aligned(w, 4) || !gg_aligned(g, 4) || !gg_aligned(m, 4) || (wn && !gg_aligned(wn, 4)))
    return GG_ERR_ALIGN;
  if (w == g || w == m || g == m || (wn && (wn == w || wn == g || wn == m))) return GG_ERR_ARG;
  return GG_OK;
}

}  // namespace

extern "C" int gg_gossip_step(gg_ctx* ctx, int64_t step, float* w, const float* g, float* m, float* w_next,
                              const int64_t* seg_offsets, int32_t nseg, void* stream) {
  int rc = check_buffers(ctx, w, g, m, w_next);
  if (rc != GG_OK) return rc;
  if (step < 0 || nseg < 0) return GG_ERR_ARG;
  if ((nseg > 0) != (seg_offsets != nullptr)) return GG_ERR_ARG;
  const gg_config& cfg = ctx->cfg;
  int64_t e_lo = 0, e_hi = cfg.n;
  if (nseg > 0) {
    if (seg_offsets[0] < 0 || seg_offsets[nseg] > cfg.n) return GG_ERR_ARG;
    for (int32_t s = 0; s < nseg; ++s)
      if (seg_offsets[s] > seg_offsets[s + 1]) return GG_ERR_ARG;
    e_lo = seg_offsets[0];
    e_hi = seg_offsets[nseg];
  }
  rc = gg_check_ctx_device(ctx);
  if (rc != GG_OK) return rc;

  const int32_t k = (int32_t)(step % ctx->L);
  const int32_t r = (int32_t)((step / ctx->L) % ctx->R);
  step_args a;
  a.w = w;
  a.g = g;
  a.m = m;
  a.wn = w_next ? w_next : w;
  a.stride = cfg.rank_stride;
  a.shift = int32_t(1) << k;
  a.p = cfg.p;
  a.lr = cfg.lr;
  a.mu = cfg.momentum;
  a.tiles = 0;
  a.rng = gg_range{0, 0, INT64_MAX, 0};

  int kind, mode;
  if (cfg.avg_mode == GG_AVG_NONE) {
    kind = KIND_SGD;
    mode = MODE_SYNC;
  } else {
    kind = cfg.topology == GG_TOPO_HYPERCUBE ? KIND_PAIR : KIND_CYCLE;
    // Dissemination with shift p/2: receiving from v - p/2 is receiving from v + p/2, the
    // map is an involution and its 2-cycles are exactly the pairs (v, v | p/2) -- same
    // arithmetic (the sum of the two contributions commutes), faster kernel.
    if (kind == KIND_CYCLE && 2 * a.shift == cfg.p) kind = KIND_PAIR;
    mode = cfg.avg_mode == GG_AVG_GRAD ? MODE_GRAD : (cfg.staleness ? MODE_STALE : MODE_SYNC);
  }
  return enqueue_step(ctx, kind, mode, a, &ctx->sigma[(size_t)r * cfg.p], e_lo, e_hi, (hipStream_t)stream);
}

extern "C" int gg_sgd_step(gg_ctx* ctx, float* w, const float* g, float* m, void* stream) {
  int rc = check_buffers(ctx, w, g, m, nullptr);
  if (rc != GG_OK) return rc;
  rc = gg_check_ctx_device(ctx);
  if (rc != GG_OK) return rc;
  step_args a;
  a.w = w;
  a.g = g;
  a.m = m;
  a.wn = w;
  a.stride = ctx->cfg.rank_stride;
  a.shift = 1;
  a.p = ctx->cfg.p;
  a.lr = ctx->cfg.lr;
  a.mu = ctx->cfg.momentum;
  a.tiles = 0;
  a.rng = gg_range{0, 0, INT64_MAX, 0};
  return enqueue_step(ctx, KIND_SGD, MODE_SYNC, a, ctx->sigma.data(), 0, ctx->cfg.n, (hipStream_t)stream);
}
