// Recursive-doubling all-reduce over the virtual ranks (Sec. 3.1, Sec. 4.1): the
// Theta(log p) method GossipGraD is compared with, plus its one-pass form.
#pragma clang fp contract(off)

#include "gg_internal.h"

namespace {

struct ar_args {
  float* g;
  int64_t stride;
  gg_range rng;
  int64_t tiles;
  int32_t shift;  // 2^k of this round
  int32_t p;
  float scale;    // applied after the add when `scaled`
  int32_t scaled;
};


// One round: ranks j and j ^ shift both end with g[j] + g[j ^ shift].  A thread
// owns the same chunk of both, so the round is in place: 8 B / rank / element.
template <typename V, int U, bool NT>
__global__ void __launch_bounds__(256) allreduce_round_kernel(ar_args a) {
  const int32_t q = blockIdx.y;
  const int32_t low = a.shift - 1;
  const int64_t j = ((q & ~low) << 1) | (q & low);
  const int64_t c = j | a.shift;
  V* gj = reinterpret_cast<V*>(a.g + j * a.stride);
  V* gc = reinterpret_cast<V*>(a.g + c * a.stride);
  const int64_t per_tile = (int64_t)blockDim.x * U;
  for (int64_t tile = blockIdx.x; tile < a.tiles; tile += gridDim.x) {
    const int64_t x0 = tile * per_tile + threadIdx.x;
    V A[U], B[U];
    int64_t idx[U];
    bool on[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t x = x0 + (int64_t)u * blockDim.x;
      on[u] = x < a.rng.count;
      idx[u] = gg_item_index(a.rng, x);
      if (on[u]) {
        A[u] = gg_ld<NT>(gj + idx[u]);
        B[u] = gg_ld<NT>(gc + idx[u]);
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (!on[u]) continue;
      V s = A[u] + B[u];
      if (a.scaled) s = s * a.scale;
      gg_st<NT>(gj + idx[u], s);
      gg_st<NT>(gc + idx[u], s);
    }
  }
}

// Balanced pairwise tree over ranks [r, r + 2^K): the value every rank holds after
// K recursive-doubling rounds (addition commutes, so the bits agree).
template <int K, typename V, bool NT>
struct tree_sum {
  static __device__ __forceinline__ V run(const float* g, int64_t stride, int64_t i, int64_t r) {
    const V lo = tree_sum<K - 1, V, NT>::run(g, stride, i, r);
    const V hi = tree_sum<K - 1, V, NT>::run(g, stride, i, r + (int64_t(1) << (K - 1)));
    return lo + hi;
  }
};
template <typename V, bool NT>
struct tree_sum<0, V, NT> {
  static __device__ __forceinline__ V run(const float* g, int64_t stride, int64_t i, int64_t r) {
    return gg_ld<NT>(reinterpret_cast<const V*>(g + r * stride) + i);
  }
};

// One pass: read the p values of a chunk once, add them in tree order, write the
// result to every rank: 8 B / rank / element in total instead of 8 B per round.
// General form (scalar instantiation for ragged or unaligned buffers).
template <int K, typename V, bool NT>
__global__ void __launch_bounds__(256) allreduce_onepass_kernel(ar_args a) {
  for (int64_t tile = blockIdx.x; tile < a.tiles; tile += gridDim.x) {
    const int64_t x = tile * blockDim.x + threadIdx.x;
    if (x >= a.rng.count) continue;
    const int64_t i = gg_item_index(a.rng, x);
    V s = tree_sum<K, V, NT>::run(a.g, a.stride, i, 0);
    if (a.scaled) s = s * a.scale;
    for (int64_t r = 0; r < (int64_t(1) << K); ++r) gg_st<NT>(reinterpret_cast<V*>(a.g + r * a.stride) + i, s);
  }
}

// Default form for 16-byte aligned buffers: the same tree, walked so that the chip
// streams a few ranks at a time instead of all p.  A workgroup of W wavefronts owns
// W*U tiles `step` tiles apart (32 KB: same DRAM channel, eight of them one DRAM row),
// visits the ranks in order 2^B at a time and passes a barrier after each such group,
// first reading (partial sums wait on a register stack of depth K), then writing.
struct walk_shape {
  int32_t step;
  int32_t barrier;
};

template <int K, int B, int U>
struct tree_walk {
  static __device__ __forceinline__ void run(const ar_args& a, const walk_shape& ws, const int64_t* idx,
                                             const bool* on, int64_t r, v4f* out) {
    v4f lo[U], hi[U];
    tree_walk<K - 1, B, U>::run(a, ws, idx, on, r, lo);
    tree_walk<K - 1, B, U>::run(a, ws, idx, on, r + (int64_t(1) << (K - 1)), hi);
#pragma unroll
    for (int u = 0; u < U; ++u) out[u] = lo[u] + hi[u];
    if (K >= B) {
      // Every sum from a group of 2^B ranks upwards is formed here and now: left alone, the
      // compiler keeps the values in registers and adds at the very end, which no register
      // file holds at p = 128.  This way at most one partial sum per tree level is alive.
#pragma unroll
      for (int u = 0; u < U; ++u) asm volatile("" : "+v"(out[u]));
      // every wavefront of the workgroup passes here once per group of 2^B ranks
      if (K == B && ws.barrier) __syncthreads();
    }
  }
};
template <int B, int U>
struct tree_walk<0, B, U> {
  static __device__ __forceinline__ void run(const ar_args& a, const walk_shape& ws, const int64_t* idx,
                                             const bool* on, int64_t r, v4f* out) {
    const v4f* row = reinterpret_cast<const v4f*>(a.g + r * a.stride);
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (on[u]) out[u] = gg_ld<true>(row + idx[u]);
    if (B == 0) {
#pragma unroll
      for (int u = 0; u < U; ++u) asm volatile("" : "+v"(out[u]));
      if (ws.barrier) __syncthreads();
    }
  }
};

template <int K, int B, int U>
__global__ void __launch_bounds__(512 / U) allreduce_walk_kernel(ar_args a, walk_shape ws) {
  int64_t idx[U];
  bool on[U];
  {
    const int64_t bx = blockIdx.x, step = ws.step;
    const int64_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63, W = blockDim.x >> 6;
    const int64_t tile0 = (bx / step) * (step * W * U) + bx % step + wave * U * step;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t x = (tile0 + u * step) * 64 + lane;
      on[u] = x < a.rng.count;
      idx[u] = a.rng.lo + x;
    }
  }
  v4f s[U];
  tree_walk<K, (B < K ? B : K), U>::run(a, ws, idx, on, 0, s);
  if (a.scaled) {
#pragma unroll
    for (int u = 0; u < U; ++u) s[u] = s[u] * a.scale;
  }
  for (int64_t r = 0; r < (int64_t(1) << K); ++r) {
    v4f* row = reinterpret_cast<v4f*>(a.g + r * a.stride);
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (on[u]) __builtin_nontemporal_store(s[u], row + idx[u]);
    if (ws.barrier && ((r + 1) & ((int64_t(1) << B) - 1)) == 0) __syncthreads();
  }
}

template <typename V>
void launch_round(int U, bool nt, const gg_grid& gd, hipStream_t s, const ar_args& a) {
#define GG_CASE(UU)                                                                            \
  case UU:                                                                                     \
    if (nt)                                                                                    \
      hipLaunchKernelGGL((allreduce_round_kernel<V, UU, true>), gd.grid, gd.block, gd.lds_bytes, s, a);   \
    else                                                                                       \
      hipLaunchKernelGGL((allreduce_round_kernel<V, UU, false>), gd.grid, gd.block, gd.lds_bytes, s, a);  \
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
void launch_onepass(int K, const gg_grid& gd, hipStream_t s, const ar_args& a) {
#define GG_CASE(KK)                                                                            \
  case KK:                                                                                     \
    hipLaunchKernelGGL((allreduce_onepass_kernel<KK, V, true>), gd.grid, gd.block, gd.lds_bytes, s, a);   \
    break;
  switch (K) {
    GG_CASE(1)
    GG_CASE(2)
    GG_CASE(3)
    GG_CASE(4)
    GG_CASE(5)
    GG_CASE(6)
    default:
      GG_CASE(7)
  }
#undef GG_CASE
}

template <int B, int U>
void launch_walk_k(int K, dim3 grid, dim3 block, uint32_t lds, hipStream_t s, const ar_args& a, const walk_shape& ws) {
#define GG_CASE(KK)                                                                              \
  case KK:                                                                                       \
    hipLaunchKernelGGL((allreduce_walk_kernel<KK, B, U>), grid, block, lds, s, a, ws);           \
    break;
  switch (K) {
    GG_CASE(1)
    GG_CASE(2)
    GG_CASE(3)
    GG_CASE(4)
    GG_CASE(5)
    GG_CASE(6)
    default:
      GG_CASE(7)
  }
#undef GG_CASE
}

template <int B>
void launch_walk_u(int U, int K, dim3 grid, dim3 block, uint32_t lds, hipStream_t s, const ar_args& a,
                   const walk_shape& ws) {
  if (U == 1)
    launch_walk_k<B, 1>(K, grid, block, lds, s, a, ws);
  else
    launch_walk_k<B, 2>(K, grid, block, lds, s, a, ws);  // four chunks per thread measured far slower
}

enum { MAX_ONEPASS_LOG2 = 7 };

// body (16-byte) + edge (scalar) split shared by both forms
struct split {
  gg_range body, edge;
};
split make_split(const float* g, int64_t stride, int64_t n) {
  split s;
  const bool vec_ok = gg_aligned(g, 16) && stride % 4 == 0;
  const int64_t body_hi = vec_ok ? n / 4 * 4 : 0;
  s.body = gg_range{0, body_hi / 4, INT64_MAX, 0};
  s.edge = gg_range{body_hi, n - body_hi, INT64_MAX, 0};
  return s;
}

int check(const gg_ctx* ctx, const float* g) {
  if (!ctx || !g) return GG_ERR_ARG;
  if (!gg_aligned(g, 4)) return GG_ERR_ALIGN;
  if (!gg_is_pow2(ctx->cfg.p)) return GG_ERR_NOT_POW2;
  return gg_check_ctx_device(ctx);
}

}  // namespace

extern "C" int gg_allreduce_baseline(gg_ctx* ctx, float* g, int32_t average, void* stream) {
  int rc = check(ctx, g);
  if (rc != GG_OK) return rc;
  const int32_t p = ctx->cfg.p;
  const split sp = make_split(g, ctx->cfg.rank_stride, ctx->cfg.n);
  const bool nt = ctx->tune.nontemporal != 0;
  for (int32_t k = 0; k < ctx->L; ++k) {
    ar_args a;
    a.g = g;
    a.stride = ctx->cfg.rank_stride;
    a.shift = int32_t(1) << k;
    a.p = p;
    a.scaled = (average && k == ctx->L - 1) ? 1 : 0;  // scaling the last round's sum is the same
    a.scale = 1.0f / (float)p;                        // rounding as scaling afterwards
    if (sp.body.count > 0) {
      a.rng = sp.body;
      gg_grid gd = gg_make_grid(ctx, a.rng.count, ctx->tune.chunks, p / 2, 2);
      a.tiles = gd.tiles;
      launch_round<v4f>(ctx->tune.chunks, nt, gd, (hipStream_t)stream, a);
      GG_HIP_TRY(hipGetLastError());
    }
    if (sp.edge.count > 0) {
      a.rng = sp.edge;
      gg_grid gd = gg_make_grid(ctx, a.rng.count, 1, p / 2, 2);
      a.tiles = gd.tiles;
      launch_round<float>(1, nt, gd, (hipStream_t)stream, a);
      GG_HIP_TRY(hipGetLastError());
    }
  }
  return GG_OK;
}

extern "C" int gg_allreduce_onepass(gg_ctx* ctx, float* g, int32_t average, void* stream) {
  int rc = check(ctx, g);
  if (rc != GG_OK) return rc;
  if (ctx->L > MAX_ONEPASS_LOG2) return gg_allreduce_baseline(ctx, g, average, stream);
  const split sp = make_split(g, ctx->cfg.rank_stride, ctx->cfg.n);
  ar_args a;
  a.g = g;
  a.stride = ctx->cfg.rank_stride;
  a.shift = 1;
  a.p = ctx->cfg.p;
  a.scaled = average ? 1 : 0;
  a.scale = 1.0f / (float)ctx->cfg.p;
  if (sp.body.count > 0) {
    a.rng = sp.body;
    // measured best at 25.6 M parameters per rank for p = 16, 64 and 128: 4 wavefronts x 1 chunk, 3 workgroups
    // per CU, a barrier every 4 ranks
    const gg_walk_shape own{1, 4, 32, 3, 1, 2};
    const gg_walk_launch wl = gg_walk_geometry(ctx, own, 2, (a.rng.count + 63) / 64);
    if (wl.grid_x > 0) {
      walk_shape ws{wl.shape.step, wl.shape.barrier};
      const dim3 grid((unsigned)wl.grid_x), block(64u * (unsigned)wl.shape.waves);
      const int U = wl.shape.chunks;
      switch (wl.shape.group_log2) {
        case 0: launch_walk_u<0>(U, ctx->L, grid, block, wl.lds_bytes, (hipStream_t)stream, a, ws); break;
        case 1: launch_walk_u<1>(U, ctx->L, grid, block, wl.lds_bytes, (hipStream_t)stream, a, ws); break;
        case 2: launch_walk_u<2>(U, ctx->L, grid, block, wl.lds_bytes, (hipStream_t)stream, a, ws); break;
        default: launch_walk_u<3>(U, ctx->L, grid, block, wl.lds_bytes, (hipStream_t)stream, a, ws); break;
      }
    } else {
      gg_grid gd = gg_make_grid(ctx, a.rng.count, 1, 1, 12);
      a.tiles = gd.tiles;
      launch_onepass<v4f>(ctx->L, gd, (hipStream_t)stream, a);
    }
    GG_HIP_TRY(hipGetLastError());
  }
  if (sp.edge.count > 0) {
    a.rng = sp.edge;
    gg_grid gd = gg_make_grid(ctx, a.rng.count, 1, 1, 12);
    a.tiles = gd.tiles;
    launch_onepass<float>(ctx->L, gd, (hipStream_t)stream, a);
    GG_HIP_TRY(hipGetLastError());
  }
  return GG_OK;
}
