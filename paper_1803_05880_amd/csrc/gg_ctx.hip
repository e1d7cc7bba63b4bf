// Context, partner schedule and partner rotation (Sec. 4.3, 4.4, 4.5.1): host side.
#include <string.h>

#include <new>

#include "gg_internal.h"

namespace {

int ceil_log2(int32_t p) {
  int L = 0;
  while ((int64_t(1) << L) < p) ++L;
  return L;
}

// Communicator r >= 1: Fisher-Yates shuffle of the identity, one 32-bit word per
// swap, words taken in order from blocks (n, r, 0, GG_TAG_COMM), n = 0, 1, ...
// The swap partner of position i is floor(u * (i+1) / 2^32).
void draw_communicator(int32_t p, uint64_t seed, uint32_t r, uint16_t* a) {
  for (int32_t v = 0; v < p; ++v) a[v] = (uint16_t)v;
  if (r == 0) return;  // the original communicator
  const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
  uint32_t words[4];
  uint32_t block = 0;
  int have = 0;
  for (int32_t i = p - 1; i >= 1; --i) {
    if (have == 0) {
      gg_u32x4 o = gg_philox4x32_10(block++, r, 0u, (uint32_t)GG_TAG_COMM, k0, k1);
      words[0] = o.x; words[1] = o.y; words[2] = o.z; words[3] = o.w;
      have = 4;
    }
    const uint32_t u = words[4 - have];
    --have;
    const uint32_t q = (uint32_t)(((uint64_t)u * (uint64_t)(i + 1)) >> 32);
    const uint16_t tmp = a[i];
    a[i] = a[q];
    a[q] = tmp;
  }
}

}  // namespace

int gg_check_ctx_device(const gg_ctx* ctx) {
  if (ctx->device < 0) return GG_ERR_HIP;  // host-only context: no GPU was present at gg_init
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) {
    (void)hipGetLastError();
    return GG_ERR_HIP;
  }
  return dev == ctx->device ? GG_OK : GG_ERR_ARG;
}

gg_grid gg_make_grid(const gg_ctx* ctx, int64_t items, int32_t chunks, int64_t rows, int32_t loads) {
  gg_grid out;
  const int64_t per_tile = (int64_t)ctx->tune.threads * chunks;
  out.tiles = (items + per_tile - 1) / per_tile;
  int64_t gx = out.tiles;
  if (gx > 0x7fffffffLL) gx = 0x7fffffffLL;  // the kernels loop over tiles, any gx works
  if (gx < 1) gx = 1;
  out.grid = dim3((unsigned)gx, (unsigned)rows, 1);
  out.block = dim3((unsigned)ctx->tune.threads, 1, 1);
  // Occupancy cap: a CU has 160 KB of LDS, so a workgroup that reserves 160 KB / k of
  // it leaves room for k workgroups.  The streaming kernels run fastest with about
  // one wavefront per SIMD: more waves in flight widen the window of DRAM rows
  // touched at once and cost row-buffer hits.
  out.lds_bytes = 0;
  if (ctx->tune.blocks_per_cu > 0) {
    // the cap is stated for 6 loads per thread and 64 threads; scale to this launch
    int64_t cap = ((int64_t)ctx->tune.blocks_per_cu * 6 * 64 + (int64_t)loads * chunks * ctx->tune.threads / 2) /
                  ((int64_t)loads * chunks * ctx->tune.threads);
    if (cap < 2) cap = 2;
    if (cap > 64) cap = 64;
    uint32_t b = (uint32_t)(160u * 1024u / (uint32_t)cap) & ~255u;
    if (b > 64u * 1024u - 4096u) b = 64u * 1024u - 4096u;  // stay below the default dynamic-LDS limit
    out.lds_bytes = b;
  }
  return out;
}

gg_walk_launch gg_walk_geometry(const gg_ctx* ctx, const gg_walk_shape& d, int32_t max_chunks, int64_t tiles) {
  const gg_walk_shape& t = ctx->tune.walk;
  gg_walk_launch out;
  gg_walk_shape& sh = out.shape;
  sh.chunks = t.chunks == GG_WALK_UNSET ? d.chunks : t.chunks;
  sh.waves = t.waves == GG_WALK_UNSET ? d.waves : t.waves;
  sh.step = t.step == GG_WALK_UNSET ? d.step : t.step;
  sh.wg_per_cu = t.wg_per_cu == GG_WALK_UNSET ? d.wg_per_cu : t.wg_per_cu;
  sh.barrier = t.barrier == GG_WALK_UNSET ? d.barrier : t.barrier;
  sh.group_log2 = t.group_log2 == GG_WALK_UNSET ? d.group_log2 : t.group_log2;
  if (sh.chunks > max_chunks) sh.chunks = max_chunks;
  while (sh.chunks * sh.waves > 8) sh.waves /= 2;  // an override of one may meet the default of the other
  if (sh.waves == 1) sh.barrier = 0;
  out.grid_x = 0;
  out.lds_bytes = 0;
  if (sh.chunks <= 0 || !ctx->tune.nontemporal) return out;
  const int64_t span = (int64_t)sh.step * sh.waves * sh.chunks;
  const int64_t gx = (tiles + span - 1) / span * sh.step;
  if (gx < 1 || gx > 0x7fffffffLL) return out;
  out.grid_x = gx;
  if (sh.wg_per_cu > 0) {
    uint32_t b = (160u * 1024u / (uint32_t)sh.wg_per_cu) & ~255u;
    if (b > 64u * 1024u - 4096u) b = 64u * 1024u - 4096u;  // stay below the default dynamic-LDS limit
    out.lds_bytes = b;
  }
  return out;
}

extern "C" int gg_init(const gg_config* cfg, gg_ctx** out) {
  if (!cfg || !out) return GG_ERR_ARG;
  if (cfg->p < 2 || cfg->p > GG_MAX_RANKS) return GG_ERR_ARG;
  if (cfg->n < 0 || cfg->rank_stride < cfg->n) return GG_ERR_ARG;
  if (cfg->rank_stride > (int64_t(1) << 40)) return GG_ERR_ARG;
  if (cfg->topology != GG_TOPO_HYPERCUBE && cfg->topology != GG_TOPO_DISSEMINATION) return GG_ERR_ARG;
  if (cfg->avg_mode != GG_AVG_MODEL && cfg->avg_mode != GG_AVG_GRAD && cfg->avg_mode != GG_AVG_NONE)
    return GG_ERR_ARG;
  if (cfg->staleness != 0 && cfg->staleness != 1) return GG_ERR_ARG;
  if (cfg->staleness == 1 && cfg->avg_mode != GG_AVG_MODEL) return GG_ERR_ARG;
  if (cfg->num_comms < 0 || cfg->num_comms > 4096 || cfg->reserved != 0) return GG_ERR_ARG;
  if (!(cfg->lr == cfg->lr) || !(cfg->momentum == cfg->momentum)) return GG_ERR_ARG;  // NaN
  if (cfg->topology == GG_TOPO_HYPERCUBE && !gg_is_pow2(cfg->p)) return GG_ERR_NOT_POW2;

  gg_ctx* ctx = new (std::nothrow) gg_ctx();
  if (!ctx) return GG_ERR_NOMEM;
  ctx->cfg = *cfg;
  ctx->L = ceil_log2(cfg->p);
  ctx->R = cfg->num_comms == 0 ? cfg->p : cfg->num_comms;
  ctx->d_sigma = nullptr;
  ctx->d_scratch = nullptr;
  ctx->scratch_cap = 0;
  ctx->d_offsets = nullptr;
  ctx->h_offsets_pinned = nullptr;
  ctx->tune = gg_tuning{64, 1, 7, 1, gg_walk_shape{GG_WALK_UNSET, GG_WALK_UNSET, GG_WALK_UNSET, GG_WALK_UNSET, GG_WALK_UNSET, GG_WALK_UNSET}};

  const size_t entries = (size_t)ctx->R * (size_t)cfg->p;
  try {
    ctx->sigma.resize(entries);
    ctx->inv.resize(entries);
  } catch (...) {
    delete ctx;
    return GG_ERR_NOMEM;
  }
  for (int32_t r = 0; r < ctx->R; ++r) {
    uint16_t* s = &ctx->sigma[(size_t)r * cfg->p];
    uint16_t* iv = &ctx->inv[(size_t)r * cfg->p];
    draw_communicator(cfg->p, cfg->seed, (uint32_t)r, s);
    for (int32_t v = 0; v < cfg->p; ++v) iv[s[v]] = (uint16_t)v;
  }

  // Without a GPU the context is host-only: gg_partner works (it is a pure host
  // function), every entry point that would enqueue device work returns GG_ERR_HIP.
  int rc = GG_OK;
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || ndev <= 0) {
    (void)hipGetLastError();
    ctx->device = -1;
    ctx->num_cus = 0;
    *out = ctx;
    return GG_OK;
  }
  hipDeviceProp_t prop;
  if (hipGetDevice(&ctx->device) != hipSuccess || hipGetDeviceProperties(&prop, ctx->device) != hipSuccess) {
    rc = GG_ERR_HIP;
  } else {
    ctx->num_cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    // failure here only disables gg_shuffle_noalloc on this device (it then returns GG_ERR_HIP)
    (void)gg_static_scratch_setup(ctx->device);
    if (hipMalloc((void**)&ctx->d_sigma, entries * sizeof(uint16_t)) != hipSuccess) {
      rc = GG_ERR_NOMEM;
    } else if (hipMemcpy(ctx->d_sigma, ctx->sigma.data(), entries * sizeof(uint16_t), hipMemcpyHostToDevice) !=
               hipSuccess) {
      rc = GG_ERR_HIP;
    }
  }
  if (rc != GG_OK) {
    (void)hipGetLastError();
    if (ctx->d_sigma) (void)hipFree(ctx->d_sigma);
    delete ctx;
    return rc;
  }
  *out = ctx;
  return GG_OK;
}

extern "C" int gg_set_hyper(gg_ctx* ctx, float lr, float momentum) {
  if (!ctx || !(lr == lr) || !(momentum == momentum)) return GG_ERR_ARG;
  ctx->cfg.lr = lr;
  ctx->cfg.momentum = momentum;
  return GG_OK;
}

extern "C" int gg_destroy(gg_ctx* ctx) {
  if (!ctx) return GG_ERR_ARG;
  int rc = GG_OK;
  if (ctx->device < 0) {
    delete ctx;
    return GG_OK;
  }
  if (hipDeviceSynchronize() != hipSuccess) rc = GG_ERR_HIP;
  if (ctx->d_sigma && hipFree(ctx->d_sigma) != hipSuccess) rc = GG_ERR_HIP;
  if (ctx->d_scratch && hipFree(ctx->d_scratch) != hipSuccess) rc = GG_ERR_HIP;
  if (ctx->d_offsets && hipFree(ctx->d_offsets) != hipSuccess) rc = GG_ERR_HIP;
  if (ctx->h_offsets_pinned && hipHostFree(ctx->h_offsets_pinned) != hipSuccess) rc = GG_ERR_HIP;
  if (rc != GG_OK) (void)hipGetLastError();
  delete ctx;
  return rc;
}

extern "C" int gg_partner(const gg_ctx* ctx, int64_t step, int32_t* send_to, int32_t* recv_from) {
  if (!ctx || !send_to || step < 0) return GG_ERR_ARG;
  const int32_t p = ctx->cfg.p;
  const int32_t k = (int32_t)(step % ctx->L);
  const int32_t r = (int32_t)((step / ctx->L) % ctx->R);
  const uint16_t* s = &ctx->sigma[(size_t)r * p];
  const uint16_t* iv = &ctx->inv[(size_t)r * p];
  const int32_t shift = int32_t(1) << k;
  for (int32_t j = 0; j < p; ++j) {
    const int32_t v = iv[j];
    if (ctx->cfg.topology == GG_TOPO_HYPERCUBE) {
      const int32_t partner = s[v ^ shift];
      send_to[j] = partner;
      if (recv_from) recv_from[j] = partner;
    } else {
      send_to[j] = s[(v + shift) % p];
      if (recv_from) recv_from[j] = s[(v + p - shift) % p];
    }
  }
  return GG_OK;
}

extern "C" const char* gg_strerror(int code) {
  switch (code) {
    case GG_OK: return "ok";
    case GG_ERR_ARG: return "invalid argument";
    case GG_ERR_NOT_POW2: return "number of ranks must be a power of two";
    case GG_ERR_ALIGN: return "device pointer is not 4-byte aligned";
    case GG_ERR_HIP: return "HIP runtime error";
    case GG_ERR_NOMEM: return "out of memory";
    case GG_ERR_UNSUPPORTED: return "not supported";
    case GG_ERR_LIMIT: return "size exceeds the fixed scratch of the non-allocating entry point";
    default: return "unknown error";
  }
}
