// Internal declarations shared by the library's translation units (not part of
// the C ABI).  gfx950 only.
#ifndef GG_INTERNAL_H_
#define GG_INTERNAL_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "gg.h"
#include "gg_probe.h"

#define GG_HIP_TRY(expr)                      \
  do {                                        \
    hipError_t gg_e_ = (expr);                \
    if (gg_e_ != hipSuccess) {                \
      (void)hipGetLastError();                \
      return GG_ERR_HIP;                      \
    }                                         \
  } while (0)

// 16-byte vector of four floats: one global_load_dwordx4 / global_store_dwordx4.
typedef float v4f __attribute__((ext_vector_type(4)));

// A run of `count` consecutive work items starting at index `lo` (in units of the
// kernel's access type), with an optional hole: items at or beyond `gap_at` are
// shifted up by `gap_len`.  The hole lets one scalar launch cover the ragged
// head and tail that surround the 16-byte aligned body.
struct gg_range {
  int64_t lo;
  int64_t count;
  int64_t gap_at;
  int64_t gap_len;
};

// ---- device helpers shared by the streaming kernels
// Nothing these kernels touch is read twice, so loads and stores carry the
// non-temporal hint (NT) unless it is switched off for comparison.
template <bool NT, typename V>
__device__ __forceinline__ V gg_ld(const V* ptr) {
  if (NT) return __builtin_nontemporal_load(ptr);
  return *ptr;
}
template <bool NT, typename V>
__device__ __forceinline__ void gg_st(V* ptr, V val) {
  if (NT)
    __builtin_nontemporal_store(val, ptr);
  else
    *ptr = val;
}
// Work item x of a range -> index in units of the access type (skips the hole).
__device__ __forceinline__ int64_t gg_item_index(const gg_range& r, int64_t x) {
  int64_t i = r.lo + x;
  if (i >= r.gap_at) i += r.gap_len;
  return i;
}

// Workgroup shape of a kernel that walks over many ranks (dissemination cycles, one-pass
// all-reduce, payload ring).  In gg_tuning a field of GG_WALK_UNSET means "the kernel's own
// default"; gg_walk_geometry fills those in.
enum { GG_WALK_UNSET = -1 };
struct gg_walk_shape {
  int32_t chunks;      // 16-byte chunks per thread (1, 2, 4, 8); 0: the kernel's general form instead
  int32_t waves;       // wavefronts per workgroup (1, 2, 4, 8); chunks * waves <= 8
  int32_t step;        // tiles between two tiles of one workgroup (32 = 32 KB: same DRAM channel)
  int32_t wg_per_cu;   // cap on resident workgroups per CU (0: none)
  int32_t barrier;     // barrier after every hop keeps a workgroup's wavefronts on one rank
  int32_t group_log2;  // 2^this ranks are read (written) between two barriers, where a kernel groups ranks
};

struct gg_tuning {
  int32_t threads;         // workgroup size of the general kernels
  int32_t chunks;          // access-type items per thread per tile: 1, 2, 4, 8
  int32_t blocks_per_cu;   // 0: no cap; >0: at most this many resident workgroups per CU (LDS reservation)
  int32_t nontemporal;     // 1: streaming (nt) loads and stores
  gg_walk_shape walk;      // overrides of the walking kernels' defaults
};

struct gg_ctx {
  gg_config cfg;
  int32_t L;       // phases per communicator, ceil(log2 p)
  int32_t R;       // communicators
  int device;
  int num_cus;
  gg_tuning tune;
  std::vector<uint16_t> sigma;  // [R][p] virtual rank -> world rank
  std::vector<uint16_t> inv;    // [R][p] world rank  -> virtual rank
  uint16_t* d_sigma;            // device copy of sigma
  // shuffle state
  int32_t* d_scratch;           // device int32[scratch_cap]
  int64_t scratch_cap;
  int64_t* d_offsets;           // device int64[p+1]
  int64_t* h_offsets_pinned;    // pinned staging for the upload
  std::vector<int64_t> offsets_cached;
};

// ---- Philox4x32-10 (Salmon et al., SC'11): counter (c0..c3), key (k0,k1) -> 4 words.
// One round: (hi0:lo0) = M0*c0, (hi1:lo1) = M1*c2,
//            c <- (hi1^c1^k0, lo1, hi0^c3^k1, lo0); key += (W0, W1) between rounds.
struct gg_u32x4 {
  uint32_t x, y, z, w;
};

__host__ __device__ inline gg_u32x4 gg_philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2,
                                                     uint32_t c3, uint32_t k0, uint32_t k1) {
  const uint32_t kM0 = 0xD2511F53u, kM1 = 0xCD9E8D57u;
  const uint32_t kW0 = 0x9E3779B9u, kW1 = 0xBB67AE85u;
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint64_t p0 = (uint64_t)kM0 * c0;
    const uint64_t p1 = (uint64_t)kM1 * c2;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    c1 = (uint32_t)p1;
    c3 = (uint32_t)p0;
    c0 = n0;
    c2 = n2;
    k0 += kW0;
    k1 += kW1;
  }
  return gg_u32x4{c0, c1, c2, c3};
}

enum { GG_TAG_COMM = 1, GG_TAG_SHUF = 2 };

// Resolves, once per device and with that device current, the device address of the static
// scratch array that gg_shuffle_noalloc uses (gg_shuffle.hip); called by gg_init.
int gg_static_scratch_setup(int device);

// Validation helpers (gg_ctx.hip)
int gg_check_ctx_device(const gg_ctx* ctx);
inline bool gg_is_pow2(int64_t x) { return x >= 1 && (x & (x - 1)) == 0; }
inline bool gg_aligned(const void* ptr, uintptr_t a) { return ((uintptr_t)ptr % a) == 0; }

// Launch geometry for a streaming kernel over `items` work items per grid row.
struct gg_grid {
  dim3 grid;
  dim3 block;
  int64_t tiles;       // tiles per row
  uint32_t lds_bytes;  // dynamic LDS reserved only to cap the workgroups resident on a CU; the kernels launched
                       // with it use no LDS of their own, so the cap is exactly what the reservation says
};
// `loads` = 16-byte loads one thread keeps in flight; the occupancy cap is stated for the
// pair kernel (6 loads per thread) and scaled so that every kernel keeps about the same
// number of bytes in flight per CU.
gg_grid gg_make_grid(const gg_ctx* ctx, int64_t items, int32_t chunks, int64_t rows, int32_t loads);

// Launch geometry of a walking kernel over `tiles` 1 KB tiles: workgroup bx handles the tiles
//   (bx / step) * step*waves*chunks + bx % step + i * step,   i < waves*chunks,
// so grid_x = ceil(tiles / (step*waves*chunks)) * step workgroups of 64*waves threads.
struct gg_walk_launch {
  gg_walk_shape shape;  // defaults resolved, chunks clamped to max_chunks
  int64_t grid_x;       // 0 when the walking form does not apply (chunks == 0 or the grid would not fit)
  uint32_t lds_bytes;   // LDS reserved (never touched) to cap the resident workgroups per CU; a kernel that
                        // also has static LDS (the payload ring: 8 KB of queue heads) fits fewer than asked
};
gg_walk_launch gg_walk_geometry(const gg_ctx* ctx, const gg_walk_shape& kernel_default, int32_t max_chunks,
                                int64_t tiles);

#endif  // GG_INTERNAL_H_
