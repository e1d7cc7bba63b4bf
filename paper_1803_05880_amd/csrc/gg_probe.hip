// Measurement aids (gg_probe.h): calibration copy, stand-ins for the forward/backward
// computation, launch-shape knobs.  Nothing here is a step of the method.
#include "gg_internal.h"

namespace {

__global__ void __launch_bounds__(256) copy_kernel(v4f* dst, const v4f* src, int64_t count) {
  const int64_t step = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += step)
    __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

__global__ void __launch_bounds__(256) busy_kernel(int64_t iters, float* sink) {
  float x = 1.0f + (float)threadIdx.x * 1e-7f, y = 0.999999f;
  for (int64_t i = 0; i < iters; ++i) x = x * y + 1e-9f;
  if (x == -1.0f) *sink = x;  // never true: the chain stays positive
}

// Read 16 bytes, run a dependent chain on them, write them back: arithmetic and memory
// traffic in a ratio set by iters.  A fixed number of workgroups strides over the buffer,
// four chunks per thread in flight, so the stand-in leaves wavefront slots to the kernels
// it runs beside (as a computation that is not purely memory-bound does).
__global__ void __launch_bounds__(256) stream_kernel(int64_t iters, v4f* buf, int64_t count) {
  const int64_t step = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += 4 * step) {
    v4f x[4];
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (i + u * step < count) x[u] = __builtin_nontemporal_load(buf + i + u * step);
#pragma unroll
    for (int u = 0; u < 4; ++u) x[u] = x[u] * 0.0f + 1.0f;  // whatever finite values the buffer held: start from 1
    for (int64_t k = 0; k < iters; ++k) {
#pragma unroll
      for (int u = 0; u < 4; ++u) x[u] = x[u] * 0.999999f + 1e-9f;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (i + u * step < count) __builtin_nontemporal_store(x[u], buf + i + u * step);
  }
}

}  // namespace

#ifndef GG_BUILD_ID
#define GG_BUILD_ID "unknown"
#endif
extern "C" const char* gg_build_id(void) { return GG_BUILD_ID; }

extern "C" int gg_copy_probe(void* dst, const void* src, int64_t nbytes, void* stream) {
  if (!dst || !src || nbytes < 0 || nbytes % 16) return GG_ERR_ARG;
  if (!gg_aligned(dst, 16) || !gg_aligned(src, 16)) return GG_ERR_ALIGN;
  if (nbytes == 0) return GG_OK;
  // one wavefront per workgroup, one 16-byte chunk per thread, no occupancy cap: the
  // shape that copies fastest on this part
  const int64_t count = nbytes / 16;
  int64_t blocks = (count + 63) / 64;
  if (blocks > 0x7fffffffLL) blocks = 0x7fffffffLL;
  hipLaunchKernelGGL(copy_kernel, dim3((unsigned)blocks), dim3(64), 0, (hipStream_t)stream, (v4f*)dst,
                     (const v4f*)src, count);
  GG_HIP_TRY(hipGetLastError());
  return GG_OK;
}

extern "C" int gg_busy_probe(int64_t iters, int32_t blocks, float* sink, void* stream) {
  if (!sink || iters < 0 || blocks < 1 || blocks > 65536) return GG_ERR_ARG;
  if (!gg_aligned(sink, 4)) return GG_ERR_ALIGN;
  hipLaunchKernelGGL(busy_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, iters, sink);
  GG_HIP_TRY(hipGetLastError());
  return GG_OK;
}

extern "C" int gg_stream_probe(int64_t iters, int32_t blocks, void* buf, int64_t nbytes, void* stream) {
  if (!buf || iters < 0 || blocks < 1 || blocks > 65536 || nbytes < 0 || nbytes % 16) return GG_ERR_ARG;
  if (!gg_aligned(buf, 16)) return GG_ERR_ALIGN;
  if (nbytes == 0) return GG_OK;
  hipLaunchKernelGGL(stream_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, iters, (v4f*)buf,
                     nbytes / 16);
  GG_HIP_TRY(hipGetLastError());
  return GG_OK;
}

extern "C" int gg_set_tuning(gg_ctx* ctx, int32_t key, int32_t value) {
  if (!ctx) return GG_ERR_ARG;
  gg_tuning& tn = ctx->tune;
  const bool one_of_1248 = value == 1 || value == 2 || value == 4 || value == 8;
  switch (key) {
    case GG_TUNE_THREADS:
      if (value != 64 && value != 128 && value != 256) return GG_ERR_ARG;
      tn.threads = value;
      return GG_OK;
    case GG_TUNE_CHUNKS:
      if (!one_of_1248) return GG_ERR_ARG;
      tn.chunks = value;
      return GG_OK;
    case GG_TUNE_BLOCKS_PER_CU:
      if (value != 0 && (value < 3 || value > 64)) return GG_ERR_ARG;
      tn.blocks_per_cu = value;
      return GG_OK;
    case GG_TUNE_NONTEMPORAL:
      if (value != 0 && value != 1) return GG_ERR_ARG;
      tn.nontemporal = value;
      return GG_OK;
    case GG_TUNE_WALK_CHUNKS:
      if (value != 0 && !one_of_1248) return GG_ERR_ARG;
      if (tn.walk.waves != GG_WALK_UNSET && value * tn.walk.waves > 8) return GG_ERR_ARG;
      tn.walk.chunks = value;
      return GG_OK;
    case GG_TUNE_WALK_WAVES:
      if (!one_of_1248) return GG_ERR_ARG;
      if (tn.walk.chunks != GG_WALK_UNSET && value * tn.walk.chunks > 8) return GG_ERR_ARG;
      tn.walk.waves = value;
      return GG_OK;
    case GG_TUNE_WALK_STEP:
      if (value < 1 || value > 65536) return GG_ERR_ARG;
      tn.walk.step = value;
      return GG_OK;
    case GG_TUNE_WALK_WG_PER_CU:
      if (value != 0 && (value < 3 || value > 64)) return GG_ERR_ARG;
      tn.walk.wg_per_cu = value;
      return GG_OK;
    case GG_TUNE_WALK_BARRIER:
      if (value != 0 && value != 1) return GG_ERR_ARG;
      tn.walk.barrier = value;
      return GG_OK;
    case GG_TUNE_WALK_GROUP_LOG2:
      if (value < 0 || value > 3) return GG_ERR_ARG;
      tn.walk.group_log2 = value;
      return GG_OK;
    default:
      return GG_ERR_ARG;
  }
}
