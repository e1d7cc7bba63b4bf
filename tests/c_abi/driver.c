/*
 * Plain-C caller of the gg.h ABI: no Python, no torch.  Reads a problem from a
 * binary file, runs it through the library on the GPU, writes the results.
 * Used by tests/test_gpu_c_abi.py, which compares the output with the CPU oracle.
 *
 * input file:  int32 p, topology, avg_mode, staleness, steps, first_step;
 *              int64 n, rank_stride; uint64 seed; float lr, momentum;
 *              float w[p*rank_stride], g[p*rank_stride], m[p*rank_stride]
 * output file: float w[p*rank_stride], m[p*rank_stride]; int32 send_to[steps*p]
 */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "gg.h"

#define DIE(msg)                          \
  do {                                    \
    fprintf(stderr, "driver: %s\n", msg); \
    return 1;                             \
  } while (0)

int main(int argc, char** argv) {
  if (argc != 3) DIE("usage: driver <input> <output>");
  FILE* in = fopen(argv[1], "rb");
  if (!in) DIE("cannot open input");
  int32_t hdr[6];
  int64_t dims[2];
  uint64_t seed;
  float hyper[2];
  if (fread(hdr, sizeof hdr, 1, in) != 1 || fread(dims, sizeof dims, 1, in) != 1 ||
      fread(&seed, sizeof seed, 1, in) != 1 || fread(hyper, sizeof hyper, 1, in) != 1)
    DIE("short header");
  const int32_t p = hdr[0], steps = hdr[4], first = hdr[5];
  const size_t count = (size_t)p * (size_t)dims[1];
  float* host = (float*)malloc(3 * count * sizeof(float));
  int32_t* partners = (int32_t*)malloc((size_t)steps * p * sizeof(int32_t));
  if (!host || !partners) DIE("out of memory");
  if (fread(host, sizeof(float), 3 * count, in) != 3 * count) DIE("short payload");
  fclose(in);

  gg_config cfg;
  cfg.p = p;
  cfg.topology = hdr[1];
  cfg.n = dims[0];
  cfg.rank_stride = dims[1];
  cfg.num_comms = 0;
  cfg.avg_mode = hdr[2];
  cfg.staleness = hdr[3];
  cfg.reserved = 0;
  cfg.seed = seed;
  cfg.lr = hyper[0];
  cfg.momentum = hyper[1];
  gg_ctx* ctx = NULL;
  int rc = gg_init(&cfg, &ctx);
  if (rc != GG_OK) DIE(gg_strerror(rc));

  float *w, *g, *m;
  if (hipMalloc((void**)&w, count * sizeof(float)) != hipSuccess || hipMalloc((void**)&g, count * sizeof(float)) != hipSuccess ||
      hipMalloc((void**)&m, count * sizeof(float)) != hipSuccess)
    DIE("hipMalloc failed");
  hipStream_t stream;
  if (hipStreamCreate(&stream) != hipSuccess) DIE("hipStreamCreate failed");
  if (hipMemcpy(w, host, count * sizeof(float), hipMemcpyHostToDevice) != hipSuccess ||
      hipMemcpy(g, host + count, count * sizeof(float), hipMemcpyHostToDevice) != hipSuccess ||
      hipMemcpy(m, host + 2 * count, count * sizeof(float), hipMemcpyHostToDevice) != hipSuccess)
    DIE("upload failed");

  for (int32_t t = 0; t < steps; ++t) {
    rc = gg_partner(ctx, first + t, partners + (size_t)t * p, NULL);
    if (rc != GG_OK) DIE(gg_strerror(rc));
    rc = gg_gossip_step(ctx, first + t, w, g, m, NULL, NULL, 0, stream);
    if (rc != GG_OK) DIE(gg_strerror(rc));
  }
  if (hipStreamSynchronize(stream) != hipSuccess) DIE("stream failed");
  if (hipMemcpy(host, w, count * sizeof(float), hipMemcpyDeviceToHost) != hipSuccess ||
      hipMemcpy(host + count, m, count * sizeof(float), hipMemcpyDeviceToHost) != hipSuccess)
    DIE("download failed");

  FILE* out = fopen(argv[2], "wb");
  if (!out) DIE("cannot open output");
  if (fwrite(host, sizeof(float), 2 * count, out) != 2 * count ||
      fwrite(partners, sizeof(int32_t), (size_t)steps * p, out) != (size_t)steps * p)
    DIE("short write");
  fclose(out);
  rc = gg_destroy(ctx);
  if (rc != GG_OK) DIE(gg_strerror(rc));
  (void)hipStreamDestroy(stream);
  (void)hipFree(w);
  (void)hipFree(g);
  (void)hipFree(m);
  free(host);
  free(partners);
  return 0;
}
