/*
 * Plain C program that drives libodmoe.so through include/odmoe.h alone (no Python, no torch):
 * a small cacheless stack, one decode token with and without expert hints, and once more with the
 * experts read in place from pinned host memory.
 *
 *   c_abi_demo <input file> <output file>
 *
 * Input file (little endian, written by the caller):
 *   int32 hidden, ffn, n_experts, top_k, n_layers, n_slots, dtype, glue
 *   then per layer: router Wg[E,H], then E expert buffers (W1|W3|W2), all in dtype
 *   then x[H] in dtype
 * Output file: y[H] in dtype, int32 idx[L,k], uint64 loads, uint64 hint_hits (second pass).
 * Exit status 0 on success; messages go to stderr.
 *
 * Device memory comes from the HIP runtime's C API; expert buffers live in pinned host memory
 * from odmoe_pinned_alloc, as the header asks for a cacheless stack.
 */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "odmoe.h"

#define HIP_OK(call)                                                              \
  do {                                                                            \
    hipError_t e_ = (call);                                                       \
    if (e_ != hipSuccess) {                                                       \
      fprintf(stderr, "%s: %s\n", #call, hipGetErrorString(e_));                  \
      return 2;                                                                   \
    }                                                                             \
  } while (0)
#define ODMOE_OK_OR_DIE(call)                                                     \
  do {                                                                            \
    int rc_ = (call);                                                             \
    if (rc_ != ODMOE_OK) {                                                        \
      fprintf(stderr, "%s -> %d: %s\n", #call, rc_, odmoe_last_error());          \
      return 3;                                                                   \
    }                                                                             \
  } while (0)

static int read_exact(FILE* f, void* dst, size_t bytes) { return fread(dst, 1, bytes, f) == bytes; }

int main(int argc, char** argv) {
  if (argc != 3) {
    fprintf(stderr, "usage: %s <input> <output>\n", argv[0]);
    return 1;
  }
  FILE* in = fopen(argv[1], "rb");
  if (!in) { perror(argv[1]); return 1; }
  int32_t hdr[8];
  if (!read_exact(in, hdr, sizeof hdr)) { fprintf(stderr, "short header\n"); return 1; }
  odmoe_config cfg = {hdr[0], hdr[1], hdr[2], hdr[3], hdr[4], hdr[5], hdr[6], hdr[7], ODMOE_Q_NONE};
  const int L = cfg.n_layers, E = cfg.n_experts, k = cfg.top_k;
  const size_t es = cfg.dtype == ODMOE_F32 ? 4 : 2;
  const size_t router_bytes = (size_t)E * cfg.hidden * es;
  const size_t expert_bytes = (size_t)3 * cfg.hidden * cfg.ffn * es;
  const size_t x_bytes = (size_t)cfg.hidden * es;
  if (L < 1 || L > 64 || E < 1 || E > ODMOE_MAX_EXPERTS || cfg.n_slots < k) {
    fprintf(stderr, "this demo wants a cacheless stack of 1..64 layers\n");
    return 1;
  }

  void** router_w = calloc((size_t)L, sizeof(void*));
  void** expert_w = calloc((size_t)L * E, sizeof(void*));
  void* stage = malloc(router_bytes > x_bytes ? router_bytes : x_bytes);
  if (!router_w || !expert_w || !stage) return 1;
  for (int l = 0; l < L; ++l) {
    if (!read_exact(in, stage, router_bytes)) { fprintf(stderr, "short router\n"); return 1; }
    HIP_OK(hipMalloc(&router_w[l], router_bytes));
    HIP_OK(hipMemcpy(router_w[l], stage, router_bytes, hipMemcpyHostToDevice));
    for (int e = 0; e < E; ++e) {
      void* pinned = NULL;
      ODMOE_OK_OR_DIE(odmoe_pinned_alloc(expert_bytes, &pinned));
      if (!read_exact(in, pinned, expert_bytes)) { fprintf(stderr, "short expert\n"); return 1; }
      expert_w[(size_t)l * E + e] = pinned;
    }
  }
  if (!read_exact(in, stage, x_bytes)) { fprintf(stderr, "short x\n"); return 1; }
  fclose(in);
  void *x_dev = NULL, *y_dev = NULL;
  HIP_OK(hipMalloc(&x_dev, x_bytes));
  HIP_OK(hipMalloc(&y_dev, x_bytes));
  HIP_OK(hipMemcpy(x_dev, stage, x_bytes, hipMemcpyHostToDevice));

  hipStream_t compute;
  HIP_OK(hipStreamCreate(&compute));
  odmoe_layer_t* h = NULL;
  ODMOE_OK_OR_DIE(odmoe_layer_init(&cfg, (const void* const*)router_w, NULL, (const void* const*)expert_w,
                                   compute, NULL, &h));

  int32_t* idx = calloc((size_t)L * k, sizeof(int32_t));
  void* y_first = malloc(x_bytes);
  void* y_second = malloc(x_bytes);
  if (!idx || !y_first || !y_second) return 1;
  odmoe_stats st;
  memset(&st, 0, sizeof st);
  /* pass 1: no hints; the library tells us which experts the router used */
  ODMOE_OK_OR_DIE(odmoe_decode_step(h, x_dev, y_dev, NULL, idx, &st));
  HIP_OK(hipMemcpy(y_first, y_dev, x_bytes, hipMemcpyDeviceToHost));
  if (st.loads != (uint64_t)L * k) { fprintf(stderr, "loads %llu\n", (unsigned long long)st.loads); return 4; }
  /* pass 2: those experts as hints: same output, every hint confirmed */
  ODMOE_OK_OR_DIE(odmoe_decode_step(h, x_dev, y_dev, idx, NULL, &st));
  HIP_OK(hipMemcpy(y_second, y_dev, x_bytes, hipMemcpyDeviceToHost));
  if (memcmp(y_first, y_second, x_bytes) != 0) { fprintf(stderr, "hints changed the output\n"); return 4; }

  /* pass 3: a second handle with no slot pool at all, whose kernels read the same pinned expert
     buffers in place (n_slots = 0 accepts any address the GPU can read): same output again */
  {
    odmoe_config cfg_in_place = cfg;
    cfg_in_place.n_slots = 0;
    odmoe_layer_t* h2 = NULL;
    void* y_third = malloc(x_bytes);
    if (!y_third) return 1;
    ODMOE_OK_OR_DIE(odmoe_layer_init(&cfg_in_place, (const void* const*)router_w, NULL,
                                     (const void* const*)expert_w, compute, NULL, &h2));
    ODMOE_OK_OR_DIE(odmoe_decode_step(h2, x_dev, y_dev, NULL, NULL, NULL));
    HIP_OK(hipStreamSynchronize(compute));
    HIP_OK(hipMemcpy(y_third, y_dev, x_bytes, hipMemcpyDeviceToHost));
    ODMOE_OK_OR_DIE(odmoe_layer_destroy(h2));
    if (memcmp(y_first, y_third, x_bytes) != 0) { fprintf(stderr, "reading experts in place changed the output\n"); return 4; }
    free(y_third);
  }

  FILE* out = fopen(argv[2], "wb");
  if (!out) { perror(argv[2]); return 1; }
  fwrite(y_second, 1, x_bytes, out);
  fwrite(idx, sizeof(int32_t), (size_t)L * k, out);
  fwrite(&st.loads, sizeof(uint64_t), 1, out);
  fwrite(&st.hint_hits, sizeof(uint64_t), 1, out);
  fclose(out);

  ODMOE_OK_OR_DIE(odmoe_layer_destroy(h));
  for (int l = 0; l < L; ++l) {
    HIP_OK(hipFree(router_w[l]));
    for (int e = 0; e < E; ++e) ODMOE_OK_OR_DIE(odmoe_pinned_free(expert_w[(size_t)l * E + e]));
  }
  HIP_OK(hipFree(x_dev));
  HIP_OK(hipFree(y_dev));
  HIP_OK(hipStreamDestroy(compute));
  free(router_w); free(expert_w); free(stage); free(idx); free(y_first); free(y_second);
  return 0;
}
