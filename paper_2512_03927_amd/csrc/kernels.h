// Internal launcher interface between the C-ABI layer and the HIP kernels.
// Not part of the public boundary (that is include/odmoe.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/odmoe.h"

namespace odmoe {

// Where the weights of the i-th selected expert (rank i in idx) live.
//   resolved : resolved != nullptr, pointer = resolved[i]   (device array the router kernel filled)
//   resident : table != nullptr, pointer = table[table_off + idx[i]]   (device table, L*E entries);
//              idx[i] outside [0, n_experts) selects nothing: that rank gets gate weight 0
//   cacheless: otherwise, pointer = slot[i]                            (HBM slot bases by rank)
struct ExpertSrc {
  const void* slot[ODMOE_MAX_TOPK];
  const void* const* table;
  const void* const* resolved;
  int32_t table_off;
  int32_t n_experts;
};

struct Shape {
  int32_t H, F, E, k;
  int32_t dtype;  // odmoe_dtype
  // Expert weights are read in place from pinned host memory, across the host link.  The link is
  // saturated by about a hundred waves that each stream a long contiguous run; thousands of short
  // runs lose 4-7 % of its rate.
  int32_t host_link = 0;
  // odmoe_quant of the expert buffers: 0 = weights in `dtype`; ODMOE_Q_INT8_ROW = int8 codes with
  // one fp32 scale per weight row; ODMOE_Q_INT4_G64 = packed 4-bit codes with one fp32 scale per
  // group of 64; ODMOE_Q_F16 = binary16 weights (x, y and the router stay in `dtype`).
  int32_t quant = 0;
};

// Device scratch that lets the router spread one token over several blocks: logits
// [max_tokens, E] fp32 and counters [max_tokens] int32, the counters zero before the first launch
// (every launch leaves them zero).  Launches that share a scratch must not overlap.
struct RouteScratch {
  float* logits;
  int32_t* counters;
  int32_t max_tokens;
};
constexpr int32_t ROUTE_SPLIT_MAX_TOKENS = 16;

// Router GEMV + top-k + gate for T tokens.  idx_mirror (may be null) is a second int32[T*k]
// destination (host-mapped pinned memory) written together with idx.  With eptr_out != null the
// kernel also stores table[table_off + idx] there (T*k pointers), which saves the FFN kernels
// one dependent load.  With a scratch, more than 16 experts and T <= scratch->max_tokens the
// experts of a token are spread over several blocks (same results).
// With glue_x_prev != null (T must be 1, route_glue_fusable(sh) true) the token's input is the
// previous layer's glue, done at the head of the same kernel: x = rmsnorm(glue_x_prev +
// glue_y_prev) is written to glue_x_out (the bits launch_glue gives) and routed; `x` is not read.
hipError_t launch_route_topk(hipStream_t s, const Shape& sh, const void* Wg, const float* b,
                             const void* x, int32_t T, int32_t* idx, float* gate,
                             int32_t* idx_mirror, const void* const* table, int32_t table_off,
                             const void** eptr_out, const RouteScratch* scratch = nullptr,
                             const void* glue_x_prev = nullptr, const void* glue_y_prev = nullptr,
                             void* glue_x_out = nullptr);
bool route_glue_fusable(const Shape& sh);   // the hidden vector fits the router kernel's LDS

// h[i, :] = silu(W1 x) * (W3 x) for the k selected experts of ONE token.  hbuf: fp32 [k, F].
hipError_t launch_ffn_up(hipStream_t s, const Shape& sh, const ExpertSrc& src, const int32_t* idx,
                         const void* x, float* hbuf);

// y = sum_i gate[i] * (W2_i h_i) for ONE token; y in sh.dtype [H].
hipError_t launch_ffn_down(hipStream_t s, const Shape& sh, const ExpertSrc& src,
                           const int32_t* idx, const float* gate, const float* hbuf, void* y);

// The same two GEMVs over int8 expert buffers (codes W1 | W3 | W2 offset-binary, then fp32 scales
// s1[F] | s3[F] | s2[H]); launch_ffn_up / launch_ffn_down forward here when sh.quant says so.
bool q8_supported(const Shape& sh);   // H and F multiples of 16, H <= 8192
hipError_t launch_ffn_up_q8(hipStream_t s, const Shape& sh, const ExpertSrc& src, const int32_t* idx,
                            const void* x, float* hbuf);
hipError_t launch_ffn_down_q8(hipStream_t s, const Shape& sh, const ExpertSrc& src, const int32_t* idx,
                              const float* gate, const float* hbuf, void* y);

// ... and over 4-bit expert buffers (codes packed two per byte W1 | W3 | W2, then one fp32 scale
// per group of 64 weights s1[F][H/64] | s3[F][H/64] | s2[H][F/64]); sh.quant == ODMOE_Q_INT4_G64.
bool q4_supported(const Shape& sh);   // H and F multiples of 64, H <= 8192
hipError_t launch_ffn_up_q4(hipStream_t s, const Shape& sh, const ExpertSrc& src, const int32_t* idx,
                            const void* x, float* hbuf);
hipError_t launch_ffn_down_q4(hipStream_t s, const Shape& sh, const ExpertSrc& src, const int32_t* idx,
                              const float* gate, const float* hbuf, void* y);
// w[rows, cols] (dtype, cols a multiple of 64) -> packed 4-bit codes [rows, cols/2] and scales
// [rows, cols/64]: the codes of launch_quantize(ODMOE_Q_INT4_G64), two per byte.
hipError_t launch_quantize_pack4(hipStream_t s, const void* w, int32_t dtype, int64_t rows, int64_t cols,
                                 uint8_t* packed, float* scale);

// ... and over binary16 expert buffers W1 | W3 | W2 (layers of dtype fp32 only: x, h, y fp32);
// sh.quant == ODMOE_Q_F16.
bool f16_supported(const Shape& sh);   // fp32 layer, H and F multiples of 8, H <= 8192, F <= 32768
hipError_t launch_ffn_up_f16(hipStream_t s, const Shape& sh, const ExpertSrc& src, const int32_t* idx,
                             const void* x, float* hbuf);
hipError_t launch_ffn_down_f16(hipStream_t s, const Shape& sh, const ExpertSrc& src, const int32_t* idx,
                               const float* gate, const float* hbuf, void* y);
// w[n] (dtype) -> binary16 bits (nearest, ties to even, clipped to the largest finite value) in
// code, and the value they stand for rounded to dtype in deq; either may be null.
hipError_t launch_round_f16(hipStream_t s, const void* w, int32_t dtype, size_t n, uint16_t* code, void* deq);

// Symmetric absmax quantisation of w[rows, cols] (dtype) on the device; kind is an odmoe_quant.
// code (u8, offset-binary), scale (fp32, per row or per group of 64) and deq (code * scale rounded
// once to dtype) may each be null.
hipError_t launch_quantize(hipStream_t s, const void* w, int32_t dtype, int64_t rows, int64_t cols,
                           int32_t kind, uint8_t* code, float* scale, void* deq);

// glue = 1: x_next = rmsnorm(x + y) (eps 1e-6).  All [H] in sh.dtype.
hipError_t launch_glue(hipStream_t s, const Shape& sh, const void* x, const void* y, void* x_next);

// Prefill (bf16 and fp32 layers): tokens grouped by expert, grouped GEMMs on the matrix cores.
// Workspace sizes in bytes for T tokens; the workspace is carved by the launcher.
bool prefill_supported(const Shape& sh);  // H and F multiples of 64
size_t prefill_workspace_bytes(const Shape& sh, int32_t T);
hipError_t launch_prefill(hipStream_t s, const Shape& sh, const void* const* table,
                          int32_t table_off, const int32_t* idx, const float* gate, const void* x,
                          int32_t T, void* y, void* workspace, size_t workspace_bytes);
// The same in phases, for experts that are streamed in one at a time: bucket the token-slots;
// run both GEMMs for the chunk-list entries [tile_first, tile_first + tile_count) with the weights
// at expert_override (or from the table when null); combine.  The chunk list holds the experts
// in the order prefill_expert_order gives for their token-slot counts (count[E] -> order[E]: by
// count, the larger half interleaved with the smaller half), each with prefill_chunks_of(count)
// entries.  A range given to prefill_gemms must hold all entries of each expert it touches.
hipError_t prefill_sort(hipStream_t s, const Shape& sh, const int32_t* idx, int32_t T, void* workspace,
                        size_t workspace_bytes);
hipError_t prefill_gemms(hipStream_t s, const Shape& sh, const void* const* table, int32_t table_off,
                         const void* expert_override, int32_t tile_first, int32_t tile_count,
                         const void* x, int32_t T, void* workspace);
hipError_t prefill_combine(hipStream_t s, const Shape& sh, const float* gate, int32_t T, void* y,
                           void* workspace);
int prefill_chunks_of(int32_t count);
void prefill_expert_order(const int32_t* count, int32_t E, int32_t* order);

// Plain streaming kernel over `bytes` (multiple of 16): mode 0 copies src to dst, mode 1 only
// reads src (dst: 4 bytes of scratch).
hipError_t launch_probe(hipStream_t s, void* dst, const void* src, size_t bytes, int mode);

// One-time per-process kernel attribute setup (large dynamic LDS).
hipError_t kernels_init();

}  // namespace odmoe
