// Device helpers and launch policies shared by the decode GEMV kernels (stored-dtype weights in
// decode_kernels.hip, int8 weights in quant_kernels.hip).  Internal: not part of the boundary.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.h"

namespace odmoe {

constexpr int WAVE = 64;
typedef uint16_t bf16_t;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

// fp32 -> bf16, round to nearest even (finite values).
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

template <typename T>
struct DT;
template <>
struct DT<float> {
  static constexpr int VEC = 4;  // elements per 128-bit load
  static __device__ __forceinline__ void unpack(u32x4 q, float* f) {
    f[0] = __uint_as_float(q.x); f[1] = __uint_as_float(q.y);
    f[2] = __uint_as_float(q.z); f[3] = __uint_as_float(q.w);
  }
  static __device__ __forceinline__ float to_f32(float v) { return v; }
  static __device__ __forceinline__ float from_f32(float v) { return v; }
};
template <>
struct DT<bf16_t> {
  static constexpr int VEC = 8;
  static __device__ __forceinline__ void unpack(u32x4 q, float* f) {
    f[0] = bf16_lo(q.x); f[1] = bf16_hi(q.x); f[2] = bf16_lo(q.y); f[3] = bf16_hi(q.y);
    f[4] = bf16_lo(q.z); f[5] = bf16_hi(q.z); f[6] = bf16_lo(q.w); f[7] = bf16_hi(q.w);
  }
  static __device__ __forceinline__ float to_f32(bf16_t v) { return __uint_as_float((uint32_t)v << 16); }
  static __device__ __forceinline__ bf16_t from_f32(float v) { return f32_to_bf16(v); }
};

template <typename T>
__device__ __forceinline__ u32x4 load16(const T* p) {
  return *reinterpret_cast<const u32x4*>(p);
}
// Streaming load for weights: each byte is used once, keep it out of the way of reused lines.
// Expert pointers reach the kernels through a struct or a table, so the compiler cannot tell
// that they are global addresses; the explicit address-space cast turns what would be flat
// loads into global loads.
typedef const __attribute__((address_space(1))) u32x4* global_u32x4_ptr;
template <typename T>
__device__ __forceinline__ u32x4 load16_stream(const T* p) {
  return __builtin_nontemporal_load((global_u32x4_ptr)(p));
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, WAVE);
  return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, WAVE);
  return v;
}

// Base address of the expert of rank i.  idx reaches the table path from the caller's device
// memory, which the host cannot check without blocking: an entry that is not an expert id must not
// index past the table.  It is replaced by expert 0 and *valid is cleared; the w2 kernels then give
// that rank the gate weight 0, so it adds nothing to y (as in the grouped path).  No branch: a
// null test on the pointer cost the w2 GEMV of the Mixtral layer 11 us of 37, and forcing the
// pointer into scalar registers 4 us.
__device__ __forceinline__ const void* expert_ptr(const ExpertSrc& s, const int32_t* idx, int i,
                                                  bool* valid = nullptr) {
  if (valid) *valid = true;
  if (s.resolved) return s.resolved[i];
  if (!s.table) return s.slot[i];
  const uint32_t e = (uint32_t)idx[i];
  const bool ok = e < (uint32_t)s.n_experts;
  if (valid) *valid = ok;
  return s.table[s.table_off + (ok ? e : 0u)];
}

// Launch-shape overrides for tuning sweeps, compiled in only with -DODMOE_TUNING (never in the
// library that ships: the expert-group count changes the order of fp32 additions).  0 = the
// built-in policy.  Read once from the environment by kernels_init(): ODMOE_TUNE_UP_RPW (rows per
// wave of the w1/w3 GEMV), ODMOE_TUNE_DOWN_RPB (rows per block of the w2 GEMV), ODMOE_TUNE_DOWN_EG
// (its expert groups per block), ODMOE_TUNE_ROUTE_SPLIT_E (fewest experts for the multi-block
// router), ODMOE_TUNE_Q8_RIF (rows in flight per wave of the int8 w2 GEMV).
#ifdef ODMOE_TUNING
extern int g_tune_up_rpw, g_tune_down_rpb, g_tune_down_eg, g_tune_route_split_e, g_tune_q8_rif;
#else
constexpr int g_tune_up_rpw = 0, g_tune_down_rpb = 0, g_tune_down_eg = 0, g_tune_route_split_e = 0,
              g_tune_q8_rif = 0;
#endif

// Compute units of the current device (256 on MI355X; cached after the first query).
int num_cu();

// Split of the NC column chunks of a w2 row over the waves of a block: CPW chunks per wave.
// Up to 4 chunks per wave (blocks of up to 16 waves) with the least padding, ties going to
// more chunks per wave; rows too long for that take 5..8 chunks per wave (up to 8 waves).
inline bool pick_down_split(int nc, int* cpw_out, int* nwb_out) {
  int best_cpw = 0, best_waste = 1 << 30;
  for (int cpw = 1; cpw <= 4; ++cpw) {
    const int nwb = (nc + cpw - 1) / cpw;
    if (nwb > 16) continue;
    const int waste = nwb * cpw - nc;
    if (waste <= best_waste) { best_waste = waste; best_cpw = cpw; }
  }
  for (int cpw = 5; cpw <= 8 && !best_cpw; ++cpw)
    if ((nc + cpw - 1) / cpw <= 8) best_cpw = cpw;
  if (!best_cpw) return false;
  *cpw_out = best_cpw;
  *nwb_out = (nc + best_cpw - 1) / best_cpw;
  return true;
}

// Block shape of the w2 GEMV for a row split into nwb column slices of cpw chunks: expert groups
// per block (waves left over in a block take different experts) and output rows per block.
// tune_eg / tune_rpb: overrides of tuning builds (0 = none).
inline void down_block_shape(const Shape& sh, int cpw, int nwb, int tune_eg, int tune_rpb, int* n_eg_out,
                             int* rpb_out) {
  const int max_waves = cpw <= 4 ? 16 : 8;
  int n_eg = 1;
  if (nwb <= 2) n_eg = sh.k < max_waves / nwb ? sh.k : max_waves / nwb;
  else if (nwb <= 4) n_eg = sh.k < 2 ? sh.k : 2;   // blocks of at least 6 waves keep enough loads in flight
  if (n_eg > 8) n_eg = 8;
  if (tune_eg > 0) n_eg = tune_eg;
  if (n_eg > max_waves / nwb) n_eg = max_waves / nwb;   // block size limit of the kernel
  if (n_eg > sh.k) n_eg = sh.k;
  if (n_eg < 1) n_eg = 1;
  int rpb = (sh.H + num_cu() - 1) / num_cu();
  if (n_eg > 1 && nwb <= 2 && rpb > 4) rpb = 4;  // small layers: more, shorter blocks
  rpb = (rpb + 1) & ~1;              // two rows in flight
  // Across the host link: fewer blocks with longer runs.  The expert groups stay as they are, so
  // that the order of the fp32 additions, and with it every output bit, is that of experts in HBM.
  if (rpb > 64 || sh.host_link) rpb = 64;
  if (tune_rpb > 0) rpb = (tune_rpb + 1) & ~1;
  *n_eg_out = n_eg;
  *rpb_out = rpb;
}

}  // namespace odmoe
