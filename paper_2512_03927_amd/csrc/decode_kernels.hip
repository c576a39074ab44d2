// Decode-path kernels for gfx950 (wave64): router + top-k gate, the two expert GEMVs with the
// SiLU gate and the weighted combine, and the inter-layer glue.
//
// The expert GEMVs are bound by HBM bandwidth (one multiply-add per weight element, every weight
// read exactly once per token), so they stream the weights with 128-bit non-temporal loads,
// keep the input vector slice in registers (in LDS for shapes too large for that) and never
// touch the matrix cores.
#include "gemv_common.hpp"

#include <cstdlib>

namespace odmoe {
namespace {

// ---------------------------------------------------------------------------------------------
// LDS layout of an fp32 vector that 128-bit weight loads are multiplied with.  Vector element
// group v (VEC consecutive elements, the ones lane v%64 of chunk v/64 multiplies) is stored so
// that every ds_read_b128 of a wave touches 64 consecutive float4s:
//   VEC = 4 :  float4 at  chunk*256 + lane*4
//   VEC = 8 :  float4 at  chunk*512 + lane*4  and  chunk*512 + 256 + lane*4
// ---------------------------------------------------------------------------------------------
template <int VEC>
__device__ __forceinline__ int lds_pos(int v, int half) {
  return (v >> 6) * (WAVE * VEC) + half * (WAVE * 4) + (v & 63) * 4;
}

// dot( row[0:n], vec ) over one wave; vec is in LDS in the layout above; n % VEC == 0.
template <typename T>
__device__ __forceinline__ float wave_dot(const T* __restrict__ row, const float* __restrict__ svec,
                                          int nvec, int lane) {
  constexpr int VEC = DT<T>::VEC;
  float acc = 0.f;
  int v = lane;
#pragma unroll 4
  for (; v < nvec; v += WAVE) {
    u32x4 q = load16_stream(row + (size_t)v * VEC);
    float f[VEC];
    DT<T>::unpack(q, f);
    f32x4 a = *reinterpret_cast<const f32x4*>(svec + lds_pos<VEC>(v, 0));
    acc = fmaf(f[0], a.x, acc); acc = fmaf(f[1], a.y, acc);
    acc = fmaf(f[2], a.z, acc); acc = fmaf(f[3], a.w, acc);
    if constexpr (VEC == 8) {
      f32x4 b = *reinterpret_cast<const f32x4*>(svec + lds_pos<VEC>(v, 1));
      acc = fmaf(f[4], b.x, acc); acc = fmaf(f[5], b.y, acc);
      acc = fmaf(f[6], b.z, acc); acc = fmaf(f[7], b.w, acc);
    }
  }
  return wave_sum(acc);
}

// Two rows against the same vector (the w1 / w3 pair): twice the loads in flight per wave.
template <typename T>
__device__ __forceinline__ void wave_dot2(const T* __restrict__ row_a, const T* __restrict__ row_b,
                                          const float* __restrict__ svec, int nvec, int lane,
                                          float& out_a, float& out_b) {
  constexpr int VEC = DT<T>::VEC;
  float acc_a = 0.f, acc_b = 0.f;
#pragma unroll 4
  for (int v = lane; v < nvec; v += WAVE) {
    u32x4 qa = load16_stream(row_a + (size_t)v * VEC);
    u32x4 qb = load16_stream(row_b + (size_t)v * VEC);
    float fa[VEC], fb[VEC];
    DT<T>::unpack(qa, fa);
    DT<T>::unpack(qb, fb);
    f32x4 x0 = *reinterpret_cast<const f32x4*>(svec + lds_pos<VEC>(v, 0));
    acc_a = fmaf(fa[0], x0.x, acc_a); acc_a = fmaf(fa[1], x0.y, acc_a);
    acc_a = fmaf(fa[2], x0.z, acc_a); acc_a = fmaf(fa[3], x0.w, acc_a);
    acc_b = fmaf(fb[0], x0.x, acc_b); acc_b = fmaf(fb[1], x0.y, acc_b);
    acc_b = fmaf(fb[2], x0.z, acc_b); acc_b = fmaf(fb[3], x0.w, acc_b);
    if constexpr (VEC == 8) {
      f32x4 x1 = *reinterpret_cast<const f32x4*>(svec + lds_pos<VEC>(v, 1));
      acc_a = fmaf(fa[4], x1.x, acc_a); acc_a = fmaf(fa[5], x1.y, acc_a);
      acc_a = fmaf(fa[6], x1.z, acc_a); acc_a = fmaf(fa[7], x1.w, acc_a);
      acc_b = fmaf(fb[4], x1.x, acc_b); acc_b = fmaf(fb[5], x1.y, acc_b);
      acc_b = fmaf(fb[6], x1.z, acc_b); acc_b = fmaf(fb[7], x1.w, acc_b);
    }
  }
  out_a = wave_sum(acc_a);
  out_b = wave_sum(acc_b);
}

// Stage n elements of a stored-dtype vector into LDS as fp32 (layout above).  n % VEC == 0.
template <typename T, int VEC_OF_WEIGHTS>
__device__ __forceinline__ void stage_vec(const T* __restrict__ src, float* __restrict__ svec, int n) {
  constexpr int SV = DT<T>::VEC;  // elements per 128-bit load of the source
  for (int s = threadIdx.x; s * SV < n; s += blockDim.x) {
    float f[SV];
    DT<T>::unpack(load16(src + (size_t)s * SV), f);
#pragma unroll
    for (int q = 0; q < SV / 4; ++q) {
      int f4 = s * (SV / 4) + q;  // index of this float4 in the source vector
      int v, half;
      if constexpr (VEC_OF_WEIGHTS == 8) { v = f4 >> 1; half = f4 & 1; } else { v = f4; half = 0; }
      *reinterpret_cast<f32x4*>(svec + lds_pos<VEC_OF_WEIGHTS>(v, half)) =
          f32x4{f[4 * q], f[4 * q + 1], f[4 * q + 2], f[4 * q + 3]};
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Inter-layer glue for one block: z = x + y, out = z / sqrt(mean(z^2) + 1e-6), rounded to the
// storage dtype and handed element by element to `store`.  The sum of squares is taken in the
// order of a block of 1024 threads (thread v sums elements v, v + 1024, ...; waves of 64
// consecutive threads are reduced as a tree; the 16 wave sums are added in order), whatever the
// real block size (any divisor of 1024 that is a multiple of 64): the stand-alone glue kernel and
// the router kernels that start with the glue give the same bits.  part: 16 floats of LDS.
// ---------------------------------------------------------------------------------------------
template <typename T, typename Store>
__device__ __forceinline__ void glue_block(const T* __restrict__ xp, const T* __restrict__ yp, int H,
                                           float* part, Store store) {
  const int lane = threadIdx.x & 63;
  for (int v = threadIdx.x; v < 1024; v += blockDim.x) {
    float ss = 0.f;
    for (int i = v; i < H; i += 1024) {
      const float z = DT<T>::to_f32(xp[i]) + DT<T>::to_f32(yp[i]);
      ss = fmaf(z, z, ss);
    }
    ss = wave_sum(ss);
    if (lane == 0) part[v >> 6] = ss;
  }
  __syncthreads();
  float tot = 0.f;
  for (int w = 0; w < 16; ++w) tot += part[w];
  const float scale = 1.f / sqrtf(tot / (float)H + 1e-6f);
  for (int i = threadIdx.x; i < H; i += blockDim.x) {
    const float z = DT<T>::to_f32(xp[i]) + DT<T>::to_f32(yp[i]);
    store(i, DT<T>::from_f32(z * scale));
  }
}

// ---------------------------------------------------------------------------------------------
// Router GEMV + top-k + renormalised softmax gate.
// Logits are summed in float64 and rounded once to fp32, so the selection agrees with a float64
// reference rounded the same way regardless of summation order.  Ties: lowest index first.
// ---------------------------------------------------------------------------------------------

// One wave: logit of one expert row against one token, float64 accumulation (all lanes get it).
template <typename T>
__device__ __forceinline__ double wave_logit(const T* __restrict__ row, const T* __restrict__ xt, int nvec,
                                             int lane) {
  constexpr int VEC = DT<T>::VEC;
  constexpr int U = 8;            // 16-byte groups per lane whose loads are issued together
  double acc0 = 0.0, acc1 = 0.0;  // two chains: half the dependent-FMA latency
  // All loads of a round go out before the first is used: a row of up to U*64 groups (4096 bf16
  // elements) costs one memory latency instead of one per pair of groups.
  for (int g0 = 0; g0 < nvec; g0 += U * WAVE) {   // g0: first group of the round (wave-uniform)
    u32x4 qw[U], qx[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (g0 + u * WAVE >= nvec) break;             // whole wave past the end of the row
      const int v = g0 + u * WAVE + lane;
      if (v < nvec) {
        qw[u] = load16(row + (size_t)v * VEC);
        qx[u] = load16(xt + (size_t)v * VEC);
      } else {
        qw[u] = u32x4{0u, 0u, 0u, 0u};
        qx[u] = u32x4{0u, 0u, 0u, 0u};
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (g0 + u * WAVE >= nvec) break;
      float fw[VEC], fx[VEC];
      DT<T>::unpack(qw[u], fw);
      DT<T>::unpack(qx[u], fx);
#pragma unroll
      for (int j = 0; j < VEC; ++j) {
        if (u & 1) acc1 = fma((double)fw[j], (double)fx[j], acc1);
        else acc0 = fma((double)fw[j], (double)fx[j], acc0);
      }
    }
  }
  return wave_sum(acc0 + acc1);
}

// The whole block: from the E logits in slog (LDS, complete and visible) to idx / gate of token t.
// sel_v / sel_i: LDS scratch of ODMOE_MAX_TOPK entries.
__device__ __forceinline__ void select_topk_and_gate(const float* slog, float* sel_v, int* sel_i, int E,
                                                     int k, int t, int32_t* __restrict__ idx,
                                                     float* __restrict__ gate,
                                                     int32_t* __restrict__ idx_mirror,
                                                     const void* const* __restrict__ table,
                                                     int table_off, const void** __restrict__ eptr_out) {
  // NaN logits take no position in the order below; pre-filling the selection keeps every
  // index in range even then (which experts are picked is unspecified in that case).
  if (threadIdx.x < k) { sel_v[threadIdx.x] = 0.f; sel_i[threadIdx.x] = threadIdx.x; }
  __syncthreads();
  // Position of every expert in the total order (logit descending, index ascending): the
  // number of experts that come before it.  Experts at positions < k are the selection.
  for (int e = threadIdx.x; e < E; e += blockDim.x) {
    const float v = slog[e];
    int before = 0;
    for (int j = 0; j < E; ++j) {
      const float u = slog[j];
      before += (u > v) || (u == v && j < e);
    }
    if (before < k) { sel_v[before] = v; sel_i[before] = e; }
  }
  __syncthreads();
  if (threadIdx.x < k) {
    const int i = threadIdx.x;
    const float v0 = sel_v[0];
    float s = 0.f;
    for (int j = 0; j < k; ++j) s += expf(sel_v[j] - v0);  // fixed order j = 0..k-1
    const int e = sel_i[i];
    idx[(size_t)t * k + i] = e;
    gate[(size_t)t * k + i] = expf(sel_v[i] - v0) / s;
    if (idx_mirror) idx_mirror[(size_t)t * k + i] = e;
    if (eptr_out) eptr_out[(size_t)t * k + i] = table[table_off + e];
  }
}

// The glue of the previous layer done at the head of a router kernel (one token): the router's
// input x = rmsnorm(x_prev + y_prev) is made in LDS by every block, and written to x_out by one.
template <typename T>
struct GlueIn {
  const T* x_prev;
  const T* y_prev;
  T* x_out;
};

// One block per token: one wave per expert, in rounds.  GLUE: one token whose input comes out of
// the previous layer's glue, computed here first (dynamic LDS: H elements of T).
template <typename T, bool GLUE>
__global__ __launch_bounds__(512) void route_topk_kernel(const T* __restrict__ Wg,
                                                          const float* __restrict__ bias,
                                                          const T* __restrict__ x, int H, int E, int k,
                                                          int32_t* __restrict__ idx,
                                                          float* __restrict__ gate,
                                                          int32_t* __restrict__ idx_mirror,
                                                          const void* const* __restrict__ table,
                                                          int table_off,
                                                          const void** __restrict__ eptr_out, GlueIn<T> gl) {
  __shared__ float slog[ODMOE_MAX_EXPERTS];
  __shared__ float sel_v[ODMOE_MAX_TOPK];
  __shared__ int sel_i[ODMOE_MAX_TOPK];
  extern __shared__ __attribute__((aligned(16))) unsigned char glue_lds[];
  const int t = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  const T* xt = x + (size_t)t * H;
  if constexpr (GLUE) {
    __shared__ float part[16];
    T* sx = reinterpret_cast<T*>(glue_lds);
    glue_block<T>(gl.x_prev, gl.y_prev, H, part, [&](int i, T v) { sx[i] = v; gl.x_out[i] = v; });
    __syncthreads();
    xt = sx;
  }
  const int nvec = H / DT<T>::VEC;
  for (int e = wave; e < E; e += nw) {
    const double acc = wave_logit<T>(Wg + (size_t)e * H, xt, nvec, lane);
    if (lane == 0) slog[e] = (float)(acc + (bias ? (double)bias[e] : 0.0));
  }
  __syncthreads();
  select_topk_and_gate(slog, sel_v, sel_i, E, k, t, idx, gate, idx_mirror, table, table_off, eptr_out);
}

// Few tokens, many experts: gridDim.x blocks per token, each taking 8 experts (one per wave), so
// the router matrix is read by many CUs at once.  The logits go to `logits` [T, E]; the block
// that finishes last for its token (a ticket from counters[t], which it leaves at zero again)
// does the selection.  No block waits for another.
template <typename T, bool GLUE>
__global__ __launch_bounds__(512) void route_topk_split_kernel(
    const T* __restrict__ Wg, const float* __restrict__ bias, const T* __restrict__ x, int H, int E, int k,
    int32_t* __restrict__ idx, float* __restrict__ gate, int32_t* __restrict__ idx_mirror,
    const void* const* __restrict__ table, int table_off, const void** __restrict__ eptr_out,
    float* logits, int32_t* counters, GlueIn<T> gl) {
  __shared__ float slog[ODMOE_MAX_EXPERTS];
  __shared__ float sel_v[ODMOE_MAX_TOPK];
  __shared__ int sel_i[ODMOE_MAX_TOPK];
  __shared__ int s_ticket;
  extern __shared__ __attribute__((aligned(16))) unsigned char glue_lds[];
  const int t = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int e = blockIdx.x * 8 + wave;
  const T* xt = x + (size_t)t * H;
  if constexpr (GLUE) {   // every block makes the router's input for itself; block 0 also publishes it
    __shared__ float part[16];
    T* sx = reinterpret_cast<T*>(glue_lds);
    const bool publish = blockIdx.x == 0;
    glue_block<T>(gl.x_prev, gl.y_prev, H, part, [&](int i, T v) { sx[i] = v; if (publish) gl.x_out[i] = v; });
    __syncthreads();
    xt = sx;
  }
  if (e < E) {
    const double acc = wave_logit<T>(Wg + (size_t)e * H, xt, H / DT<T>::VEC, lane);
    if (lane == 0)
      __hip_atomic_store(logits + (size_t)t * E + e, (float)(acc + (bias ? (double)bias[e] : 0.0)),
                         __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  __threadfence();       // this block's logits are visible device-wide before its ticket is
  __syncthreads();
  if (threadIdx.x == 0)
    s_ticket = __hip_atomic_fetch_add(counters + t, 1, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
  __syncthreads();
  if (s_ticket != (int)gridDim.x - 1) return;
  __threadfence();
  for (int j = threadIdx.x; j < E; j += blockDim.x)
    slog[j] = __hip_atomic_load(logits + (size_t)t * E + j, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (threadIdx.x == 0) counters[t] = 0;
  __syncthreads();
  select_topk_and_gate(slog, sel_v, sel_i, E, k, t, idx, gate, idx_mirror, table, table_off, eptr_out);
}

// ---------------------------------------------------------------------------------------------
// h[i, j] = silu(W1_i[j,:] . x) * (W3_i[j,:] . x)  for the k selected experts of one token.
// One wave per (expert rank, ffn row) pair; RPW consecutive pairs per wave.
// ---------------------------------------------------------------------------------------------
template <typename T, int RPW>
__global__ __launch_bounds__(256) void ffn_up_kernel(ExpertSrc src, const int32_t* __restrict__ idx,
                                                      const T* __restrict__ x,
                                                      float* __restrict__ hbuf, int H, int F, int k) {
  constexpr int VEC = DT<T>::VEC;
  extern __shared__ float svec[];
  stage_vec<T, VEC>(x, svec, H);
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  const int nvec = H / VEC;
  const long total = (long)k * F;
  const long r0 = ((long)blockIdx.x * nw + wave) * RPW;
#pragma unroll 1
  for (int rr = 0; rr < RPW; ++rr) {
    const long r = r0 + rr;
    if (r >= total) break;
    const int i = (int)(r / F), j = (int)(r % F);
    const T* base = static_cast<const T*>(expert_ptr(src, idx, i));
    const T* w1 = base + (size_t)j * H;
    const T* w3 = base + (size_t)F * H + (size_t)j * H;
    float a, b;
    wave_dot2<T>(w1, w3, svec, nvec, lane, a, b);
    if (lane == 0) hbuf[r] = a / (1.f + expf(-a)) * b;
  }
}

// ---------------------------------------------------------------------------------------------
// y[r] = sum_i gate[i] * (W2_i[r,:] . h_i)   -- w2 GEMV with the weighted combine fused, no
// atomics: the block that owns output row r walks the k experts in order.
// ---------------------------------------------------------------------------------------------
template <typename T, int RPW>
__global__ __launch_bounds__(512) void ffn_down_kernel(ExpertSrc src, const int32_t* __restrict__ idx,
                                                        const float* __restrict__ gate,
                                                        const float* __restrict__ hbuf,
                                                        T* __restrict__ y, int H, int F, int k) {
  constexpr int VEC = DT<T>::VEC;
  extern __shared__ float svec[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  const int nvec = F / VEC;
  const int r0 = (blockIdx.x * nw + wave) * RPW;
  float acc[RPW];
#pragma unroll
  for (int rr = 0; rr < RPW; ++rr) acc[rr] = 0.f;
  for (int i = 0; i < k; ++i) {
    bool ok;
    const T* w2 = static_cast<const T*>(expert_ptr(src, idx, i, &ok)) + (size_t)2 * F * H;
    __syncthreads();
    stage_vec<float, VEC>(hbuf + (size_t)i * F, svec, F);
    __syncthreads();
    const float g = ok ? gate[i] : 0.f;   // an idx entry that is no expert id adds nothing
#pragma unroll
    for (int rr = 0; rr < RPW; ++rr) {
      const int r = r0 + rr;
      if (r < H) {
        float d = wave_dot<T>(w2 + (size_t)r * F, svec, nvec, lane);
        acc[rr] = fmaf(g, d, acc[rr]);
      }
    }
  }
  if (lane == 0) {
#pragma unroll
    for (int rr = 0; rr < RPW; ++rr)
      if (r0 + rr < H) y[r0 + rr] = DT<T>::from_f32(acc[rr]);
  }
}

// ---------------------------------------------------------------------------------------------
// Inter-layer glue: out = (x + y) / sqrt(mean((x + y)^2) + 1e-6).  One block.
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(1024) void glue_kernel(const T* x, const T* y, T* out, int H) {
  __shared__ float part[16];
  glue_block<T>(x, y, H, part, [&](int i, T v) { out[i] = v; });
}

// =============================================================================================
// Register-resident GEMV kernels (the fast path).  The input vector slice a lane multiplies
// with lives in VGPRs, so the inner loop is nothing but 128-bit streaming loads and FMAs.
// A partially filled last chunk is handled by zeroing the vector registers of the lanes past
// the end and clamping their load address (their products are exactly zero).
// =============================================================================================

// Unpack one 128-bit group of the stored vector into fp32 registers.
template <typename T>
__device__ __forceinline__ void load_vec_regs(const T* __restrict__ vec, int v, int nvec, float* out) {
  constexpr int VEC = DT<T>::VEC;
  if (v < nvec) {
    DT<T>::unpack(load16(vec + (size_t)v * VEC), out);
  } else {
#pragma unroll
    for (int j = 0; j < VEC; ++j) out[j] = 0.f;
  }
}
// Same for an fp32 source vector feeding VEC-wide weight groups (the h vector of the w2 GEMV).
template <int VEC>
__device__ __forceinline__ void load_f32_regs(const float* __restrict__ vec, int v, int nvec, float* out) {
  if (v < nvec) {
#pragma unroll
    for (int q = 0; q < VEC / 4; ++q) {
      f32x4 a = *reinterpret_cast<const f32x4*>(vec + (size_t)v * VEC + 4 * q);
      out[4 * q] = a.x; out[4 * q + 1] = a.y; out[4 * q + 2] = a.z; out[4 * q + 3] = a.w;
    }
  } else {
#pragma unroll
    for (int j = 0; j < VEC; ++j) out[j] = 0.f;
  }
}

template <typename T>
__device__ __forceinline__ float dot_group(u32x4 q, const float* v, float acc) {
  constexpr int VEC = DT<T>::VEC;
  float f[VEC];
  DT<T>::unpack(q, f);
#pragma unroll
  for (int j = 0; j < VEC; ++j) acc = fmaf(f[j], v[j], acc);
  return acc;
}

// bf16 weights against the bf16 input vector kept packed, as it is stored: one v_dot2c_f32_bf16
// per two elements (products exact, sum in fp32) instead of two unpacks and two FMAs.  The pairs
// are cut out of the whole 128-bit value with vector shuffles: bit-casting the 32-bit members
// (q.x, q.y, ...) one by one made hipcc 7.2 multiply the first pair four times.
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
__device__ __forceinline__ float dot_group_packed(u32x4 q, u32x4 xq, float acc) {
  const bf16x8_t w = __builtin_bit_cast(bf16x8_t, q), xv = __builtin_bit_cast(bf16x8_t, xq);
#define ODMOE_DOT2(A, B)                                                                         \
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(w, w, A, B),                     \
                                        __builtin_shufflevector(xv, xv, A, B), acc, false)
  ODMOE_DOT2(0, 1);
  ODMOE_DOT2(2, 3);
  ODMOE_DOT2(4, 5);
  ODMOE_DOT2(6, 7);
#undef ODMOE_DOT2
  return acc;
}

// h[i, j] = silu(W1_i[j,:] . x) * (W3_i[j,:] . x).  x in registers (NCH chunks of 64*VEC
// elements); every wave owns `rpw` consecutive (expert rank, row) pairs, i.e. one long
// contiguous run of W1 and one of W3.  FULL: H is exactly NCH chunks (constant load offsets).
template <typename T, int NCH, bool FULL>
__global__ __launch_bounds__(256) void ffn_up_reg_kernel(ExpertSrc src, const int32_t* __restrict__ idx,
                                                          const T* __restrict__ x,
                                                          float* __restrict__ hbuf, int H, int F, int k,
                                                          int rpw) {
  constexpr int VEC = DT<T>::VEC;
  constexpr int CHUNK = WAVE * VEC;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  const int nvec = H / VEC;
  constexpr bool PACKED = sizeof(T) == 2;   // bf16: x stays packed for the dot2 instruction
  float xr[PACKED ? 1 : NCH][VEC];
  u32x4 xq[PACKED ? NCH : 1];
  int off[NCH];  // element offset of this lane's group in chunk c (clamped into the row)
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int v = c * WAVE + lane;
    if constexpr (PACKED) xq[c] = v < nvec ? load16(x + (size_t)v * VEC) : u32x4{0u, 0u, 0u, 0u};
    else load_vec_regs<T>(x, v, nvec, xr[c]);
    off[c] = FULL ? c * CHUNK + lane * VEC : (v < nvec ? v : nvec - 1) * VEC;
  }
  const int total = k * F;
  const int r_begin = (blockIdx.x * nw + wave) * rpw;
  const int r_end = (r_begin + rpw < total) ? r_begin + rpw : total;
  int r = r_begin;
  while (r < r_end) {
    const int i = r / F;
    const int j0 = r - i * F;
    const int seg_end = ((i + 1) * F < r_end) ? (i + 1) * F : r_end;
    const int nrow = seg_end - r;
    const T* base = static_cast<const T*>(expert_ptr(src, idx, i));
    float* hout = hbuf + (size_t)i * F + j0;
    // Two row pairs alternate between two register sets: the loads of the next pair are on their
    // way while the current one is multiplied and reduced, so the wave (one per SIMD) always has
    // loads in flight.
    auto issue = [&](int rr, u32x4 (&qa)[NCH], u32x4 (&qb)[NCH]) {
      const T* w1 = base + (size_t)(j0 + rr) * H;
      const T* w3 = w1 + (size_t)F * H;
#pragma unroll
      for (int c = 0; c < NCH; ++c) {
        if constexpr (FULL) {
          qa[c] = load16_stream(w1 + lane * VEC + c * CHUNK);
          qb[c] = load16_stream(w3 + lane * VEC + c * CHUNK);
        } else {
          qa[c] = load16_stream(w1 + off[c]);
          qb[c] = load16_stream(w3 + off[c]);
        }
      }
    };
    auto finish = [&](int rr, const u32x4 (&qa)[NCH], const u32x4 (&qb)[NCH]) {
      float a = 0.f, b = 0.f;
#pragma unroll
      for (int c = 0; c < NCH; ++c) {
        if constexpr (PACKED) {
          a = dot_group_packed(qa[c], xq[c], a);
          b = dot_group_packed(qb[c], xq[c], b);
        } else {
          a = dot_group<T>(qa[c], xr[c], a);
          b = dot_group<T>(qb[c], xr[c], b);
        }
      }
      a = wave_sum(a);
      b = wave_sum(b);
      if (lane == 0) hout[rr] = a / (1.f + expf(-a)) * b;
    };
    u32x4 qa0[NCH], qb0[NCH], qa1[NCH], qb1[NCH];
    int rr = 0;
    issue(0, qa0, qb0);
#pragma unroll 1
    for (; rr + 2 <= nrow; rr += 2) {
      issue(rr + 1, qa1, qb1);
      finish(rr, qa0, qb0);
      if (rr + 2 < nrow) issue(rr + 2, qa0, qb0);
      finish(rr + 1, qa1, qb1);
    }
    if (rr < nrow) finish(rr, qa0, qb0);
    r = seg_end;
  }
}

// y[r] = sum_i gate[i] * (W2_i[r,:] . h_i).  The block owns `rpb` output rows.  Its waves form
// a grid of nwc column slices x n_eg expert groups: a wave owns CPW consecutive column chunks of
// the experts of its group and keeps that slice of h_i in registers; two rows are in flight per
// wave.  Per-wave partial sums meet in LDS and are added in wave order: no atomics, fixed order.
template <typename T, int CPW>
__global__ __launch_bounds__(CPW <= 4 ? 1024 : 512) void ffn_down_reg_kernel(ExpertSrc src, const int32_t* __restrict__ idx,
                                                             const float* __restrict__ gate,
                                                             const float* __restrict__ hbuf,
                                                             T* __restrict__ y, int H, int F, int k,
                                                             int rpb, int nwc) {
  constexpr int VEC = DT<T>::VEC;
  constexpr int RIF = 2;  // rows in flight
  extern __shared__ float part[];  // [nw][rpb]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  const int cw = wave % nwc;   // which column slice this wave owns
  const int eg = wave / nwc;   // which expert group (experts eg, eg + n_eg, ...)
  const int n_eg = nw / nwc;
  const int nvec = F / VEC;
  const int r0 = blockIdx.x * rpb;
  float* mypart = part + wave * rpb;
  if (lane == 0)
    for (int t = 0; t < rpb; ++t) mypart[t] = 0.f;
  int off[CPW];
#pragma unroll
  for (int c = 0; c < CPW; ++c) {
    const int v = (cw * CPW + c) * WAVE + lane;
    off[c] = (v < nvec ? v : nvec - 1) * VEC;
  }
  for (int i = eg; i < k; i += n_eg) {
    bool ok;
    const T* w2 = static_cast<const T*>(expert_ptr(src, idx, i, &ok)) + (size_t)2 * F * H;
    const float g = ok ? gate[i] : 0.f;   // an idx entry that is no expert id adds nothing
    const float* hv = hbuf + (size_t)i * F;
    float hr[CPW][VEC];
#pragma unroll
    for (int c = 0; c < CPW; ++c) load_f32_regs<VEC>(hv, (cw * CPW + c) * WAVE + lane, nvec, hr[c]);
#pragma unroll 1
    for (int rr = 0; rr < rpb; rr += RIF) {
      u32x4 q[RIF][CPW];
#pragma unroll
      for (int u = 0; u < RIF; ++u) {
        int row = r0 + rr + u;
        row = row < H ? row : H - 1;
        const T* p = w2 + (size_t)row * F;
#pragma unroll
        for (int c = 0; c < CPW; ++c) q[u][c] = load16_stream(p + off[c]);
      }
#pragma unroll
      for (int u = 0; u < RIF; ++u) {
        float d = 0.f;
#pragma unroll
        for (int c = 0; c < CPW; ++c) d = dot_group<T>(q[u][c], hr[c], d);
        d = wave_sum(d);
        if (lane == 0 && rr + u < rpb) mypart[rr + u] = fmaf(g, d, mypart[rr + u]);
      }
    }
  }
  __syncthreads();
  for (int t = threadIdx.x; t < rpb; t += blockDim.x) {
    if (r0 + t < H) {
      float sum = 0.f;
      for (int w = 0; w < nw; ++w) sum += part[w * rpb + t];
      y[r0 + t] = DT<T>::from_f32(sum);
    }
  }
}

inline size_t lds_vec_bytes(int n, int vec) {
  const int chunk = WAVE * vec;
  return (size_t)((n + chunk - 1) / chunk) * chunk * sizeof(float);
}

constexpr int UP_RPW = 4;
constexpr int DOWN_RPW = 2;
constexpr int UP_THREADS = 256;
constexpr int DOWN_THREADS = 512;
constexpr size_t MAX_LDS = 160 * 1024;

}  // namespace

#ifdef ODMOE_TUNING
int g_tune_up_rpw = 0, g_tune_down_rpb = 0, g_tune_down_eg = 0, g_tune_route_split_e = 0, g_tune_q8_rif = 0;
namespace {
int env_int(const char* name) {
  const char* v = getenv(name);
  const int n = v ? atoi(v) : 0;
  return n > 0 ? n : 0;
}
}  // namespace
#endif

int num_cu() {
  static int n_cached = 0;
  if (n_cached == 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
      n_cached = n;
    else
      n_cached = 256;
  }
  return n_cached;
}

hipError_t kernels_init() {
#ifdef ODMOE_TUNING
  g_tune_up_rpw = env_int("ODMOE_TUNE_UP_RPW");
  g_tune_route_split_e = env_int("ODMOE_TUNE_ROUTE_SPLIT_E");
  g_tune_down_rpb = env_int("ODMOE_TUNE_DOWN_RPB");
  g_tune_down_eg = env_int("ODMOE_TUNE_DOWN_EG");
  g_tune_q8_rif = env_int("ODMOE_TUNE_Q8_RIF");
#endif
  hipError_t e;
  const int big = (int)MAX_LDS;
#define ODMOE_SET_LDS(fn)                                                                    \
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(fn),                                 \
                          hipFuncAttributeMaxDynamicSharedMemorySize, big);                  \
  if (e != hipSuccess) return e;
  ODMOE_SET_LDS((ffn_up_kernel<float, UP_RPW>));
  ODMOE_SET_LDS((ffn_up_kernel<bf16_t, UP_RPW>));
  ODMOE_SET_LDS((ffn_down_kernel<float, DOWN_RPW>));
  ODMOE_SET_LDS((ffn_down_kernel<bf16_t, DOWN_RPW>));
#undef ODMOE_SET_LDS
  return hipSuccess;
}

namespace {
template <typename T, bool GLUE>
hipError_t launch_route_t(hipStream_t s, const Shape& sh, const void* Wg, const float* b, const void* x,
                          int32_t T_tokens, int32_t* idx, float* gate, int32_t* idx_mirror,
                          const void* const* table, int32_t table_off, const void** eptr_out,
                          const RouteScratch* scratch, GlueIn<T> gl) {
  const size_t lds = GLUE ? (size_t)sh.H * sizeof(T) : 0;
  // (up to 16 experts, two rounds of one block cost less than the tickets of the spread variant:
  // 4.3-6.8 us against 6.7-8.1 us; at 32 experts one block takes 18-22 us, the spread variant 9-10)
  const int split_from = g_tune_route_split_e > 0 ? g_tune_route_split_e : 17;
  if (scratch && scratch->logits && sh.E >= split_from && T_tokens <= scratch->max_tokens) {
    const dim3 grid((sh.E + 7) / 8, T_tokens);
    route_topk_split_kernel<T, GLUE><<<grid, 512, lds, s>>>(static_cast<const T*>(Wg), b, static_cast<const T*>(x),
                                                            sh.H, sh.E, sh.k, idx, gate, idx_mirror, table,
                                                            table_off, eptr_out, scratch->logits,
                                                            scratch->counters, gl);
    return hipGetLastError();
  }
  // one wave per expert up to 8 waves
  const int threads = sh.E >= 8 ? 512 : (sh.E >= 4 ? 256 : 128);
  route_topk_kernel<T, GLUE><<<T_tokens, threads, lds, s>>>(static_cast<const T*>(Wg), b, static_cast<const T*>(x),
                                                            sh.H, sh.E, sh.k, idx, gate, idx_mirror, table,
                                                            table_off, eptr_out, gl);
  return hipGetLastError();
}
}  // namespace

bool route_glue_fusable(const Shape& sh) {
  return (size_t)sh.H * (sh.dtype == ODMOE_F32 ? 4 : 2) <= 32 * 1024;   // the router's input in LDS
}

hipError_t launch_route_topk(hipStream_t s, const Shape& sh, const void* Wg, const float* b,
                             const void* x, int32_t T, int32_t* idx, float* gate,
                             int32_t* idx_mirror, const void* const* table, int32_t table_off,
                             const void** eptr_out, const RouteScratch* scratch, const void* glue_x_prev,
                             const void* glue_y_prev, void* glue_x_out) {
  if (T <= 0) return hipSuccess;
  if (glue_x_prev) {
    if (T != 1 || !glue_y_prev || !glue_x_out || !route_glue_fusable(sh)) return hipErrorInvalidValue;
    if (sh.dtype == ODMOE_F32)
      return launch_route_t<float, true>(s, sh, Wg, b, nullptr, 1, idx, gate, idx_mirror, table, table_off, eptr_out,
                                         scratch, GlueIn<float>{static_cast<const float*>(glue_x_prev),
                                                                static_cast<const float*>(glue_y_prev),
                                                                static_cast<float*>(glue_x_out)});
    return launch_route_t<bf16_t, true>(s, sh, Wg, b, nullptr, 1, idx, gate, idx_mirror, table, table_off, eptr_out,
                                        scratch, GlueIn<bf16_t>{static_cast<const bf16_t*>(glue_x_prev),
                                                                static_cast<const bf16_t*>(glue_y_prev),
                                                                static_cast<bf16_t*>(glue_x_out)});
  }
  if (sh.dtype == ODMOE_F32)
    return launch_route_t<float, false>(s, sh, Wg, b, x, T, idx, gate, idx_mirror, table, table_off, eptr_out,
                                        scratch, GlueIn<float>{nullptr, nullptr, nullptr});
  return launch_route_t<bf16_t, false>(s, sh, Wg, b, x, T, idx, gate, idx_mirror, table, table_off, eptr_out,
                                       scratch, GlueIn<bf16_t>{nullptr, nullptr, nullptr});
}

namespace {


template <typename T, int NCH>
hipError_t launch_up_reg_n(hipStream_t s, const Shape& sh, const ExpertSrc& src, const int32_t* idx,
                           const void* x, float* hbuf) {
  const int nw = 4;
  const long total = (long)sh.k * sh.F;
  // one block per CU when the rows allow it: every wave streams one long contiguous run
  long rpw = (total + (long)num_cu() * nw - 1) / ((long)num_cu() * nw);
  // Four times as many waves (16 per CU) where one wave per SIMD does not keep enough loads in
  // flight: small layers (latency bound), rows of fewer than 8 chunks (a wave has 2*NCH loads of
  // 1 KB in flight), and rows of more than 8 chunks whose vector still fits 64 registers (fp32: a
  // wave cannot hold a whole W1/W3 row pair in flight, and its register count still allows four
  // waves per SIMD).
  constexpr bool more_waves = NCH < 8 || (NCH > 8 && NCH * DT<T>::VEC <= 64);
  if (rpw < 16 || more_waves) rpw = (total + (long)num_cu() * nw * 4 - 1) / ((long)num_cu() * nw * 4);
  if (sh.host_link) rpw = (total + 127) / 128;  // 32 blocks of 4 waves
  if (rpw < 1) rpw = 1;
  if (g_tune_up_rpw > 0) rpw = g_tune_up_rpw;
  const int grid = (int)((total + nw * rpw - 1) / (nw * rpw));
  if (sh.H == NCH * WAVE * DT<T>::VEC)
    ffn_up_reg_kernel<T, NCH, true><<<grid, nw * WAVE, 0, s>>>(src, idx, static_cast<const T*>(x), hbuf,
                                                                sh.H, sh.F, sh.k, (int)rpw);
  else
    ffn_up_reg_kernel<T, NCH, false><<<grid, nw * WAVE, 0, s>>>(src, idx, static_cast<const T*>(x), hbuf,
                                                                 sh.H, sh.F, sh.k, (int)rpw);
  return hipGetLastError();
}

template <typename T>
hipError_t launch_up_reg(hipStream_t s, const Shape& sh, const ExpertSrc& src, const int32_t* idx,
                         const void* x, float* hbuf, int nch) {
  switch (nch) {
#define ODMOE_CASE(N) case N: return launch_up_reg_n<T, N>(s, sh, src, idx, x, hbuf);
    ODMOE_CASE(1) ODMOE_CASE(2) ODMOE_CASE(3) ODMOE_CASE(4) ODMOE_CASE(5) ODMOE_CASE(6)
    ODMOE_CASE(7) ODMOE_CASE(8) ODMOE_CASE(9) ODMOE_CASE(10) ODMOE_CASE(11) ODMOE_CASE(12)
    ODMOE_CASE(13) ODMOE_CASE(14) ODMOE_CASE(15) ODMOE_CASE(16)
#undef ODMOE_CASE
  }
  return hipErrorInvalidValue;
}

template <typename T, int CPW>
hipError_t launch_down_reg_n(hipStream_t s, const Shape& sh, const ExpertSrc& src, const int32_t* idx,
                             const float* gate, const float* hbuf, void* y, int nwb) {
  int n_eg, rpb;
  down_block_shape(sh, CPW, nwb, g_tune_down_eg, g_tune_down_rpb, &n_eg, &rpb);
  const int grid = (sh.H + rpb - 1) / rpb;
  const int nw = nwb * n_eg;
  const size_t lds = (size_t)nw * rpb * sizeof(float);
  ffn_down_reg_kernel<T, CPW><<<grid, nw * WAVE, lds, s>>>(src, idx, gate, hbuf, static_cast<T*>(y),
                                                           sh.H, sh.F, sh.k, rpb, nwb);
  return hipGetLastError();
}

template <typename T>
hipError_t launch_down_reg(hipStream_t s, const Shape& sh, const ExpertSrc& src, const int32_t* idx,
                           const float* gate, const float* hbuf, void* y, int cpw, int nwb) {
  switch (cpw) {
#define ODMOE_CASE(N) case N: return launch_down_reg_n<T, N>(s, sh, src, idx, gate, hbuf, y, nwb);
    ODMOE_CASE(1) ODMOE_CASE(2) ODMOE_CASE(3) ODMOE_CASE(4) ODMOE_CASE(5) ODMOE_CASE(6)
    ODMOE_CASE(7) ODMOE_CASE(8)
#undef ODMOE_CASE
  }
  return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_ffn_up(hipStream_t s, const Shape& sh, const ExpertSrc& src, const int32_t* idx,
                         const void* x, float* hbuf) {
  if (sh.quant == ODMOE_Q_INT8_ROW) return launch_ffn_up_q8(s, sh, src, idx, x, hbuf);
  if (sh.quant == ODMOE_Q_INT4_G64) return launch_ffn_up_q4(s, sh, src, idx, x, hbuf);
  if (sh.quant == ODMOE_Q_F16) return launch_ffn_up_f16(s, sh, src, idx, x, hbuf);
  const int vec = sh.dtype == ODMOE_F32 ? 4 : 8;
  const int nch = (sh.H + WAVE * vec - 1) / (WAVE * vec);
  if (nch <= 16) {
    return sh.dtype == ODMOE_F32 ? launch_up_reg<float>(s, sh, src, idx, x, hbuf, nch)
                                 : launch_up_reg<bf16_t>(s, sh, src, idx, x, hbuf, nch);
  }
  // generic fallback: x staged in LDS
  const int nw = UP_THREADS / WAVE;
  const long total = (long)sh.k * sh.F;
  const int grid = (int)((total + nw * UP_RPW - 1) / (nw * UP_RPW));
  const size_t lds = lds_vec_bytes(sh.H, vec);
  if (lds > MAX_LDS) return hipErrorInvalidValue;
  if (sh.dtype == ODMOE_F32)
    ffn_up_kernel<float, UP_RPW><<<grid, UP_THREADS, lds, s>>>(src, idx, static_cast<const float*>(x),
                                                               hbuf, sh.H, sh.F, sh.k);
  else
    ffn_up_kernel<bf16_t, UP_RPW><<<grid, UP_THREADS, lds, s>>>(src, idx, static_cast<const bf16_t*>(x),
                                                                hbuf, sh.H, sh.F, sh.k);
  return hipGetLastError();
}

hipError_t launch_ffn_down(hipStream_t s, const Shape& sh, const ExpertSrc& src,
                           const int32_t* idx, const float* gate, const float* hbuf, void* y) {
  if (sh.quant == ODMOE_Q_INT8_ROW) return launch_ffn_down_q8(s, sh, src, idx, gate, hbuf, y);
  if (sh.quant == ODMOE_Q_INT4_G64) return launch_ffn_down_q4(s, sh, src, idx, gate, hbuf, y);
  if (sh.quant == ODMOE_Q_F16) return launch_ffn_down_f16(s, sh, src, idx, gate, hbuf, y);
  const int vec = sh.dtype == ODMOE_F32 ? 4 : 8;
  const int nc = (sh.F + WAVE * vec - 1) / (WAVE * vec);
  int cpw = 0, nwb = 0;
  if (pick_down_split(nc, &cpw, &nwb)) {
    return sh.dtype == ODMOE_F32 ? launch_down_reg<float>(s, sh, src, idx, gate, hbuf, y, cpw, nwb)
                                 : launch_down_reg<bf16_t>(s, sh, src, idx, gate, hbuf, y, cpw, nwb);
  }
  // generic fallback: h staged in LDS, one expert at a time
  const int nw = DOWN_THREADS / WAVE;
  const int grid = (sh.H + nw * DOWN_RPW - 1) / (nw * DOWN_RPW);
  const size_t lds = lds_vec_bytes(sh.F, vec);
  if (lds > MAX_LDS) return hipErrorInvalidValue;
  if (sh.dtype == ODMOE_F32)
    ffn_down_kernel<float, DOWN_RPW><<<grid, DOWN_THREADS, lds, s>>>(
        src, idx, gate, hbuf, static_cast<float*>(y), sh.H, sh.F, sh.k);
  else
    ffn_down_kernel<bf16_t, DOWN_RPW><<<grid, DOWN_THREADS, lds, s>>>(
        src, idx, gate, hbuf, static_cast<bf16_t*>(y), sh.H, sh.F, sh.k);
  return hipGetLastError();
}

// Plain streaming kernels over a buffer of known size: the measured HBM ceiling next to the
// GEMVs, and the reference a profiler's byte counters are scaled by.  128-bit loads; the read
// kernel gives every wave one contiguous span, the copy kernel every block.
namespace {
__global__ __launch_bounds__(256) void probe_read_kernel(const u32x4* __restrict__ src, size_t n16,
                                                          uint32_t* __restrict__ sink) {
  // The assignment the w1/w3 GEMV uses, which is also the fastest plain read found: one block of
  // four waves per CU, every wave one long contiguous run, sixteen 1 KB loads in flight per wave.
  const int lane = threadIdx.x & 63;
  const size_t nw = (size_t)gridDim.x * 4, w = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const size_t per = (n16 + nw - 1) / nw;
  const size_t b0 = w * per, b1 = b0 + per < n16 ? b0 + per : n16;
  uint32_t acc = 0;
  size_t i = b0 + lane;
  for (; i + 15 * 64 < b1; i += 16 * 64) {
    u32x4 q[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) q[u] = __builtin_nontemporal_load(src + i + u * 64);
#pragma unroll
    for (int u = 0; u < 16; ++u) acc ^= q[u].x ^ q[u].y ^ q[u].z ^ q[u].w;
  }
  for (; i < b1; i += 64) { const u32x4 q = src[i]; acc ^= q.x ^ q.y ^ q.z ^ q.w; }
  if (acc == 0x9e3779b9u) sink[0] = acc;  // practically never: keeps the loads alive
}
__global__ __launch_bounds__(256) void probe_copy_kernel(const u32x4* __restrict__ src,
                                                          u32x4* __restrict__ dst, size_t n16) {
  const size_t per = (n16 + gridDim.x - 1) / gridDim.x;
  const size_t b0 = (size_t)blockIdx.x * per, b1 = b0 + per < n16 ? b0 + per : n16;
  for (size_t i = b0 + threadIdx.x; i < b1; i += 256) dst[i] = src[i];
}
}  // namespace

hipError_t launch_probe(hipStream_t s, void* dst, const void* src, size_t bytes, int mode) {
  const size_t n16 = bytes / 16;
  if (n16 == 0) return hipSuccess;
  const int grid = num_cu() * 8;
  if (mode == 1)
    probe_read_kernel<<<num_cu(), 256, 0, s>>>(static_cast<const u32x4*>(src), n16, static_cast<uint32_t*>(dst));
  else
    probe_copy_kernel<<<grid, 256, 0, s>>>(static_cast<const u32x4*>(src), static_cast<u32x4*>(dst), n16);
  return hipGetLastError();
}

hipError_t launch_glue(hipStream_t s, const Shape& sh, const void* x, const void* y, void* x_next) {
  if (sh.dtype == ODMOE_F32)
    glue_kernel<float><<<1, 1024, 0, s>>>(static_cast<const float*>(x), static_cast<const float*>(y),
                                          static_cast<float*>(x_next), sh.H);
  else
    glue_kernel<bf16_t><<<1, 1024, 0, s>>>(static_cast<const bf16_t*>(x),
                                           static_cast<const bf16_t*>(y),
                                           static_cast<bf16_t*>(x_next), sh.H);
  return hipGetLastError();
}

}  // namespace odmoe
