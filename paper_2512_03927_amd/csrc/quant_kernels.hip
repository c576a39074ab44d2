// The quantised shadow model's side of the path (paper Sections 1 and 3.2: the expert-activation
// predictor is a quantised copy of the model that runs ahead of the full-precision one because
// it is cheaper to run).  Two things live here:
//
//   quantiser   symmetric absmax quantisation of a weight matrix on the device: int8 per row
//               (127 levels each side) or 4 bits per group of 64 consecutive elements of a row
//               (7 levels each side), round half to even, decided in float64 so that every code
//               equals the one a float64 CPU computation gives;
//   int8 GEMVs  the two expert GEMVs of the decode path over int8 codes with one fp32 scale per
//               weight row: half the bytes of bf16 per token.  Still bound by the weight stream,
//               so still no matrix cores: codes are dequantised in registers (one conversion and
//               one FMA per weight) and accumulated in fp32.
//
// The paper does not print its quantisers (it names FP16 / INT8 / NF4); these are the plain
// absmax schemes.  Codes are stored offset-binary, code = q + 128 (q + 8 for 4 bits, one per
// byte), so that a byte converts to fp32 with a single instruction; the offset comes out of the
// dot product as  sum_j (q_j + 128) x_j - 128 sum_j x_j.
#include "gemv_common.hpp"

namespace odmoe {
namespace {

// ---------------------------------------------------------------------------------------------
// Quantiser
// ---------------------------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ double elem_f64(const T* w, size_t i) {
  return (double)DT<T>::to_f32(w[i]);
}

// float64 -> stored dtype with ONE rounding to nearest even (going through fp32 first would round
// twice for bf16).
__device__ __forceinline__ void store_rne(float* dst, size_t i, double v) { dst[i] = (float)v; }
__device__ __forceinline__ void store_rne(bf16_t* dst, size_t i, double v) {
  const uint64_t b = (uint64_t)__double_as_longlong(v);
  const uint32_t sign = (uint32_t)(b >> 63) << 15;
  const int e = (int)((b >> 52) & 0x7ff) - 1023 + 127;       // bf16 / fp32 biased exponent
  if (e <= 0 || e >= 255) {   // zero, below the normal range, infinity: fp32's rounding is exact enough there
    dst[i] = f32_to_bf16((float)v);
    return;
  }
  const uint64_t man = b & ((1ull << 52) - 1);
  const uint32_t keep = (uint32_t)(man >> 45);                // 7 mantissa bits
  const uint64_t rem = man & ((1ull << 45) - 1), half = 1ull << 44;
  const uint32_t up = (rem > half || (rem == half && (keep & 1u))) ? 1u : 0u;
  dst[i] = (bf16_t)(sign | ((((uint32_t)e << 7) | keep) + up));   // a carry moves into the exponent
}

// scale = amax / levels; q = clip(rint(w / scale), -levels, levels); all in float64.  The code is
// an integer: a small negative weight gives 0, not -0.0 (its dequantised value is +0).
__device__ __forceinline__ int quant_code(double w, double scale, int levels) {
  if (!(scale > 0.0)) return 0;
  const int q = (int)rint(w / scale);
  return q > levels ? levels : (q < -levels ? -levels : q);
}

// One block per row: absmax over the row, then the codes.
template <typename T>
__global__ __launch_bounds__(256) void quantize_rows_kernel(const T* __restrict__ w, long cols, int levels,
                                                             uint8_t* __restrict__ code,
                                                             float* __restrict__ scale, T* __restrict__ deq) {
  __shared__ float part[4];
  const size_t row0 = (size_t)blockIdx.x * cols;
  float amax = 0.f;                                         // |w| is exact in fp32 for both dtypes
  for (long c = threadIdx.x; c < cols; c += blockDim.x) amax = fmaxf(amax, fabsf(DT<T>::to_f32(w[row0 + c])));
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off, WAVE));
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = amax;
  __syncthreads();
  amax = fmaxf(fmaxf(part[0], part[1]), fmaxf(part[2], part[3]));
  const double s = (double)amax / (double)levels;
  if (threadIdx.x == 0 && scale) scale[blockIdx.x] = (float)s;
  for (long c = threadIdx.x; c < cols; c += blockDim.x) {
    const int q = quant_code(elem_f64(w, row0 + c), s, levels);
    if (code) code[row0 + c] = (uint8_t)(q + levels + 1);
    if (deq) store_rne(deq, row0 + c, (double)q * s);
  }
}

// One wave per group of 64 consecutive elements of a row (cols is a multiple of 64, so groups
// never straddle rows and group g covers elements 64 g .. 64 g + 63 of the flat matrix).
template <typename T>
__global__ __launch_bounds__(256) void quantize_groups64_kernel(const T* __restrict__ w, size_t n_groups,
                                                                 int levels, uint8_t* __restrict__ code,
                                                                 float* __restrict__ scale,
                                                                 T* __restrict__ deq) {
  const size_t g = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (g >= n_groups) return;
  const int lane = threadIdx.x & 63;
  const size_t i = g * 64 + lane;
  const float v = DT<T>::to_f32(w[i]);
  float amax = fabsf(v);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off, WAVE));
  const double s = (double)amax / (double)levels;
  if (lane == 0 && scale) scale[g] = (float)s;
  const int q = quant_code((double)v, s, levels);
  if (code) code[i] = (uint8_t)(q + levels + 1);
  if (deq) store_rne(deq, i, (double)q * s);
}

// ---------------------------------------------------------------------------------------------
// int8 GEMVs.  A 128-bit load brings 16 codes; a chunk is 64 lanes x 16 = 1024 weights.
// ---------------------------------------------------------------------------------------------
constexpr int QV = 16;            // codes per 128-bit load
constexpr int QCHUNK = WAVE * QV;

// acc + sum_j code_j * v_j over the 16 codes of q (each byte -> fp32 is one conversion instruction)
__device__ __forceinline__ float dot_codes(u32x4 q, const float* v, float acc) {
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    const uint32_t w = q[d];
    acc = fmaf((float)(w & 0xffu), v[4 * d], acc);
    acc = fmaf((float)((w >> 8) & 0xffu), v[4 * d + 1], acc);
    acc = fmaf((float)((w >> 16) & 0xffu), v[4 * d + 2], acc);
    acc = fmaf((float)(w >> 24), v[4 * d + 3], acc);
  }
  return acc;
}

// The 16 elements of group v of a stored vector as fp32 registers (zeros past the end).
template <typename XT>
__device__ __forceinline__ void load_group16(const XT* __restrict__ vec, int v, int nvec, float* out) {
  if (v < nvec) {
    constexpr int PER = DT<XT>::VEC;   // elements per 128-bit load of the vector's dtype
#pragma unroll
    for (int p = 0; p < QV / PER; ++p) DT<XT>::unpack(load16(vec + (size_t)v * QV + p * PER), out + p * PER);
  } else {
#pragma unroll
    for (int j = 0; j < QV; ++j) out[j] = 0.f;
  }
}

// h[i, j] = silu(s1[j] * (Q1_i[j,:] . x)) * (s3[j] * (Q3_i[j,:] . x)).  Same shape as the
// stored-dtype kernel: x in registers, every wave streams one contiguous run of rows of W1 and of
// W3 through two register sets.  Expert buffer: codes W1[F,H] | W3[F,H] | W2[H,F], then fp32
// scales s1[F] | s3[F] | s2[H].
template <typename XT, int NCH>
__global__ __launch_bounds__(256) void ffn_up_q8_kernel(ExpertSrc src, const int32_t* __restrict__ idx,
                                                         const XT* __restrict__ x,
                                                         float* __restrict__ hbuf, int H, int F, int k,
                                                         int rpw) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  const int nvec = H / QV;
  float xr[NCH][QV];
  int off[NCH];
  float sx = 0.f;   // sum of this lane's x elements: the offset-binary correction
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int v = c * WAVE + lane;
    load_group16<XT>(x, v, nvec, xr[c]);
    off[c] = (v < nvec ? v : nvec - 1) * QV;
#pragma unroll
    for (int j = 0; j < QV; ++j) sx += xr[c][j];
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
    const uint8_t* base = static_cast<const uint8_t*>(expert_ptr(src, idx, i));
    const float* sc = reinterpret_cast<const float*>(base + (size_t)3 * H * F);
    float* hout = hbuf + (size_t)i * F + j0;
    auto issue = [&](int rr, u32x4 (&qa)[NCH], u32x4 (&qb)[NCH], float& sa, float& sb) {
      const uint8_t* w1 = base + (size_t)(j0 + rr) * H;
      const uint8_t* w3 = w1 + (size_t)F * H;
#pragma unroll
      for (int c = 0; c < NCH; ++c) {
        qa[c] = load16_stream(w1 + off[c]);
        qb[c] = load16_stream(w3 + off[c]);
      }
      sa = sc[j0 + rr];
      sb = sc[F + j0 + rr];
    };
    auto finish = [&](int rr, const u32x4 (&qa)[NCH], const u32x4 (&qb)[NCH], float sa, float sb) {
      float a = 0.f, b = 0.f;
#pragma unroll
      for (int c = 0; c < NCH; ++c) {
        a = dot_codes(qa[c], xr[c], a);
        b = dot_codes(qb[c], xr[c], b);
      }
      a = wave_sum(fmaf(-128.f, sx, a)) * sa;
      b = wave_sum(fmaf(-128.f, sx, b)) * sb;
      if (lane == 0) hout[rr] = a / (1.f + expf(-a)) * b;
    };
    u32x4 qa0[NCH], qb0[NCH], qa1[NCH], qb1[NCH];
    float sa0, sb0, sa1, sb1;
    int rr = 0;
    issue(0, qa0, qb0, sa0, sb0);
#pragma unroll 1
    for (; rr + 2 <= nrow; rr += 2) {
      issue(rr + 1, qa1, qb1, sa1, sb1);
      finish(rr, qa0, qb0, sa0, sb0);
      if (rr + 2 < nrow) issue(rr + 2, qa0, qb0, sa0, sb0);
      finish(rr + 1, qa1, qb1, sa1, sb1);
    }
    if (rr < nrow) finish(rr, qa0, qb0, sa0, sb0);
    r = seg_end;
  }
}

// y[r] = sum_i gate[i] * s2_i[r] * (Q2_i[r,:] . h_i).  Same block shape as the stored-dtype
// kernel: rpb output rows per block, waves = nwc column slices x expert groups, h slice in
// registers, two rows in flight, partial sums meet in LDS in wave order.
template <typename YT, int CPW, int RIF>
__global__ __launch_bounds__(1024) void ffn_down_q8_kernel(ExpertSrc src, const int32_t* __restrict__ idx,
                                                            const float* __restrict__ gate,
                                                            const float* __restrict__ hbuf,
                                                            YT* __restrict__ y, int H, int F, int k, int rpb,
                                                            int nwc) {
  extern __shared__ float part[];  // [nw][rpb]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  const int cw = wave % nwc, eg = wave / nwc, n_eg = nw / nwc;
  const int nvec = F / QV;
  const int r0 = blockIdx.x * rpb;
  float* mypart = part + wave * rpb;
  if (lane == 0)
    for (int t = 0; t < rpb; ++t) mypart[t] = 0.f;
  int off[CPW];
#pragma unroll
  for (int c = 0; c < CPW; ++c) {
    const int v = (cw * CPW + c) * WAVE + lane;
    off[c] = (v < nvec ? v : nvec - 1) * QV;
  }
  for (int i = eg; i < k; i += n_eg) {
    bool ok;
    const uint8_t* base = static_cast<const uint8_t*>(expert_ptr(src, idx, i, &ok));
    const float g = ok ? gate[i] : 0.f;   // an idx entry that is no expert id adds nothing
    const uint8_t* w2 = base + (size_t)2 * F * H;
    const float* s2 = reinterpret_cast<const float*>(base + (size_t)3 * H * F) + 2 * F;
    const float* hv = hbuf + (size_t)i * F;
    float hr[CPW][QV];
    float sh = 0.f;
#pragma unroll
    for (int c = 0; c < CPW; ++c) {
      load_group16<float>(hv, (cw * CPW + c) * WAVE + lane, nvec, hr[c]);
#pragma unroll
      for (int j = 0; j < QV; ++j) sh += hr[c][j];
    }
#pragma unroll 1
    for (int rr = 0; rr < rpb; rr += RIF) {
      u32x4 q[RIF][CPW];
      float sr[RIF];
#pragma unroll
      for (int u = 0; u < RIF; ++u) {
        int row = r0 + rr + u;
        row = row < H ? row : H - 1;
        const uint8_t* p = w2 + (size_t)row * F;
#pragma unroll
        for (int c = 0; c < CPW; ++c) q[u][c] = load16_stream(p + off[c]);
        sr[u] = s2[row];
      }
#pragma unroll
      for (int u = 0; u < RIF; ++u) {
        float d = 0.f;
#pragma unroll
        for (int c = 0; c < CPW; ++c) d = dot_codes(q[u][c], hr[c], d);
        d = wave_sum(fmaf(-128.f, sh, d));
        if (lane == 0 && rr + u < rpb) mypart[rr + u] = fmaf(g * sr[u], d, mypart[rr + u]);
      }
    }
  }
  __syncthreads();
  for (int t = threadIdx.x; t < rpb; t += blockDim.x) {
    if (r0 + t < H) {
      float sum = 0.f;
      for (int w = 0; w < nw; ++w) sum += part[w * rpb + t];
      y[r0 + t] = DT<YT>::from_f32(sum);
    }
  }
}

template <typename XT, int NCH>
hipError_t launch_up_q8_n(hipStream_t s, const Shape& sh, const ExpertSrc& src, const int32_t* idx,
                          const void* x, float* hbuf) {
  const int nw = 4;
  const long total = (long)sh.k * sh.F;
  // Two waves per SIMD (eight per CU): a wave converts and multiplies one row pair while the loads
  // of its next pair are in flight, and the second wave fills the gaps the reductions leave.
  long rpw = (total + (long)num_cu() * nw * 2 - 1) / ((long)num_cu() * nw * 2);
  if (sh.host_link) rpw = (total + 127) / 128;
  if (rpw < 1) rpw = 1;
  if (g_tune_up_rpw > 0) rpw = g_tune_up_rpw;
  const int grid = (int)((total + nw * rpw - 1) / (nw * rpw));
  ffn_up_q8_kernel<XT, NCH><<<grid, nw * WAVE, 0, s>>>(src, idx, static_cast<const XT*>(x), hbuf, sh.H, sh.F,
                                                      sh.k, (int)rpw);
  return hipGetLastError();
}

template <typename XT>
hipError_t launch_up_q8(hipStream_t s, const Shape& sh, const ExpertSrc& src, const int32_t* idx,
                        const void* x, float* hbuf) {
  switch ((sh.H + QCHUNK - 1) / QCHUNK) {
#define ODMOE_CASE(N) case N: return launch_up_q8_n<XT, N>(s, sh, src, idx, x, hbuf);
    ODMOE_CASE(1) ODMOE_CASE(2) ODMOE_CASE(3) ODMOE_CASE(4) ODMOE_CASE(5) ODMOE_CASE(6)
    ODMOE_CASE(7) ODMOE_CASE(8)
#undef ODMOE_CASE
  }
  return hipErrorInvalidValue;
}

template <typename YT, int CPW>
hipError_t launch_down_q8_n(hipStream_t s, const Shape& sh, const ExpertSrc& src, const int32_t* idx,
                            const float* gate, const float* hbuf, void* y, int nwb) {
  int n_eg, rpb;
  down_block_shape(sh, CPW, nwb, g_tune_down_eg, g_tune_down_rpb, &n_eg, &rpb);
  // A row of codes is half as many bytes as a bf16 row: blocks of 5 to 8 column slices take two
  // expert groups (up to 16 waves) and every wave keeps four rows in flight to have as many bytes
  // on their way (Mixtral layer: 30.3 us with one group and two rows, 22.7 us so).
  if (g_tune_down_eg == 0 && nwb > 4 && nwb <= 8 && sh.k >= 2) n_eg = 2;
  rpb = (rpb + 3) & ~3;   // whole groups of rows in flight
  const int grid = (sh.H + rpb - 1) / rpb;
  const int nw = nwb * n_eg;
  const size_t lds = (size_t)nw * rpb * sizeof(float);
  if (g_tune_q8_rif == 2)
    ffn_down_q8_kernel<YT, CPW, 2><<<grid, nw * WAVE, lds, s>>>(src, idx, gate, hbuf, static_cast<YT*>(y), sh.H,
                                                               sh.F, sh.k, rpb, nwb);
  else
    ffn_down_q8_kernel<YT, CPW, 4><<<grid, nw * WAVE, lds, s>>>(src, idx, gate, hbuf, static_cast<YT*>(y), sh.H,
                                                               sh.F, sh.k, rpb, nwb);
  return hipGetLastError();
}

template <typename YT>
hipError_t launch_down_q8(hipStream_t s, const Shape& sh, const ExpertSrc& src, const int32_t* idx,
                          const float* gate, const float* hbuf, void* y) {
  int cpw = 0, nwb = 0;
  if (!pick_down_split((sh.F + QCHUNK - 1) / QCHUNK, &cpw, &nwb) || cpw > 4) return hipErrorInvalidValue;
  switch (cpw) {
#define ODMOE_CASE(N) case N: return launch_down_q8_n<YT, N>(s, sh, src, idx, gate, hbuf, y, nwb);
    ODMOE_CASE(1) ODMOE_CASE(2) ODMOE_CASE(3) ODMOE_CASE(4)
#undef ODMOE_CASE
  }
  return hipErrorInvalidValue;
}

}  // namespace

bool q8_supported(const Shape& sh) {
  int cpw = 0, nwb = 0;
  return sh.H % QV == 0 && sh.F % QV == 0 && sh.H <= 8 * QCHUNK &&
         pick_down_split((sh.F + QCHUNK - 1) / QCHUNK, &cpw, &nwb) && cpw <= 4;
}

hipError_t launch_ffn_up_q8(hipStream_t s, const Shape& sh, const ExpertSrc& src, const int32_t* idx,
                            const void* x, float* hbuf) {
  if (!q8_supported(sh)) return hipErrorInvalidValue;
  return sh.dtype == ODMOE_F32 ? launch_up_q8<float>(s, sh, src, idx, x, hbuf)
                               : launch_up_q8<bf16_t>(s, sh, src, idx, x, hbuf);
}

hipError_t launch_ffn_down_q8(hipStream_t s, const Shape& sh, const ExpertSrc& src, const int32_t* idx,
                              const float* gate, const float* hbuf, void* y) {
  if (!q8_supported(sh)) return hipErrorInvalidValue;
  return sh.dtype == ODMOE_F32 ? launch_down_q8<float>(s, sh, src, idx, gate, hbuf, y)
                               : launch_down_q8<bf16_t>(s, sh, src, idx, gate, hbuf, y);
}

hipError_t launch_quantize(hipStream_t s, const void* w, int32_t dtype, int64_t rows, int64_t cols,
                           int32_t kind, uint8_t* code, float* scale, void* deq) {
  if (rows <= 0 || cols <= 0) return hipSuccess;
  if (kind == ODMOE_Q_INT8_ROW) {
    if (rows > 0x7fffffffLL) return hipErrorInvalidValue;
    if (dtype == ODMOE_F32)
      quantize_rows_kernel<float><<<(unsigned)rows, 256, 0, s>>>(static_cast<const float*>(w), (long)cols, 127, code,
                                                                scale, static_cast<float*>(deq));
    else
      quantize_rows_kernel<bf16_t><<<(unsigned)rows, 256, 0, s>>>(static_cast<const bf16_t*>(w), (long)cols, 127,
                                                                 code, scale, static_cast<bf16_t*>(deq));
    return hipGetLastError();
  }
  if (kind == ODMOE_Q_INT4_G64) {
    if (cols % 64) return hipErrorInvalidValue;
    const size_t n_groups = (size_t)rows * (size_t)(cols / 64);
    const size_t blocks = (n_groups + 3) / 4;
    if (blocks > 0x7fffffffULL) return hipErrorInvalidValue;
    if (dtype == ODMOE_F32)
      quantize_groups64_kernel<float><<<(unsigned)blocks, 256, 0, s>>>(static_cast<const float*>(w), n_groups, 7, code,
                                                                      scale, static_cast<float*>(deq));
    else
      quantize_groups64_kernel<bf16_t><<<(unsigned)blocks, 256, 0, s>>>(static_cast<const bf16_t*>(w), n_groups, 7,
                                                                       code, scale, static_cast<bf16_t*>(deq));
    return hipGetLastError();
  }
  return hipErrorInvalidValue;
}

}  // namespace odmoe
