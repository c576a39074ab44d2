// 4-bit experts of the shadow model (paper Sections 1 and 3.2: the cheapest quantised copy the
// paper runs as its predictor is a 4-bit one).  Symmetric absmax per group of 64 consecutive
// weights of a row, 7 levels each side, codes packed two per byte with one fp32 scale per group:
// 0.28 of the bytes of bf16.  The paper's NF4 code book is not reproduced; the scheme is the
// uniform one of odmoe_quantize (ODMOE_Q_INT4_G64), the codes are the same, only packed.
//
// Expert buffer:  codes W1[F][H/2] | W3[F][H/2] | W2[H][F/2]  (element 2j in the low nibble of
// byte j, offset-binary: nibble = q + 8), then fp32 scales s1[F][H/64] | s3[F][H/64] | s2[H][F/64].
//
// The two GEMVs have the shape of the other expert GEMVs (input slice in registers, every wave
// streams a contiguous run of rows, two register sets in flight).  A 128-bit load brings 32 codes,
// i.e. half a group: one scale per load.  With a quarter of the bytes per weight the conversion
// work (split nibbles, byte -> fp32, FMA: about 2.4 instructions per weight) is what bounds them,
// not the weight stream.
#include "gemv_common.hpp"

namespace odmoe {
namespace {

constexpr int NV = 32;               // codes per 128-bit load
constexpr int NCHUNK = WAVE * NV;    // weights a wave covers per load instruction: 2048
constexpr int GROUP = 64;            // weights per scale

// One wave per group of 64 weights: absmax, scale, codes (all decided in float64, as in
// odmoe_quantize), two codes packed per byte by the even lanes.
template <typename T>
__global__ __launch_bounds__(256) void quantize_pack4_kernel(const T* __restrict__ w, size_t n_groups,
                                                              uint8_t* __restrict__ packed,
                                                              float* __restrict__ scale) {
  const size_t g = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (g >= n_groups) return;
  const int lane = threadIdx.x & 63;
  const size_t i = g * GROUP + lane;
  const float v = DT<T>::to_f32(w[i]);
  float amax = fabsf(v);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off, WAVE));
  const double s = (double)amax / 7.0;
  if (lane == 0) scale[g] = (float)s;
  int q = 0;
  if (s > 0.0) {
    q = (int)rint((double)v / s);
    q = q > 7 ? 7 : (q < -7 ? -7 : q);
  }
  const int code = q + 8;
  const int other = __shfl_xor(code, 1, WAVE);
  if ((lane & 1) == 0) packed[i >> 1] = (uint8_t)(code | (other << 4));
}

// acc + sum_j code_j * v_j over the 32 codes of q.  Byte b of dword d holds elements 8d + 2b (low
// nibble) and 8d + 2b + 1 (high nibble).
__device__ __forceinline__ float dot_nibbles(u32x4 q, const float* v, float acc) {
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    uint32_t lo = q[d] & 0x0f0f0f0fu, hi = (q[d] >> 4) & 0x0f0f0f0fu;
    // Keep the two masked words as they are: left alone, the compiler turns every nibble into its own
    // bit-field extract plus conversion (3 instructions per weight instead of 2.4).
    asm volatile("" : "+v"(lo), "+v"(hi));
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      acc = fmaf((float)((lo >> (8 * b)) & 0xffu), v[8 * d + 2 * b], acc);
      acc = fmaf((float)((hi >> (8 * b)) & 0xffu), v[8 * d + 2 * b + 1], acc);
    }
  }
  return acc;
}

// The 32 elements of unit v (half a group) of a stored vector as fp32 registers; zeros past the end.
template <typename XT>
__device__ __forceinline__ void load_unit32(const XT* __restrict__ vec, int v, int nunit, float* out) {
  if (v < nunit) {
    constexpr int PER = DT<XT>::VEC;
#pragma unroll
    for (int p = 0; p < NV / PER; ++p) DT<XT>::unpack(load16(vec + (size_t)v * NV + p * PER), out + p * PER);
  } else {
#pragma unroll
    for (int j = 0; j < NV; ++j) out[j] = 0.f;
  }
}

// h[i, j] = silu(W1'_i[j,:] . x) * (W3'_i[j,:] . x) with W' = scale * (nibble - 8) per group.
template <typename XT, int NCH>
__global__ __launch_bounds__(256) void ffn_up_q4_kernel(ExpertSrc src, const int32_t* __restrict__ idx,
                                                         const XT* __restrict__ x,
                                                         float* __restrict__ hbuf, int H, int F, int k,
                                                         int rpw) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  const int nunit = H / NV;           // 32-weight units per row
  const int gpr = H / GROUP;          // scales per row
  float xr[NCH][NV];
  float sx[NCH];                      // sum of the lane's x elements per chunk: the offset correction
  int off[NCH], goff[NCH];            // byte offset of the lane's codes / index of its scale in a row
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int v = c * WAVE + lane;
    load_unit32<XT>(x, v, nunit, xr[c]);
    const int vc = v < nunit ? v : nunit - 1;
    off[c] = vc * (NV / 2);
    goff[c] = vc >> 1;
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < NV; ++j) s += xr[c][j];
    sx[c] = s;
  }
  const size_t hf2 = (size_t)H * F / 2;          // bytes of one matrix's codes
  const size_t ng1 = (size_t)F * gpr;            // scales of W1 (and of W3)
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
    const float* sc = reinterpret_cast<const float*>(base + 3 * hf2);
    float* hout = hbuf + (size_t)i * F + j0;
    auto issue = [&](int rr, u32x4 (&qa)[NCH], u32x4 (&qb)[NCH], float (&sa)[NCH], float (&sb)[NCH]) {
      const size_t row = (size_t)(j0 + rr);
      const uint8_t* w1 = base + row * (H / 2);
      const uint8_t* w3 = w1 + hf2;
      const float* s1 = sc + row * gpr;
      const float* s3 = s1 + ng1;
#pragma unroll
      for (int c = 0; c < NCH; ++c) {
        qa[c] = load16_stream(w1 + off[c]);
        qb[c] = load16_stream(w3 + off[c]);
        sa[c] = s1[goff[c]];
        sb[c] = s3[goff[c]];
      }
    };
    auto finish = [&](int rr, const u32x4 (&qa)[NCH], const u32x4 (&qb)[NCH], const float (&sa)[NCH],
                      const float (&sb)[NCH]) {
      float a = 0.f, b = 0.f;
#pragma unroll
      for (int c = 0; c < NCH; ++c) {
        a = fmaf(sa[c], fmaf(-8.f, sx[c], dot_nibbles(qa[c], xr[c], 0.f)), a);
        b = fmaf(sb[c], fmaf(-8.f, sx[c], dot_nibbles(qb[c], xr[c], 0.f)), b);
      }
      a = wave_sum(a);
      b = wave_sum(b);
      if (lane == 0) hout[rr] = a / (1.f + expf(-a)) * b;
    };
    u32x4 qa0[NCH], qb0[NCH], qa1[NCH], qb1[NCH];
    float sa0[NCH], sb0[NCH], sa1[NCH], sb1[NCH];
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

// y[r] = sum_i gate[i] * (W2'_i[r,:] . h_i).  Block shape of the other w2 kernels.
template <typename YT, int CPW>
__global__ __launch_bounds__(1024) void ffn_down_q4_kernel(ExpertSrc src, const int32_t* __restrict__ idx,
                                                            const float* __restrict__ gate,
                                                            const float* __restrict__ hbuf,
                                                            YT* __restrict__ y, int H, int F, int k, int rpb,
                                                            int nwc) {
  constexpr int RIF = 2;
  extern __shared__ float part[];  // [nw][rpb]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  const int cw = wave % nwc, eg = wave / nwc, n_eg = nw / nwc;
  const int nunit = F / NV, gpr = F / GROUP;
  const int r0 = blockIdx.x * rpb;
  float* mypart = part + wave * rpb;
  if (lane == 0)
    for (int t = 0; t < rpb; ++t) mypart[t] = 0.f;
  int off[CPW], goff[CPW];
#pragma unroll
  for (int c = 0; c < CPW; ++c) {
    const int v = (cw * CPW + c) * WAVE + lane;
    const int vc = v < nunit ? v : nunit - 1;
    off[c] = vc * (NV / 2);
    goff[c] = vc >> 1;
  }
  const size_t hf2 = (size_t)H * F / 2;
  for (int i = eg; i < k; i += n_eg) {
    bool ok;
    const uint8_t* base = static_cast<const uint8_t*>(expert_ptr(src, idx, i, &ok));
    const float g = ok ? gate[i] : 0.f;   // an idx entry that is no expert id adds nothing
    const uint8_t* w2 = base + 2 * hf2;
    const float* s2 = reinterpret_cast<const float*>(base + 3 * hf2) + 2 * (size_t)F * (H / GROUP);
    const float* hv = hbuf + (size_t)i * F;
    float hr[CPW][NV], sh[CPW];
#pragma unroll
    for (int c = 0; c < CPW; ++c) {
      load_unit32<float>(hv, (cw * CPW + c) * WAVE + lane, nunit, hr[c]);
      float s = 0.f;
#pragma unroll
      for (int j = 0; j < NV; ++j) s += hr[c][j];
      sh[c] = s;
    }
#pragma unroll 1
    for (int rr = 0; rr < rpb; rr += RIF) {
      u32x4 q[RIF][CPW];
      float sr[RIF][CPW];
#pragma unroll
      for (int u = 0; u < RIF; ++u) {
        int row = r0 + rr + u;
        row = row < H ? row : H - 1;
        const uint8_t* p = w2 + (size_t)row * (F / 2);
        const float* ps = s2 + (size_t)row * gpr;
#pragma unroll
        for (int c = 0; c < CPW; ++c) {
          q[u][c] = load16_stream(p + off[c]);
          sr[u][c] = ps[goff[c]];
        }
      }
#pragma unroll
      for (int u = 0; u < RIF; ++u) {
        float d = 0.f;
#pragma unroll
        for (int c = 0; c < CPW; ++c) d = fmaf(sr[u][c], fmaf(-8.f, sh[c], dot_nibbles(q[u][c], hr[c], 0.f)), d);
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
      y[r0 + t] = DT<YT>::from_f32(sum);
    }
  }
}

template <typename XT, int NCH>
hipError_t launch_up_q4_n(hipStream_t s, const Shape& sh, const ExpertSrc& src, const int32_t* idx,
                          const void* x, float* hbuf) {
  const int nw = 4;
  const long total = (long)sh.k * sh.F;
  // bound by the conversion arithmetic: four waves per SIMD (sixteen per CU) keep the vector units busy
  long rpw = (total + (long)num_cu() * nw * 4 - 1) / ((long)num_cu() * nw * 4);
  if (sh.host_link) rpw = (total + 127) / 128;
  if (rpw < 1) rpw = 1;
  if (g_tune_up_rpw > 0) rpw = g_tune_up_rpw;
  const int grid = (int)((total + nw * rpw - 1) / (nw * rpw));
  ffn_up_q4_kernel<XT, NCH><<<grid, nw * WAVE, 0, s>>>(src, idx, static_cast<const XT*>(x), hbuf, sh.H, sh.F,
                                                      sh.k, (int)rpw);
  return hipGetLastError();
}

template <typename XT>
hipError_t launch_up_q4(hipStream_t s, const Shape& sh, const ExpertSrc& src, const int32_t* idx,
                        const void* x, float* hbuf) {
  switch ((sh.H + NCHUNK - 1) / NCHUNK) {
    case 1: return launch_up_q4_n<XT, 1>(s, sh, src, idx, x, hbuf);
    case 2: return launch_up_q4_n<XT, 2>(s, sh, src, idx, x, hbuf);
    case 3: return launch_up_q4_n<XT, 3>(s, sh, src, idx, x, hbuf);
    case 4: return launch_up_q4_n<XT, 4>(s, sh, src, idx, x, hbuf);
  }
  return hipErrorInvalidValue;
}

template <typename YT, int CPW>
hipError_t launch_down_q4_n(hipStream_t s, const Shape& sh, const ExpertSrc& src, const int32_t* idx,
                            const float* gate, const float* hbuf, void* y, int nwb) {
  int n_eg, rpb;
  down_block_shape(sh, CPW, nwb, g_tune_down_eg, g_tune_down_rpb, &n_eg, &rpb);
  if (g_tune_down_eg == 0 && nwb > 4 && nwb <= 8 && sh.k >= 2) n_eg = 2;   // as for int8 rows: short rows, more waves
  const int grid = (sh.H + rpb - 1) / rpb;
  const int nw = nwb * n_eg;
  const size_t lds = (size_t)nw * rpb * sizeof(float);
  ffn_down_q4_kernel<YT, CPW><<<grid, nw * WAVE, lds, s>>>(src, idx, gate, hbuf, static_cast<YT*>(y), sh.H,
                                                          sh.F, sh.k, rpb, nwb);
  return hipGetLastError();
}

// Column chunks of 2048 weights: one or two per wave, up to 16 waves per expert group.
bool pick_q4_split(int F, int* cpw, int* nwb) {
  const int nc = (F + NCHUNK - 1) / NCHUNK;
  for (int c = 1; c <= 2; ++c)
    if ((nc + c - 1) / c <= 16) {
      *cpw = c;
      *nwb = (nc + c - 1) / c;
      return true;
    }
  return false;
}

template <typename YT>
hipError_t launch_down_q4(hipStream_t s, const Shape& sh, const ExpertSrc& src, const int32_t* idx,
                          const float* gate, const float* hbuf, void* y) {
  int cpw = 0, nwb = 0;
  if (!pick_q4_split(sh.F, &cpw, &nwb)) return hipErrorInvalidValue;
  return cpw == 1 ? launch_down_q4_n<YT, 1>(s, sh, src, idx, gate, hbuf, y, nwb)
                  : launch_down_q4_n<YT, 2>(s, sh, src, idx, gate, hbuf, y, nwb);
}

}  // namespace

bool q4_supported(const Shape& sh) {
  int cpw = 0, nwb = 0;
  return sh.H % GROUP == 0 && sh.F % GROUP == 0 && sh.H <= 4 * NCHUNK && pick_q4_split(sh.F, &cpw, &nwb);
}

hipError_t launch_ffn_up_q4(hipStream_t s, const Shape& sh, const ExpertSrc& src, const int32_t* idx,
                            const void* x, float* hbuf) {
  if (!q4_supported(sh)) return hipErrorInvalidValue;
  return sh.dtype == ODMOE_F32 ? launch_up_q4<float>(s, sh, src, idx, x, hbuf)
                               : launch_up_q4<bf16_t>(s, sh, src, idx, x, hbuf);
}

hipError_t launch_ffn_down_q4(hipStream_t s, const Shape& sh, const ExpertSrc& src, const int32_t* idx,
                              const float* gate, const float* hbuf, void* y) {
  if (!q4_supported(sh)) return hipErrorInvalidValue;
  return sh.dtype == ODMOE_F32 ? launch_down_q4<float>(s, sh, src, idx, gate, hbuf, y)
                               : launch_down_q4<bf16_t>(s, sh, src, idx, gate, hbuf, y);
}

hipError_t launch_quantize_pack4(hipStream_t s, const void* w, int32_t dtype, int64_t rows, int64_t cols,
                                 uint8_t* packed, float* scale) {
  if (rows <= 0 || cols <= 0) return hipSuccess;
  if (cols % GROUP || !packed || !scale) return hipErrorInvalidValue;
  const size_t n_groups = (size_t)rows * (size_t)(cols / GROUP);
  const size_t blocks = (n_groups + 3) / 4;
  if (blocks > 0x7fffffffULL) return hipErrorInvalidValue;
  if (dtype == ODMOE_F32)
    quantize_pack4_kernel<float><<<(unsigned)blocks, 256, 0, s>>>(static_cast<const float*>(w), n_groups, packed, scale);
  else
    quantize_pack4_kernel<bf16_t><<<(unsigned)blocks, 256, 0, s>>>(static_cast<const bf16_t*>(w), n_groups, packed,
                                                                  scale);
  return hipGetLastError();
}

}  // namespace odmoe
