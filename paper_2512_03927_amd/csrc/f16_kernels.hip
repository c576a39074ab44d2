// 16-bit experts of the shadow model (paper Sections 1 and 3.2: the mildest quantised copy the
// paper runs as its predictor is an FP16 copy of the FP32 model).  The expert buffer is the stored
// one, W1[F,H] | W3[F,H] | W2[H,F], with every weight rounded once to IEEE binary16 (nearest, ties to
// even, |w| clipped to 65504): half the bytes of an fp32 expert.  Activations, the SwiGLU
// intermediate and the sums stay fp32, so these are layers of dtype ODMOE_F32 only.
//
// The two GEMVs have the shape of the other expert GEMVs (input slice in registers, every wave
// streams a contiguous run of rows through two register sets; the w2 kernel's block owns a few
// output rows, its waves are column slices x expert groups).  A 128-bit load brings 8 weights;
// binary16 -> fp32 and the multiply-add are one mixed-precision FMA per weight, so the kernels
// are bound by the weight stream like the stored-dtype ones.
#include "gemv_common.hpp"

namespace odmoe {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
constexpr int HV = 8;               // weights per 128-bit load
constexpr int HCHUNK = WAVE * HV;   // weights a wave covers per load instruction: 512

// w[i] -> binary16 bits (and the value it stands for, back in the stored dtype)
template <typename T>
__global__ __launch_bounds__(256) void round_f16_kernel(const T* __restrict__ w, size_t n,
                                                         uint16_t* __restrict__ code, T* __restrict__ deq) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
    float v = DT<T>::to_f32(w[i]);
    v = fminf(fmaxf(v, -65504.f), 65504.f);
    const _Float16 h = (_Float16)v;             // round to nearest even
    if (code) code[i] = __builtin_bit_cast(uint16_t, h);
    if (deq) deq[i] = DT<T>::from_f32((float)h);
  }
}

// acc + sum_j w_j * v_j over the 8 binary16 weights of q
__device__ __forceinline__ float dot_halves(u32x4 q, const float* v, float acc) {
  const half8 w = __builtin_bit_cast(half8, q);
#pragma unroll
  for (int j = 0; j < HV; ++j) acc = fmaf((float)w[j], v[j], acc);
  return acc;
}

// The 8 fp32 elements of group v of a vector as registers (zeros past the end).
__device__ __forceinline__ void load_group8(const float* __restrict__ vec, int v, int nvec, float* out) {
  if (v < nvec) {
    DT<float>::unpack(load16(vec + (size_t)v * HV), out);
    DT<float>::unpack(load16(vec + (size_t)v * HV + 4), out + 4);
  } else {
#pragma unroll
    for (int j = 0; j < HV; ++j) out[j] = 0.f;
  }
}

// h[i, j] = silu(W1_i[j,:] . x) * (W3_i[j,:] . x), weights binary16, x fp32 in registers.
template <int NCH>
__global__ __launch_bounds__(256) void ffn_up_f16_kernel(ExpertSrc src, const int32_t* __restrict__ idx,
                                                          const float* __restrict__ x,
                                                          float* __restrict__ hbuf, int H, int F, int k,
                                                          int rpw) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  const int nvec = H / HV;
  float xr[NCH][HV];
  int off[NCH];   // element offset of this lane's group in chunk c (clamped into the row)
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int v = c * WAVE + lane;
    load_group8(x, v, nvec, xr[c]);
    off[c] = (v < nvec ? v : nvec - 1) * HV;
  }
  const size_t hf = (size_t)H * F;
  const int total = k * F;
  const int r_begin = (blockIdx.x * nw + wave) * rpw;
  const int r_end = (r_begin + rpw < total) ? r_begin + rpw : total;
  int r = r_begin;
  while (r < r_end) {
    const int i = r / F;
    const int j0 = r - i * F;
    const int seg_end = ((i + 1) * F < r_end) ? (i + 1) * F : r_end;
    const int nrow = seg_end - r;
    const uint16_t* base = static_cast<const uint16_t*>(expert_ptr(src, idx, i));
    float* hout = hbuf + (size_t)i * F + j0;
    auto issue = [&](int rr, u32x4 (&qa)[NCH], u32x4 (&qb)[NCH]) {
      const uint16_t* w1 = base + (size_t)(j0 + rr) * H;
      const uint16_t* w3 = w1 + hf;
#pragma unroll
      for (int c = 0; c < NCH; ++c) {
        qa[c] = load16_stream(w1 + off[c]);
        qb[c] = load16_stream(w3 + off[c]);
      }
    };
    auto finish = [&](int rr, const u32x4 (&qa)[NCH], const u32x4 (&qb)[NCH]) {
      float a = 0.f, b = 0.f;
#pragma unroll
      for (int c = 0; c < NCH; ++c) {
        a = dot_halves(qa[c], xr[c], a);
        b = dot_halves(qb[c], xr[c], b);
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

// y[r] = sum_i gate[i] * (W2_i[r,:] . h_i), weights binary16, h and y fp32.
template <int CPW>
__global__ __launch_bounds__(CPW <= 4 ? 1024 : 512) void ffn_down_f16_kernel(
    ExpertSrc src, const int32_t* __restrict__ idx, const float* __restrict__ gate,
    const float* __restrict__ hbuf, float* __restrict__ y, int H, int F, int k, int rpb, int nwc) {
  constexpr int RIF = 2;  // rows in flight
  extern __shared__ float part[];  // [nw][rpb]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  const int cw = wave % nwc, eg = wave / nwc, n_eg = nw / nwc;
  const int nvec = F / HV;
  const int r0 = blockIdx.x * rpb;
  float* mypart = part + wave * rpb;
  if (lane == 0)
    for (int t = 0; t < rpb; ++t) mypart[t] = 0.f;
  int off[CPW];
#pragma unroll
  for (int c = 0; c < CPW; ++c) {
    const int v = (cw * CPW + c) * WAVE + lane;
    off[c] = (v < nvec ? v : nvec - 1) * HV;
  }
  const size_t hf = (size_t)H * F;
  for (int i = eg; i < k; i += n_eg) {
    bool ok;
    const uint16_t* w2 = static_cast<const uint16_t*>(expert_ptr(src, idx, i, &ok)) + 2 * hf;
    const float g = ok ? gate[i] : 0.f;   // an idx entry that is no expert id adds nothing
    const float* hv = hbuf + (size_t)i * F;
    float hr[CPW][HV];
#pragma unroll
    for (int c = 0; c < CPW; ++c) load_group8(hv, (cw * CPW + c) * WAVE + lane, nvec, hr[c]);
#pragma unroll 1
    for (int rr = 0; rr < rpb; rr += RIF) {
      u32x4 q[RIF][CPW];
#pragma unroll
      for (int u = 0; u < RIF; ++u) {
        int row = r0 + rr + u;
        row = row < H ? row : H - 1;
        const uint16_t* p = w2 + (size_t)row * F;
#pragma unroll
        for (int c = 0; c < CPW; ++c) q[u][c] = load16_stream(p + off[c]);
      }
#pragma unroll
      for (int u = 0; u < RIF; ++u) {
        float d = 0.f;
#pragma unroll
        for (int c = 0; c < CPW; ++c) d = dot_halves(q[u][c], hr[c], d);
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
      y[r0 + t] = sum;
    }
  }
}

template <int NCH>
hipError_t launch_up_f16_n(hipStream_t s, const Shape& sh, const ExpertSrc& src, const int32_t* idx,
                           const void* x, float* hbuf) {
  const int nw = 4;
  const long total = (long)sh.k * sh.F;
  // as for the stored-dtype GEMV: one wave per SIMD when a wave's two register sets hold 16 KB or
  // more of loads in flight and the rows are many, four times as many waves otherwise
  long rpw = (total + (long)num_cu() * nw - 1) / ((long)num_cu() * nw);
  if (rpw < 16 || NCH < 8) rpw = (total + (long)num_cu() * nw * 4 - 1) / ((long)num_cu() * nw * 4);
  if (sh.host_link) rpw = (total + 127) / 128;
  if (rpw < 1) rpw = 1;
  if (g_tune_up_rpw > 0) rpw = g_tune_up_rpw;
  const int grid = (int)((total + nw * rpw - 1) / (nw * rpw));
  ffn_up_f16_kernel<NCH><<<grid, nw * WAVE, 0, s>>>(src, idx, static_cast<const float*>(x), hbuf, sh.H, sh.F,
                                                   sh.k, (int)rpw);
  return hipGetLastError();
}

template <int CPW>
hipError_t launch_down_f16_n(hipStream_t s, const Shape& sh, const ExpertSrc& src, const int32_t* idx,
                             const float* gate, const float* hbuf, void* y, int nwb) {
  int n_eg, rpb;
  down_block_shape(sh, CPW, nwb, g_tune_down_eg, g_tune_down_rpb, &n_eg, &rpb);
  const int grid = (sh.H + rpb - 1) / rpb;
  const int nw = nwb * n_eg;
  const size_t lds = (size_t)nw * rpb * sizeof(float);
  ffn_down_f16_kernel<CPW><<<grid, nw * WAVE, lds, s>>>(src, idx, gate, hbuf, static_cast<float*>(y), sh.H,
                                                       sh.F, sh.k, rpb, nwb);
  return hipGetLastError();
}

}  // namespace

bool f16_supported(const Shape& sh) {
  int cpw = 0, nwb = 0;
  return sh.dtype == ODMOE_F32 && sh.H % HV == 0 && sh.F % HV == 0 && sh.H <= 16 * HCHUNK &&
         pick_down_split((sh.F + HCHUNK - 1) / HCHUNK, &cpw, &nwb);
}

hipError_t launch_ffn_up_f16(hipStream_t s, const Shape& sh, const ExpertSrc& src, const int32_t* idx,
                             const void* x, float* hbuf) {
  if (!f16_supported(sh)) return hipErrorInvalidValue;
  switch ((sh.H + HCHUNK - 1) / HCHUNK) {
#define ODMOE_CASE(N) case N: return launch_up_f16_n<N>(s, sh, src, idx, x, hbuf);
    ODMOE_CASE(1) ODMOE_CASE(2) ODMOE_CASE(3) ODMOE_CASE(4) ODMOE_CASE(5) ODMOE_CASE(6)
    ODMOE_CASE(7) ODMOE_CASE(8) ODMOE_CASE(9) ODMOE_CASE(10) ODMOE_CASE(11) ODMOE_CASE(12)
    ODMOE_CASE(13) ODMOE_CASE(14) ODMOE_CASE(15) ODMOE_CASE(16)
#undef ODMOE_CASE
  }
  return hipErrorInvalidValue;
}

hipError_t launch_ffn_down_f16(hipStream_t s, const Shape& sh, const ExpertSrc& src, const int32_t* idx,
                               const float* gate, const float* hbuf, void* y) {
  if (!f16_supported(sh)) return hipErrorInvalidValue;
  int cpw = 0, nwb = 0;
  if (!pick_down_split((sh.F + HCHUNK - 1) / HCHUNK, &cpw, &nwb)) return hipErrorInvalidValue;
  switch (cpw) {
#define ODMOE_CASE(N) case N: return launch_down_f16_n<N>(s, sh, src, idx, gate, hbuf, y, nwb);
    ODMOE_CASE(1) ODMOE_CASE(2) ODMOE_CASE(3) ODMOE_CASE(4) ODMOE_CASE(5) ODMOE_CASE(6)
    ODMOE_CASE(7) ODMOE_CASE(8)
#undef ODMOE_CASE
  }
  return hipErrorInvalidValue;
}

hipError_t launch_round_f16(hipStream_t s, const void* w, int32_t dtype, size_t n, uint16_t* code, void* deq) {
  if (n == 0) return hipSuccess;
  const size_t want = (n + 255) / 256;
  const unsigned blocks = (unsigned)(want < 8192 ? want : 8192);
  if (dtype == ODMOE_F32)
    round_f16_kernel<float><<<blocks, 256, 0, s>>>(static_cast<const float*>(w), n, code, static_cast<float*>(deq));
  else
    round_f16_kernel<bf16_t><<<blocks, 256, 0, s>>>(static_cast<const bf16_t*>(w), n, code,
                                                   static_cast<bf16_t*>(deq));
  return hipGetLastError();
}

}  // namespace odmoe
