// Prefill path (paper Section 3.3): all experts of the layer are available, token embeddings
// are grouped by the expert they were routed to, and each expert runs one larger matrix
// multiplication.  On gfx950 that multiplication goes to the matrix cores
// (v_mfma_f32_32x32x16_bf16); everything else here is bookkeeping around it:
//
//   sort      token-slots (t, i) bucketed by expert -> offsets[E+1], perm, inv, list of M-tiles
//   gemm1     Hbuf[p, :] = silu(X[tok(p)] W1_e^T) * (X[tok(p)] W3_e^T)       bf16 [T*k, F]
//   gemm2     Ybuf[p, :] = Hbuf[p, :] W2_e^T                                  fp32 [T*k, H]
//   combine   Y[t] = sum_i gate[t,i] * Ybuf[inv[t*k+i]]                       (fixed order, no atomics)
//
// Both GEMMs are "NT": activations [M, K] and weights [N, K] are row-major with K contiguous,
// which is exactly how the MFMA operands want to be fed (8 consecutive K elements per lane).
#include "kernels.h"

namespace odmoe {
namespace {

constexpr int BM = 128;  // token rows per block tile
constexpr int BN = 64;   // weight rows per block tile (per matrix)
constexpr int BK = 64;   // K elements per pipeline step (128 bytes per row)
constexpr int GEMM_THREADS = 256;

typedef uint16_t bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef const __attribute__((address_space(1))) u32x4* global_u32x4_ptr;

__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

// ---------------------------------------------------------------------------------------------
// Bucket the n = T*k token-slots by expert.  One block.  Slots with an out-of-range expert id
// are left out (inv = -1) and contribute nothing.
// tiles: (expert, first row within the expert) pairs of BM rows each; *n_tiles their number.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void sort_slots_kernel(const int32_t* __restrict__ idx, int n, int E,
                                                           int32_t* __restrict__ offsets,
                                                           int32_t* __restrict__ perm,
                                                           int32_t* __restrict__ inv,
                                                           int32_t* __restrict__ tiles,
                                                           int32_t* __restrict__ n_tiles) {
  __shared__ int32_t cnt[ODMOE_MAX_EXPERTS];
  __shared__ int32_t start[ODMOE_MAX_EXPERTS + 1];
  for (int e = threadIdx.x; e < E; e += blockDim.x) cnt[e] = 0;
  __syncthreads();
  for (int s = threadIdx.x; s < n; s += blockDim.x) {
    const int e = idx[s];
    if (e >= 0 && e < E) atomicAdd(&cnt[e], 1);
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int run = 0, nt = 0;
    for (int e = 0; e < E; ++e) {
      start[e] = run;
      offsets[e] = run;
      for (int m0 = 0; m0 < cnt[e]; m0 += BM) {
        tiles[2 * nt] = e;
        tiles[2 * nt + 1] = m0;
        ++nt;
      }
      run += cnt[e];
    }
    start[E] = run;
    offsets[E] = run;
    *n_tiles = nt;
  }
  __syncthreads();
  for (int e = threadIdx.x; e < E; e += blockDim.x) cnt[e] = 0;  // reuse as cursors
  __syncthreads();
  for (int s = threadIdx.x; s < n; s += blockDim.x) {
    const int e = idx[s];
    if (e >= 0 && e < E) {
      const int p = start[e] + atomicAdd(&cnt[e], 1);
      perm[p] = s;
      inv[s] = p;
    } else {
      inv[s] = -1;
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Grouped GEMM.  Block tile BM x BN (x2 matrices when DUAL), K pipelined in steps of BK through
// double-buffered LDS; 4 waves as 2 (M) x 2 (N), each wave 64 x 32 outputs per matrix.
// LDS rows are 128 bytes; the 16-byte piece p of row r sits at slot p ^ (r & 7), which makes
// both the staging stores and the MFMA fragment reads conflict-free.
//   DUAL  : B0 = W1 rows, B1 = W3 rows; out = bf16( silu(A B0^T) * (A B1^T) )
//   !DUAL : out = fp32( A B0^T )
// blockIdx.x = N tile, blockIdx.y = entry of the M-tile list (blocks past *n_tiles exit).
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ int lds_slot(int row, int piece) { return row * BK + ((piece ^ (row & 7)) << 3); }

template <bool DUAL>
__global__ __launch_bounds__(GEMM_THREADS) void grouped_gemm_kernel(
    const bf16_t* __restrict__ A, int lda, const int32_t* __restrict__ a_slot, int slot_div,
    const void* const* __restrict__ table, int table_off, size_t b0_off, size_t b1_off,
    const int32_t* __restrict__ offsets, const int32_t* __restrict__ tiles,
    const int32_t* __restrict__ n_tiles, void* __restrict__ out, int ldo, int N, int K) {
  constexpr int NB = DUAL ? 2 : 1;
  extern __shared__ __attribute__((aligned(16))) bf16_t smem[];
  bf16_t* As = smem;                       // [2][BM*BK]
  bf16_t* Bs = smem + 2 * BM * BK;         // [2][NB][BN*BK]

  if ((int)blockIdx.y >= *n_tiles) return;
  const int e = tiles[2 * blockIdx.y];
  const int row_lo = offsets[e] + tiles[2 * blockIdx.y + 1];
  const int row_end = offsets[e + 1];
  const int n0 = blockIdx.x * BN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  // ---- staging assignment: thread -> (row tid/8 + 32 j, 16-byte piece tid%8)
  const int st_row = tid >> 3, st_piece = tid & 7;
  const bf16_t* a_src[BM / 32];
#pragma unroll
  for (int j = 0; j < BM / 32; ++j) {
    int p = row_lo + st_row + 32 * j;
    p = p < row_end ? p : row_end - 1;                 // rows past the group: any valid row
    const int src_row = a_slot ? a_slot[p] / slot_div : p;
    a_src[j] = A + (size_t)src_row * lda + st_piece * 8;
  }
  const bf16_t* wbase = static_cast<const bf16_t*>(table[table_off + e]);
  const bf16_t* b_src[NB][BN / 32];
#pragma unroll
  for (int j = 0; j < BN / 32; ++j) {
    int n = n0 + st_row + 32 * j;
    n = n < N ? n : N - 1;
    b_src[0][j] = wbase + b0_off + (size_t)n * K + st_piece * 8;
    if constexpr (DUAL) b_src[1][j] = wbase + b1_off + (size_t)n * K + st_piece * 8;
  }

  u32x4 ra[BM / 32], rb[NB][BN / 32];
  auto load_tile = [&](int kt) {
    const int ko = kt * BK;
#pragma unroll
    for (int j = 0; j < BM / 32; ++j) ra[j] = *reinterpret_cast<const u32x4*>(a_src[j] + ko);
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
      for (int j = 0; j < BN / 32; ++j)
        rb[b][j] = __builtin_nontemporal_load((global_u32x4_ptr)(b_src[b][j] + ko));
  };
  auto store_tile = [&](int buf) {
#pragma unroll
    for (int j = 0; j < BM / 32; ++j)
      *reinterpret_cast<u32x4*>(As + buf * BM * BK + lds_slot(st_row + 32 * j, st_piece)) = ra[j];
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
      for (int j = 0; j < BN / 32; ++j)
        *reinterpret_cast<u32x4*>(Bs + (buf * NB + b) * BN * BK + lds_slot(st_row + 32 * j, st_piece)) = rb[b][j];
  };

  f32x16 acc[2][NB];
#pragma unroll
  for (int mt = 0; mt < 2; ++mt)
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[mt][b][i] = 0.f;

  const int nk = K / BK;
  load_tile(0);
  store_tile(0);
  __syncthreads();
  const int fr = lane & 31, fg = lane >> 5;  // fragment row within a 32-tile, K half
  for (int kt = 0; kt < nk; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < nk) load_tile(kt + 1);
    const bf16_t* as = As + buf * BM * BK;
#pragma unroll
    for (int s = 0; s < BK / 16; ++s) {
      const int piece = 2 * s + fg;
      bf16x8 af[2], bfrag[NB];
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
        af[mt] = *reinterpret_cast<const bf16x8*>(as + lds_slot(wm * 64 + mt * 32 + fr, piece));
#pragma unroll
      for (int b = 0; b < NB; ++b)
        bfrag[b] = *reinterpret_cast<const bf16x8*>(Bs + (buf * NB + b) * BN * BK + lds_slot(wn * 32 + fr, piece));
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int b = 0; b < NB; ++b)
          acc[mt][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[mt], bfrag[b], acc[mt][b], 0, 0, 0);
    }
    if (kt + 1 < nk) store_tile(buf ^ 1);
    __syncthreads();
  }

  // ---- epilogue.  Accumulator layout: column = lane % 32, row = (i/4)*8 + (lane/32)*4 + i%4.
  const int col = n0 + wn * 32 + fr;
  if (col >= N) return;
#pragma unroll
  for (int mt = 0; mt < 2; ++mt) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int m = (i >> 2) * 8 + fg * 4 + (i & 3);
      const int p = row_lo + wm * 64 + mt * 32 + m;
      if (p < row_end) {
        if constexpr (DUAL) {
          const float a = acc[mt][0][i], b = acc[mt][1][i];
          static_cast<bf16_t*>(out)[(size_t)p * ldo + col] = f32_to_bf16(a / (1.f + expf(-a)) * b);
        } else {
          static_cast<float*>(out)[(size_t)p * ldo + col] = acc[mt][0][i];
        }
      }
    }
  }
}

// Y[t, :] = sum_i gate[t,i] * Ybuf[inv[t*k+i], :], rounded once to bf16.  One block per token.
__global__ __launch_bounds__(256) void combine_kernel(const float* __restrict__ ybuf,
                                                       const int32_t* __restrict__ inv,
                                                       const float* __restrict__ gate,
                                                       bf16_t* __restrict__ Y, int H, int k) {
  const int t = blockIdx.x;
  for (int c = threadIdx.x * 4; c < H; c += blockDim.x * 4) {
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int i = 0; i < k; ++i) {
      const int p = inv[t * k + i];
      if (p < 0) continue;
      const float g = gate[t * k + i];
      const f32x4 v = *reinterpret_cast<const f32x4*>(ybuf + (size_t)p * H + c);
      acc.x = fmaf(g, v.x, acc.x); acc.y = fmaf(g, v.y, acc.y);
      acc.z = fmaf(g, v.z, acc.z); acc.w = fmaf(g, v.w, acc.w);
    }
    const uint32_t lo = (uint32_t)f32_to_bf16(acc.x) | ((uint32_t)f32_to_bf16(acc.y) << 16);
    const uint32_t hi = (uint32_t)f32_to_bf16(acc.z) | ((uint32_t)f32_to_bf16(acc.w) << 16);
    *reinterpret_cast<uint2*>(Y + (size_t)t * H + c) = make_uint2(lo, hi);
  }
}

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct Carve {
  int32_t *offsets, *perm, *inv, *tiles, *n_tiles;
  bf16_t* hbuf;
  float* ybuf;
  size_t total;
};

Carve carve(const Shape& sh, int32_t T, void* base) {
  const size_t n = (size_t)T * sh.k;
  const size_t max_tiles = (size_t)sh.E + (n + BM - 1) / BM;
  char* p = static_cast<char*>(base);
  size_t off = 0;
  Carve c{};
  auto take = [&](size_t bytes) { char* q = p ? p + off : nullptr; off = align_up(off + bytes, 256); return q; };
  c.offsets = reinterpret_cast<int32_t*>(take((sh.E + 1) * sizeof(int32_t)));
  c.perm = reinterpret_cast<int32_t*>(take(n * sizeof(int32_t)));
  c.inv = reinterpret_cast<int32_t*>(take(n * sizeof(int32_t)));
  c.tiles = reinterpret_cast<int32_t*>(take(2 * max_tiles * sizeof(int32_t)));
  c.n_tiles = reinterpret_cast<int32_t*>(take(sizeof(int32_t)));
  c.hbuf = reinterpret_cast<bf16_t*>(take(n * sh.F * sizeof(bf16_t)));
  c.ybuf = reinterpret_cast<float*>(take(n * sh.H * sizeof(float)));
  c.total = off;
  return c;
}

constexpr size_t GEMM1_LDS = (2 * BM * BK + 2 * 2 * BN * BK) * sizeof(bf16_t);  // 64 KB
constexpr size_t GEMM2_LDS = (2 * BM * BK + 2 * 1 * BN * BK) * sizeof(bf16_t);  // 48 KB
bool g_prefill_attr_set = false;

}  // namespace

bool prefill_supported(const Shape& sh) {
  return sh.dtype == ODMOE_BF16 && sh.H % BK == 0 && sh.F % BK == 0;
}

size_t prefill_workspace_bytes(const Shape& sh, int32_t T) { return carve(sh, T, nullptr).total; }

hipError_t launch_prefill(hipStream_t s, const Shape& sh, const void* const* table, int32_t table_off,
                          const int32_t* idx, const float* gate, const void* x, int32_t T, void* y,
                          void* workspace, size_t workspace_bytes) {
  if (!prefill_supported(sh)) return hipErrorNotSupported;
  if (T <= 0) return hipSuccess;
  const Carve c = carve(sh, T, workspace);
  if (!workspace || c.total > workspace_bytes) return hipErrorInvalidValue;
  if (!g_prefill_attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(grouped_gemm_kernel<true>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)GEMM1_LDS);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(grouped_gemm_kernel<false>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)GEMM2_LDS);
    if (e != hipSuccess) return e;
    g_prefill_attr_set = true;
  }
  const int n = T * sh.k;
  const int max_tiles = sh.E + (n + BM - 1) / BM;
  const size_t hf = (size_t)sh.H * sh.F;

  sort_slots_kernel<<<1, 1024, 0, s>>>(idx, n, sh.E, c.offsets, c.perm, c.inv, c.tiles, c.n_tiles);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;

  dim3 g1((sh.F + BN - 1) / BN, max_tiles);
  grouped_gemm_kernel<true><<<g1, GEMM_THREADS, GEMM1_LDS, s>>>(
      static_cast<const bf16_t*>(x), sh.H, c.perm, sh.k, table, table_off, 0, hf, c.offsets, c.tiles,
      c.n_tiles, c.hbuf, sh.F, sh.F, sh.H);
  if ((e = hipGetLastError()) != hipSuccess) return e;

  dim3 g2((sh.H + BN - 1) / BN, max_tiles);
  grouped_gemm_kernel<false><<<g2, GEMM_THREADS, GEMM2_LDS, s>>>(
      c.hbuf, sh.F, nullptr, 1, table, table_off, 2 * hf, 0, c.offsets, c.tiles, c.n_tiles, c.ybuf, sh.H,
      sh.H, sh.F);
  if ((e = hipGetLastError()) != hipSuccess) return e;

  combine_kernel<<<T, 256, 0, s>>>(c.ybuf, c.inv, gate, static_cast<bf16_t*>(y), sh.H, sh.k);
  return hipGetLastError();
}

}  // namespace odmoe
