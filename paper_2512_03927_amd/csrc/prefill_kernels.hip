// Prefill path (paper Section 3.3): all experts of the layer are available, token embeddings
// are grouped by the expert they were routed to, and each expert runs one larger matrix
// multiplication.  On gfx950 that multiplication goes to the matrix cores
// (v_mfma_f32_32x32x16_bf16 for bf16 layers, v_mfma_f32_32x32x2_f32 for fp32 layers, the paper's
// full precision); everything else here is bookkeeping around it:
//
//   sort      token-slots (t, i) bucketed by expert -> offsets[E+1], perm, inv, list of M-tiles
//   gemm1     Hbuf[p, :] = silu(X[tok(p)] W1_e^T) * (X[tok(p)] W3_e^T)       dtype [T*k, F]
//   gemm2     Ybuf[p, :] = Hbuf[p, :] W2_e^T                                  fp32 [T*k, H]
//   combine   Y[t] = sum_i gate[t,i] * Ybuf[inv[t*k+i]]                       (fixed order, no atomics)
//
// Both GEMMs are "NT": activations [M, K] and weights [N, K] are row-major with K contiguous,
// which is exactly how the MFMA operands want to be fed (8 consecutive K elements per lane).
#include "kernels.h"

#include <type_traits>

namespace odmoe {
namespace {

constexpr int BMX = 320;     // most rows of one expert a block takes (one "chunk"): ten 32-row tiles, what
                             // the registers (160 accumulators of 256 per lane) and a two-deep ring allow
constexpr int BN = 256;      // weight rows per block tile: two 128-row halves (W1 and W3 rows of the
                             // same 128 ffn columns for the first GEMM, 256 consecutive rows for the second)
constexpr int GEMM_THREADS = 512;
constexpr int MAX_KSPLIT = 8;
constexpr int TILE_REC = 5;   // ints per entry of the chunk list
constexpr unsigned K_ROTATE = 24;  // K-steps between the starting points of neighbouring N tiles
constexpr size_t GEMM_LDS = 144 * 1024;  // the LDS ring; its depth depends on the rows of the chunk

typedef uint16_t bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// Element types of the grouped GEMM.  A pipeline step is one 128-byte line per row whatever the
// type; a 16-byte piece of it (what one lane fetches and what one lane reads back as an MFMA
// fragment) holds PIECE elements.
template <typename E>
struct ElemT;
template <>
struct ElemT<uint16_t> {
  static constexpr int PIECE = 8, BKE = 64;
};
template <>
struct ElemT<float> {
  static constexpr int PIECE = 4, BKE = 32;
};
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
// tiles: one record of TILE_REC ints per chunk: expert, first row in the sorted order, rows (at most
// BMX, the rows of an expert split evenly over its chunks in whole 32-row tiles), index of the expert's first chunk and
// the number of its chunks; *n_tiles their number.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void sort_slots_kernel(const int32_t* __restrict__ idx, int n, int E,
                                                           int32_t* __restrict__ offsets,
                                                           int32_t* __restrict__ perm,
                                                           int32_t* __restrict__ inv,
                                                           int32_t* __restrict__ tiles,
                                                           int32_t* __restrict__ n_tiles) {
  __shared__ int32_t cnt[ODMOE_MAX_EXPERTS];
  __shared__ int32_t start[ODMOE_MAX_EXPERTS + 1];
  __shared__ int32_t order[ODMOE_MAX_EXPERTS];
  for (int e = threadIdx.x; e < E; e += blockDim.x) cnt[e] = 0;
  __syncthreads();
  for (int s = threadIdx.x; s < n; s += blockDim.x) {
    const int e = idx[s];
    if (e >= 0 && e < E) atomicAdd(&cnt[e], 1);
  }
  __syncthreads();
  // Order in which the experts' chunks are listed (= dispatched): experts ranked by token count,
  // the larger half interleaved with the smaller half (1st, (E/2+1)th, 2nd, ...).  Large chunks are
  // bound by the matrix cores and the fills, small ones by the weight stream; running them side by
  // side is faster than either sorted order, and the smallest experts end the launch.
  for (int e = threadIdx.x; e < E; e += blockDim.x) {
    const int c = cnt[e];
    int rank = 0;
    for (int j = 0; j < E; ++j) rank += (cnt[j] > c) || (cnt[j] == c && j < e);
    const int half = (E + 1) / 2;
    order[rank < half ? 2 * rank : 2 * (rank - half) + 1] = e;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int run = 0, nt = 0;
    for (int e = 0; e < E; ++e) {
      start[e] = run;
      offsets[e] = run;
      run += cnt[e];
    }
    start[E] = run;
    offsets[E] = run;
    for (int p = 0; p < E; ++p) {
      const int e = order[p];
      const int nch = (cnt[e] + BMX - 1) / BMX;
      // rows split evenly over the chunks, rounded up to whole 32-row MFMA tiles (the number of
      // chunks stays nch: per <= BMX, and (nch - 1) * per < cnt because (nch - 1) * BMX < cnt)
      const int per = nch ? ((cnt[e] + nch - 1) / nch + 31) & ~31 : 0;
      const int first = nt;
      for (int m0 = 0; m0 < cnt[e]; m0 += per) {
        int32_t* tl = tiles + TILE_REC * nt;
        tl[0] = e;
        tl[1] = start[e] + m0;   // first row of the chunk in the sorted order
        tl[2] = (cnt[e] - m0 < per) ? cnt[e] - m0 : per;
        tl[3] = first;
        tl[4] = nch;
        ++nt;
      }
    }
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
// Grouped GEMM  C[p, n] = sum_k A[row(p), k] * W_e[n, k]  for one chunk (up to BMX = 320 rows) of
// one expert e and BN = 256 weight rows (two 128-row halves).  Built around the weight stream,
// which is what bounds it:
//   - one block takes all rows of the chunk, so an expert with up to 320 tokens reads its weights
//     exactly once; the chunks of a larger expert are started together on one XCD (see the block
//     order in grouped_gemm_kernel) so that the second one finds the weight tile in L2;
//   - global memory goes straight into LDS (global_load_lds_dwordx4: a wave fills 1 KB = 8 rows of
//     128 bytes per instruction, every 128-byte line fully coalesced) in a ring of K-steps of one
//     128-byte line per row (64 bf16 or 32 fp32 elements); no staging registers, one s_barrier per
//     step, and the only vmcnt wait is for the step about to be used.  The ring holds 3 steps of
//     40 / 48 KB for up to 64 / 128 rows and 2 steps of 56 ... 72 KB for up to 192 ... 320 rows
//     (measured: deeper rings do not help: the CU's
//     vector L1 keeps only about 125 128-byte requests in flight whatever is queued behind them);
//   - blocks start their K loops at different steps (kt0): the rows of a row-major matrix lie a
//     multiple of 4 KB apart, and blocks that walk K in lockstep keep hitting the same memory
//     channels (weight stream alone: 4.8 TB/s in lockstep, 5.8 TB/s rotated);
//   - LDS rows are 128 bytes; the 16-byte piece q of row r sits at slot q ^ (r & 7) (the lane
//     that fills slot s of row r fetches piece s ^ (r & 7)), so the MFMA fragment reads are
//     conflict-free;
//   - 8 waves as 2 (M) x 4 (N, 32 columns of each 128-row half); the chunk's NT = ceil(rows/32)
//     row tiles go alternately to the two M groups, and a wave multiplies its (up to five) row
//     tiles by its two 32-column tiles (10 MFMAs per 7 fragment reads), which keeps LDS read
//     traffic below MFMA time; NT is a template parameter, so the K loop has no per-tile branches
//     except the wave-uniform test for the odd tile;
//   - the 256-row-wide weight tile halves the activation traffic per weight byte, and the tall
//     chunk (320 rows instead of 256: the 512 tokens of config 4 in 589 instead of 655 us) saves the
//     second pass over the weights for experts with 257-320 tokens; 384 rows fit too (all 256
//     registers, 160 KB of LDS) and are no faster;
//   - the two waves a SIMD hosts (one of each M group) share its matrix pipe, so an odd number of
//     row tiles does not unbalance the SIMDs;
//   SILU  : halves = W1 / W3 rows of ffn columns n0..n0+127; out = silu(A W1^T) * (A W3^T) in the
//           element type (bf16 rounded to nearest even, fp32 as computed)
//   !SILU : halves = weight rows n0..n0+127 / n0+128..n0+255; out = fp32 partial sums for K range
//           ksplit, [gridDim.z][rows, ldo]
// K is a multiple of 64.
// ---------------------------------------------------------------------------------------------
template <typename E>
__device__ __forceinline__ int lds_slot(int row, int piece) {
  return row * ElemT<E>::BKE + (piece ^ (row & 7)) * ElemT<E>::PIECE;
}

// s_waitcnt vmcnt(N) only (other counters left at their maximum).
#define ODMOE_VMCNT(N) __builtin_amdgcn_s_waitcnt(((N) & 0xF) | (((N) >> 4) << 14) | (0x7 << 4) | (0xF << 8))

typedef const __attribute__((address_space(1))) void* global_void_ptr;
typedef __attribute__((address_space(3))) void* lds_void_ptr;

struct GemmArgs {
  const void* A;              // activations [rows, lda]
  int lda;
  const int32_t* a_slot;      // sorted position -> token-slot (row of A = slot / slot_div), or null
  int slot_div;
  const void* const* table;   // expert base pointers
  int table_off;
  const void* expert_override;  // when set: the weights of every chunk of this launch (one expert)
  int tile_first;               // first chunk-list entry of this launch
  size_t b_off[2];            // element offsets of the matrices the two 128-row halves of the tile come from
  int b_row[2];               // first weight row of each half relative to n0
  const int32_t* tiles;
  const int32_t* n_tiles;
  void* out;
  int ldo, N, K, k_per_split;
  size_t split_stride;
};

template <typename E, bool SILU, int NT, int NSTAGE>
__device__ __forceinline__ void gemm_chunk(const GemmArgs& g, E* smem, int ntile, int ksplit, int e, int row_lo, int nrows) {
  constexpr int BKE = ElemT<E>::BKE, PIECE = ElemT<E>::PIECE;
  constexpr int A_INSTR = (NT + 1) / 2;                 // A fills per wave per K-step (64 rows each)
  constexpr int A_ROWS = 64 * A_INSTR;                  // rows of activations staged (NT 32-row tiles used)
  constexpr int MTW = (NT + 1) / 2;                     // 32-row tiles per wave: tiles wm, wm+2, wm+4, ...
  constexpr int B_INSTR = BN / 64;                      // B fills per wave per K-step
  constexpr int LPS = A_INSTR + B_INSTR;                // DMA loads per wave per K-step
  constexpr bool ODD_NT = (NT & 1) != 0;                // the last 64-row group is half used
  constexpr size_t A_STAGE = (size_t)A_ROWS * BKE;
  constexpr size_t STAGE = A_STAGE + (size_t)BN * BKE;
  static_assert(NSTAGE * STAGE * sizeof(E) <= GEMM_LDS, "ring does not fit");
  static_assert((NSTAGE - 2) * LPS < 64, "vmcnt is 6 bits");

  const int n0 = ntile * (SILU ? BN / 2 : BN);
  if (n0 >= g.N) return;                                // grid.x is padded to a multiple of 8
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 2, wn = wave & 3;
  const int K = g.K;
  const int k_begin = ksplit * g.k_per_split;
  const int k_end = (k_begin + g.k_per_split < K) ? k_begin + g.k_per_split : K;
  if (k_begin >= k_end) return;
  const int nk = (k_end - k_begin) / BKE;

  // ---- what this lane fetches: row (lane >> 3) of each 8-row group, piece (lane & 7) ^ (lane >> 3)
  const int sub = lane >> 3;
  const int piece = (lane & 7) ^ sub;
  const E* a_src[A_INSTR];
#pragma unroll
  for (int i = 0; i < A_INSTR; ++i) {
    int r = (i * 8 + wave) * 8 + sub;
    r = r < nrows ? r : nrows - 1;                      // rows past the chunk: repeat its last row
    const int p = row_lo + r;
    const int src_row = g.a_slot ? g.a_slot[p] / g.slot_div : p;
    a_src[i] = static_cast<const E*>(g.A) + (size_t)src_row * g.lda + k_begin + piece * PIECE;
  }
  const E* wbase =
      static_cast<const E*>(g.expert_override ? g.expert_override : g.table[g.table_off + e]);
  const E* b_src[B_INSTR];                         // LDS rows (i*8 + wave)*8 + sub of the B tile
#pragma unroll
  for (int i = 0; i < B_INSTR; ++i) {
    const int br = (i * 8 + wave) * 8 + sub;            // 0..255: half = br / 128, row in half = br % 128
    const int half = br >> 7;
    int n = n0 + g.b_row[half] + (br & 127);
    n = n < g.N ? n : g.N - 1;                          // rows past N: any valid row (never stored)
    b_src[i] = wbase + g.b_off[half] + (size_t)n * K + k_begin + piece * PIECE;
  }
  // Blocks that run side by side start their K loops at different steps: rows of a row-major
  // matrix lie a multiple of 4 KB apart, so blocks marching through K in lockstep would keep
  // hitting the same memory channels.
  const int kt0 = (int)(((unsigned)ntile * K_ROTATE + (unsigned)ksplit * 7u) % (unsigned)nk);
  auto step_offset = [&](int kt) {
    int kr = kt + kt0;
    kr = kr >= nk ? kr - nk : kr;
    return kr * BKE;
  };
  auto issue_a = [&](int stage, int kt) {
    E* sa = smem + stage * STAGE;
    const int ko = step_offset(kt);
#pragma unroll
    for (int i = 0; i < A_INSTR; ++i)
      if (i + 1 < A_INSTR || !ODD_NT || wave < 4)   // odd tile count: the last fill covers 32 rows only
        __builtin_amdgcn_global_load_lds((global_void_ptr)(a_src[i] + ko),
                                         (lds_void_ptr)(sa + (i * 8 + wave) * 8 * BKE), 16, 0, 0);
  };
  auto issue_b = [&](int stage, int kt) {
    E* sa = smem + stage * STAGE;
    const int ko = step_offset(kt);
#pragma unroll
    for (int i = 0; i < B_INSTR; ++i)   // weights pass through once: non-temporal (cache policy 2 = nt),
                                        // so they evict fewer of the activation lines other blocks reuse
      __builtin_amdgcn_global_load_lds((global_void_ptr)(b_src[i] + ko),
                                       (lds_void_ptr)(sa + A_STAGE + (i * 8 + wave) * 8 * BKE), 16, 0, 2);
  };
  // With a two-deep ring only one step is in flight: the weight fills (HBM) go out first and the
  // activation fills (L2 hits) half a step later, which spreads the requests over the step.
  constexpr bool SPLIT_ISSUE = NSTAGE == 2;

  f32x16 acc[MTW][2];
#pragma unroll
  for (int mt = 0; mt < MTW; ++mt)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[mt][b][i] = 0.f;

  const int fr = lane & 31, fg = lane >> 5;            // fragment row within a 32-tile, K half
  // With an odd tile count the second M group of waves has one tile fewer (wave-uniform test).
  auto tile_on = [&](int mt) { return 2 * mt + 1 < NT || wm == 0; };

  const int last = nk - 1;
#pragma unroll
  for (int st = 0; st < NSTAGE - 1; ++st) {   // weights first: their addresses do not wait for the row gather
    issue_b(st, st < last ? st : last);
    issue_a(st, st < last ? st : last);
  }
  int stage = 0, refill = NSTAGE - 1;
  for (int kt = 0; kt < nk; ++kt) {
    // this wave's fills of step kt have landed (those of later steps may still fly; with an odd
    // tile count waves 4..7 issue one fill fewer per step)
    if (ODD_NT && wave >= 4) ODMOE_VMCNT((NSTAGE - 2) * (LPS - 1));
    else ODMOE_VMCNT((NSTAGE - 2) * LPS);
    __builtin_amdgcn_s_barrier();      // ... and everybody else's; everybody is done with step kt-1
    const int nxt = kt + NSTAGE - 1 < last ? kt + NSTAGE - 1 : last;
    if (!SPLIT_ISSUE) issue_a(refill, nxt);            // refill the buffer that step kt-1 used
    issue_b(refill, nxt);
    {
      const E* sa = smem + stage * STAGE;
      const E* sb = sa + A_STAGE;
      // The 128-byte line of a row is 8 pieces of 16 bytes; lane group fg takes pieces fg, 2+fg, ...
      // bf16: a piece is the 8 consecutive K elements of one 32x32x16 MFMA operand.  fp32: a piece is
      // 4 consecutive K elements; MFMA j of a piece multiplies element j of the pieces of both lane
      // groups (K indices 8s+j and 8s+4+j), the same pairing for activations and weights.
      typedef typename std::conditional<sizeof(E) == 2, bf16x8, f32x4>::type frag_t;
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const int pc = 2 * s + fg;
        if (SPLIT_ISSUE && s == 2) issue_a(refill, nxt);
        frag_t bfrag[2], afrag[MTW];
#pragma unroll
        for (int b = 0; b < 2; ++b)
          bfrag[b] = *reinterpret_cast<const frag_t*>(sb + lds_slot<E>(b * 128 + wn * 32 + fr, pc));
#pragma unroll
        for (int mt = 0; mt < MTW; ++mt)
          if (tile_on(mt)) afrag[mt] = *reinterpret_cast<const frag_t*>(sa + lds_slot<E>((2 * mt + wm) * 32 + fr, pc));
#pragma unroll
        for (int mt = 0; mt < MTW; ++mt)
          if (tile_on(mt)) {
#pragma unroll
            for (int b = 0; b < 2; ++b) {
              if constexpr (sizeof(E) == 2) {
                acc[mt][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(afrag[mt], bfrag[b], acc[mt][b], 0, 0, 0);
              } else {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                  acc[mt][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(afrag[mt][j], bfrag[b][j], acc[mt][b], 0, 0, 0);
              }
            }
          }
      }
    }
    stage = stage + 1 == NSTAGE ? 0 : stage + 1;
    refill = refill + 1 == NSTAGE ? 0 : refill + 1;
  }
  ODMOE_VMCNT(0);  // no fill may still be on its way into LDS when the block retires

  // ---- epilogue.  Accumulator layout: column = lane % 32, row = (i/4)*8 + (lane/32)*4 + i%4.
#pragma unroll
  for (int mt = 0; mt < MTW; ++mt) {
    if (!tile_on(mt)) continue;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int m = (2 * mt + wm) * 32 + (i >> 2) * 8 + fg * 4 + (i & 3);
      if (m < nrows) {
        const size_t p = (size_t)(row_lo + m);
        if constexpr (SILU) {
          const int col = n0 + wn * 32 + fr;
          if (col < g.N) {
            const float a = acc[mt][0][i], b = acc[mt][1][i];
            const float hval = a / (1.f + expf(-a)) * b;
            if constexpr (sizeof(E) == 2)
              ((__attribute__((address_space(1))) bf16_t*)g.out)[p * g.ldo + col] = f32_to_bf16(hval);
            else
              ((__attribute__((address_space(1))) float*)g.out)[p * g.ldo + col] = hval;
          }
        } else {
#pragma unroll
          for (int b = 0; b < 2; ++b) {
            const int col = n0 + b * 128 + wn * 32 + fr;
            if (col < g.N)
              ((__attribute__((address_space(1))) float*)g.out)[ksplit * g.split_stride + p * g.ldo + col] =
                  acc[mt][b][i];
          }
        }
      }
    }
  }
}

template <typename E, bool SILU>
__global__ __launch_bounds__(GEMM_THREADS) void grouped_gemm_kernel(GemmArgs g) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  E* smem = reinterpret_cast<E*>(smem_raw);
  // Blocks are dispatched in the order x + gridDim.x * (y + gridDim.y * z), round-robin over the
  // 8 XCDs.  That order is re-read as [y][x][K split]: with 8 K splits every XCD works on one K
  // range, so the blocks that read the same activation columns (all N tiles of a chunk) and the
  // same weight tile (the chunks of an expert) share one L2.
  const unsigned lin = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
  const int ksplit = (int)(lin % gridDim.z);
  const int bx = (int)((lin / gridDim.z) % gridDim.x), by = (int)(lin / gridDim.z / gridDim.x);
  const int slot = g.tile_first + by;
  if (slot >= *g.n_tiles) return;
  // Chunks of one expert read the same weights.  Within the expert's blocks (dispatched in the
  // order x + gridDim.x * y) the order is made [group of 8 N tiles][chunk][N tile in the group]:
  // the blocks that share an N tile start together, 8 block ids apart (same XCD), so the weight
  // lines one of them brings into that XCD's L2 are still there for the others.
  // (One record read gives everything when the expert has a single chunk, the usual case: the
  // weight fills then start two dependent loads after the block does: record, expert pointer.)
  const int32_t* rec = g.tiles + TILE_REC * slot;
  int e = rec[0], row_lo = rec[1], nrows = rec[2];
  const int first = rec[3], nsib = rec[4];
  int ntile = bx;
  if (nsib > 1) {
    const int lg = bx + (int)gridDim.x * (slot - first);
    const int rem = lg % (8 * nsib);
    ntile = lg / (8 * nsib) * 8 + (rem & 7);
    rec = g.tiles + TILE_REC * (first + (rem >> 3));
    e = rec[0]; row_lo = rec[1]; nrows = rec[2];
  }
  switch ((nrows + 31) >> 5) {      // 32-row tiles of the chunk
    case 1: gemm_chunk<E, SILU, 1, 3>(g, smem, ntile, ksplit, e, row_lo, nrows); break;
    case 2: gemm_chunk<E, SILU, 2, 3>(g, smem, ntile, ksplit, e, row_lo, nrows); break;
    case 3: gemm_chunk<E, SILU, 3, 3>(g, smem, ntile, ksplit, e, row_lo, nrows); break;
    case 4: gemm_chunk<E, SILU, 4, 3>(g, smem, ntile, ksplit, e, row_lo, nrows); break;
    case 5: gemm_chunk<E, SILU, 5, 2>(g, smem, ntile, ksplit, e, row_lo, nrows); break;
    case 6: gemm_chunk<E, SILU, 6, 2>(g, smem, ntile, ksplit, e, row_lo, nrows); break;
    case 7: gemm_chunk<E, SILU, 7, 2>(g, smem, ntile, ksplit, e, row_lo, nrows); break;
    case 8: gemm_chunk<E, SILU, 8, 2>(g, smem, ntile, ksplit, e, row_lo, nrows); break;
    case 9: gemm_chunk<E, SILU, 9, 2>(g, smem, ntile, ksplit, e, row_lo, nrows); break;
    default: gemm_chunk<E, SILU, 10, 2>(g, smem, ntile, ksplit, e, row_lo, nrows); break;
  }
}

// Y[t, :] = sum_i gate[t,i] * (sum_z Ybuf[z][inv[t*k+i], :]), rounded once to the layer's dtype.  Block (t, j)
// takes columns j*1024 .. j*1024+1023 of token t, four per thread; the partial sums of one slot are
// fetched together (independent loads) and added in a fixed order (z inner, i outer).
template <typename E>
__global__ __launch_bounds__(256) void combine_kernel(const float* __restrict__ ybuf,
                                                       const int32_t* __restrict__ inv,
                                                       const float* __restrict__ gate,
                                                       E* __restrict__ Y, int H, int k, int n_split,
                                                       size_t split_stride) {
  const int t = blockIdx.x;
  const int c = (blockIdx.y * 256 + threadIdx.x) * 4;
  if (c >= H) return;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  for (int i = 0; i < k; ++i) {
    const int p = inv[t * k + i];
    if (p < 0) continue;
    const float* src = ybuf + (size_t)p * H + c;
    f32x4 w[MAX_KSPLIT];
#pragma unroll
    for (int z = 0; z < MAX_KSPLIT; ++z)
      if (z < n_split) w[z] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(src + z * split_stride));
    f32x4 v = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int z = 0; z < MAX_KSPLIT; ++z)
      if (z < n_split) { v.x += w[z].x; v.y += w[z].y; v.z += w[z].z; v.w += w[z].w; }
    const float g = gate[t * k + i];
    acc.x = fmaf(g, v.x, acc.x); acc.y = fmaf(g, v.y, acc.y);
    acc.z = fmaf(g, v.z, acc.z); acc.w = fmaf(g, v.w, acc.w);
  }
  if constexpr (sizeof(E) == 2) {
    const uint32_t lo = (uint32_t)f32_to_bf16(acc.x) | ((uint32_t)f32_to_bf16(acc.y) << 16);
    const uint32_t hi = (uint32_t)f32_to_bf16(acc.z) | ((uint32_t)f32_to_bf16(acc.w) << 16);
    *reinterpret_cast<uint2*>(Y + (size_t)t * H + c) = make_uint2(lo, hi);
  } else {
    *reinterpret_cast<f32x4*>(Y + (size_t)t * H + c) = acc;
  }
}

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct Carve {
  int32_t *offsets, *perm, *inv, *tiles, *n_tiles;
  void* hbuf;
  float* ybuf;
  size_t total;
};

void w2_split(const Shape& sh, int32_t T, int* n_split, int* k_per_split);

Carve carve(const Shape& sh, int32_t T, void* base) {
  const size_t n = (size_t)T * sh.k;
  const size_t max_tiles = (size_t)sh.E + (n + BMX - 1) / BMX;
  char* p = static_cast<char*>(base);
  size_t off = 0;
  Carve c{};
  auto take = [&](size_t bytes) { char* q = p ? p + off : nullptr; off = align_up(off + bytes, 256); return q; };
  c.offsets = reinterpret_cast<int32_t*>(take((sh.E + 1) * sizeof(int32_t)));
  c.perm = reinterpret_cast<int32_t*>(take(n * sizeof(int32_t)));
  c.inv = reinterpret_cast<int32_t*>(take(n * sizeof(int32_t)));
  c.tiles = reinterpret_cast<int32_t*>(take(TILE_REC * max_tiles * sizeof(int32_t)));
  c.n_tiles = reinterpret_cast<int32_t*>(take(sizeof(int32_t)));
  c.hbuf = take(n * sh.F * (sh.dtype == ODMOE_F32 ? sizeof(float) : sizeof(bf16_t)));
  int n_split = 1, k_per_split = 0;
  w2_split(sh, T, &n_split, &k_per_split);
  c.ybuf = reinterpret_cast<float*>(take((size_t)n_split * n * sh.H * sizeof(float)));
  c.total = off;
  return c;
}

}  // namespace

bool prefill_supported(const Shape& sh) {
  return (sh.dtype == ODMOE_BF16 || sh.dtype == ODMOE_F32) && sh.H % 64 == 0 && sh.F % 64 == 0;
}

size_t prefill_workspace_bytes(const Shape& sh, int32_t T) { return carve(sh, T, nullptr).total; }

void prefill_expert_order(const int32_t* count, int32_t E, int32_t* order) {
  const int half = (E + 1) / 2;
  for (int e = 0; e < E; ++e) {
    int rank = 0;
    for (int j = 0; j < E; ++j) rank += (count[j] > count[e]) || (count[j] == count[e] && j < e);
    order[rank < half ? 2 * rank : 2 * (rank - half) + 1] = e;
  }
}

int prefill_chunks_of(int32_t count) {
  if (count <= 0) return 0;
  return (count + BMX - 1) / BMX;
}

namespace {

hipError_t ensure_attrs() {
  static bool attr_set = false;
  if (attr_set) return hipSuccess;
  const void* kernels[4] = {reinterpret_cast<const void*>(grouped_gemm_kernel<bf16_t, true>),
                            reinterpret_cast<const void*>(grouped_gemm_kernel<bf16_t, false>),
                            reinterpret_cast<const void*>(grouped_gemm_kernel<float, true>),
                            reinterpret_cast<const void*>(grouped_gemm_kernel<float, false>)};
  for (const void* fn : kernels) {
    const hipError_t ea = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)GEMM_LDS);
    if (ea != hipSuccess) return ea;
  }
  attr_set = true;
  return hipSuccess;
}

// K split of the w2 GEMM: few output tiles but a long K, so K is cut until the grid has about two
// blocks per CU, counting one chunk per expert that can have tokens (every split writes and the
// combine re-reads a full fp32 copy of the output, so no finer than that, and at least 8 K-steps
// per block).  A function of the shape and the token count only: the GEMM and the combine agree.
void w2_split(const Shape& sh, int32_t T, int* n_split, int* k_per_split) {
  const int nt2 = (sh.H + BN - 1) / BN;
  const int bk = sh.dtype == ODMOE_F32 ? ElemT<float>::BKE : ElemT<bf16_t>::BKE;
  const int ksteps = sh.F / bk;
  const long slots = (long)T * sh.k;
  const long chunks = slots < sh.E ? slots : sh.E;
  long ns = (2 * 256 + nt2 * chunks - 1) / (nt2 * chunks);
  if (ns > MAX_KSPLIT) ns = MAX_KSPLIT;
  if (ns > ksteps / 8) ns = ksteps / 8;
  if (ns < 1) ns = 1;
  *k_per_split = (int)((ksteps + ns - 1) / ns) * bk;
  *n_split = (sh.F + *k_per_split - 1) / *k_per_split;
}

}  // namespace

hipError_t prefill_sort(hipStream_t s, const Shape& sh, const int32_t* idx, int32_t T, void* workspace,
                        size_t workspace_bytes) {
  if (!prefill_supported(sh)) return hipErrorNotSupported;
  const Carve c = carve(sh, T, workspace);
  if (!workspace || c.total > workspace_bytes) return hipErrorInvalidValue;
  hipError_t e = ensure_attrs();
  if (e != hipSuccess) return e;
  sort_slots_kernel<<<1, 1024, 0, s>>>(idx, T * sh.k, sh.E, c.offsets, c.perm, c.inv, c.tiles, c.n_tiles);
  return hipGetLastError();
}

hipError_t prefill_gemms(hipStream_t s, const Shape& sh, const void* const* table, int32_t table_off,
                         const void* expert_override, int32_t tile_first, int32_t tile_count,
                         const void* x, int32_t T, void* workspace) {
  if (tile_count <= 0) return hipSuccess;
  if (tile_count > 65535) return hipErrorInvalidValue;  // grid.y
  const Carve c = carve(sh, T, workspace);
  const int n = T * sh.k;
  const size_t hf = (size_t)sh.H * sh.F;

  GemmArgs g1{};
  g1.A = x; g1.lda = sh.H; g1.a_slot = c.perm; g1.slot_div = sh.k;
  g1.table = table; g1.table_off = table_off; g1.expert_override = expert_override; g1.tile_first = tile_first;
  g1.b_off[0] = 0; g1.b_off[1] = hf; g1.b_row[0] = 0; g1.b_row[1] = 0;        // W1 and W3 rows n0..n0+127
  g1.tiles = c.tiles; g1.n_tiles = c.n_tiles;
  g1.out = c.hbuf; g1.ldo = sh.F; g1.N = sh.F; g1.K = sh.H; g1.k_per_split = sh.H; g1.split_stride = 0;
  // x = N tile (fastest; padded to a multiple of the 8 XCDs so that the chunks of one expert that
  // share an N tile land on the same XCD and its L2), y = chunk, z = K split.
  auto pad8 = [](int v) { return (v + 7) & ~7; };
  dim3 grid1(pad8((sh.F + BN / 2 - 1) / (BN / 2)), tile_count, 1);
  if (sh.dtype == ODMOE_F32) grouped_gemm_kernel<float, true><<<grid1, GEMM_THREADS, GEMM_LDS, s>>>(g1);
  else grouped_gemm_kernel<bf16_t, true><<<grid1, GEMM_THREADS, GEMM_LDS, s>>>(g1);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;

  int n_split, k_per_split;
  w2_split(sh, T, &n_split, &k_per_split);
  GemmArgs g2{};
  g2.A = c.hbuf; g2.lda = sh.F; g2.a_slot = nullptr; g2.slot_div = 1;
  g2.table = table; g2.table_off = table_off; g2.expert_override = expert_override; g2.tile_first = tile_first;
  g2.b_off[0] = 2 * hf; g2.b_off[1] = 2 * hf; g2.b_row[0] = 0; g2.b_row[1] = 128;  // W2 rows n0..n0+255
  g2.tiles = c.tiles; g2.n_tiles = c.n_tiles;
  g2.out = c.ybuf; g2.ldo = sh.H; g2.N = sh.H; g2.K = sh.F; g2.k_per_split = k_per_split;
  g2.split_stride = (size_t)n * sh.H;
  dim3 grid2(pad8((sh.H + BN - 1) / BN), tile_count, n_split);
  if (sh.dtype == ODMOE_F32) grouped_gemm_kernel<float, false><<<grid2, GEMM_THREADS, GEMM_LDS, s>>>(g2);
  else grouped_gemm_kernel<bf16_t, false><<<grid2, GEMM_THREADS, GEMM_LDS, s>>>(g2);
  return hipGetLastError();
}

hipError_t prefill_combine(hipStream_t s, const Shape& sh, const float* gate, int32_t T, void* y,
                           void* workspace) {
  const Carve c = carve(sh, T, workspace);
  int n_split, k_per_split;
  w2_split(sh, T, &n_split, &k_per_split);
  const dim3 grid(T, (sh.H + 1023) / 1024);
  const size_t stride = (size_t)T * sh.k * sh.H;
  if (sh.dtype == ODMOE_F32)
    combine_kernel<float><<<grid, 256, 0, s>>>(c.ybuf, c.inv, gate, static_cast<float*>(y), sh.H, sh.k, n_split, stride);
  else
    combine_kernel<bf16_t><<<grid, 256, 0, s>>>(c.ybuf, c.inv, gate, static_cast<bf16_t*>(y), sh.H, sh.k, n_split, stride);
  return hipGetLastError();
}

hipError_t launch_prefill(hipStream_t s, const Shape& sh, const void* const* table, int32_t table_off,
                          const int32_t* idx, const float* gate, const void* x, int32_t T, void* y,
                          void* workspace, size_t workspace_bytes) {
  if (T <= 0) return hipSuccess;
  hipError_t e = prefill_sort(s, sh, idx, T, workspace, workspace_bytes);
  if (e != hipSuccess) return e;
  const int max_tiles = sh.E + (T * sh.k + BMX - 1) / BMX;
  e = prefill_gemms(s, sh, table, table_off, nullptr, 0, max_tiles, x, T, workspace);
  if (e != hipSuccess) return e;
  return prefill_combine(s, sh, gate, T, y, workspace);
}

}  // namespace odmoe
