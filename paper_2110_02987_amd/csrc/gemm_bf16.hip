// Dense contractions of the GCN step for bfloat16 storage on the gfx950 matrix cores
// (v_mfma_f32_32x32x16_bf16: bfloat16 operands, float32 accumulation):
//   NT:  C[M x N] = A[M x K] Bt[N x K]^T       -- the feature transform H W of Eq. 7 (Bt = W^T rounded to
//                                                  bfloat16) and the input-gradient product S W^T (Bt = W)
//   TN:  P[slab][K x N] = A[rows of slab]^T G  -- the weight gradient dW = (A~ H)^T G, a reduction over the
//                                                  nodes, split into slabs that are added in slab order.
// (arXiv 2110.02987, Section 3.3: Eq. 7 forward; backward step of Algorithm 2.)
//
// One MFMA consumes, per lane, 8 consecutive elements of the contraction index for one row of the left
// operand and one column of the right operand.  Both operand tiles therefore sit in LDS with the contraction
// index contiguous (16-byte fragment reads, row stride 144 bytes: conflict free).  For NT that is the layout
// the operands already have in memory.  For TN the contraction index is the row index of both A and G, so
// each thread fetches an 8 x 8 block (eight 16-byte row pieces), transposes it in registers with byte
// permutes, and writes eight 16-byte column pieces; the 16-byte chunks of a tile row are XOR-swizzled so that
// these writes are conflict free as well.  Because the same order of the contraction index is used for both
// operands, the result does not depend on which 8 indices a lane holds.
//
// Three kernels.  gemm_nt_kernel (outputs below 256 columns, and any shape whose rows are not 16-byte aligned or
// whose K is not a multiple of 32) and gemm_tn_kernel: four wave64s per block in a 2 x 2 arrangement, a wave owns
// TM x TN accumulators of 32 x 32; the next tile (NT) or two tiles (TN) are on their way from global memory into
// registers while the current one is multiplied (double-buffered LDS, one barrier per tile).  gemm_nt_dma_kernel
// (outputs of 256 columns or more): 256 x 256 blocks of eight waves whose operand tiles go from global memory
// straight into LDS, all tiles but the one being multiplied in flight.  Blocks are renumbered so that the blocks
// sharing an operand tile run on the same XCD (consecutive workgroup ids go to different XCDs, each with an L2 of
// its own).
#include <stdlib.h>

#include <atomic>

#include "dtype.h"
#include "gad_internal.h"
#include "xcd.h"

namespace gad {
namespace {

// Operand tiles a block keeps in flight between global memory and LDS.  The TN kernel gains from two (the weight
// gradient of 4.2 M x 512 x 64: 2.09 -> 0.93 ms; there is room for two tiles of 32 registers next to the 8 x 8
// transposes).  The NT kernels were measured at one, two and three tiles in flight and are fastest with one.
constexpr int kTnDepth = 2;
template <int TN>
constexpr int nt_depth() { return 1; }

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

// Row of accumulator register r of a 32x32 MFMA result held by `lane` (its column is lane % 32).
__device__ __forceinline__ int acc_row(int r, int lane) { return 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3); }

// 8 consecutive bfloat16 of row `row` from column `col`, zero outside [0, n_rows) x [0, n_cols).
__device__ __forceinline__ uint4 load_piece(const bf16_t* __restrict__ base, int64_t ld, int64_t row, int64_t n_rows,
                                            int col, int n_cols, bool vec_ok) {
  uint4 v = make_uint4(0u, 0u, 0u, 0u);
  if (row < n_rows) {
    const bf16_t* p = base + row * ld + col;
    if (vec_ok && col + 8 <= n_cols) {
      v = *reinterpret_cast<const uint4*>(p);
    } else {
      uint32_t e[8];
#pragma unroll
      for (int q = 0; q < 8; ++q) e[q] = col + q < n_cols ? (uint32_t)p[q] : 0u;
      v.x = e[0] | (e[1] << 16);
      v.y = e[2] | (e[3] << 16);
      v.z = e[4] | (e[5] << 16);
      v.w = e[6] | (e[7] << 16);
    }
  }
  return v;
}

// v when ok, zeros otherwise (by value: selecting between two lvalues would force them into memory)
__device__ __forceinline__ uint4 keep_if(bool ok, uint4 v) {
  return make_uint4(ok ? v.x : 0u, ok ? v.y : 0u, ok ? v.z : 0u, ok ? v.w : 0u);
}

// The first n_valid (any integer; 8 or more keeps all) of the 8 bfloat16 in v, zeros in the others.
__device__ __forceinline__ uint32_t keep_pair(uint32_t w, int n_valid) {
  return n_valid >= 2 ? w : (n_valid == 1 ? (w & 0xFFFFu) : 0u);
}
__device__ __forceinline__ uint4 keep_first(uint4 v, int n_valid) {
  return make_uint4(keep_pair(v.x, n_valid), keep_pair(v.y, n_valid - 2), keep_pair(v.z, n_valid - 4),
                    keep_pair(v.w, n_valid - 6));
}

// Tile layouts in LDS (rows of BK contraction indices, 16-byte chunks of 8):
//   kPadded   row stride BK + 8 elements, chunks in place (64-deep tiles: 144-byte stride, conflict free);
//   kSwzTn    the same stride, chunk c of row r at position c ^ ((r >> 4) & 7) (the transposing writes of the TN tile);
//   kSwz32    32-deep tiles without padding (64-byte rows), chunk c of row r at position c ^ ((r >> 2) & 3): the
//             16-byte reads of 16 consecutive rows and the staging writes of 4 consecutive rows each cover 16
//             different 16-byte slots of a 256-byte window (the padded 80-byte stride made the writes collide).
enum Layout : int { kPadded = 0, kSwzTn = 1, kSwz32 = 2, kSwz64 = 3 };   // kSwz64: unpadded 128-byte rows, chunk ^ (row & 7)
template <int BK, int MODE>
constexpr int tile_ld() { return MODE == kSwz32 || MODE == kSwz64 ? BK : BK + 8; }

// Offset (in elements) of 16-byte chunk `chunk` of tile row `row`; LDK = row stride.
template <int LDK, int MODE>
__device__ __forceinline__ int tile_off(int row, int chunk) {
  const int c = MODE == kSwzTn ? (chunk ^ ((row >> 4) & 7)) : MODE == kSwz32 ? (chunk ^ ((row >> 2) & 3))
                : MODE == kSwz64 ? (chunk ^ (row & 7)) : chunk;
  return row * LDK + (c << 3);
}

// acc[tm][tn] += L[wrow + 32 tm .., :] R[wcol + 32 tn .., :]^T over the BK contraction indices of one tile.
template <int BK, int TM, int TN, int MODE>
__device__ __forceinline__ void mma_tile(const bf16_t* __restrict__ Ls, const bf16_t* __restrict__ Rs, int wrow,
                                         int wcol, v16f (&acc)[TM][TN]) {
  constexpr int LDK = tile_ld<BK, MODE>();
  const int lane = threadIdx.x & 63;
  const int i = lane & 31, kg = lane >> 5;
#pragma unroll
  for (int ks = 0; ks < BK / 16; ++ks) {
    const int chunk = ks * 2 + kg;
    bf16x8 a[TM], b[TN];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
      a[tm] = *reinterpret_cast<const bf16x8*>(Ls + tile_off<LDK, MODE>(wrow + tm * 32 + i, chunk));
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
      b[tn] = *reinterpret_cast<const bf16x8*>(Rs + tile_off<LDK, MODE>(wcol + tn * 32 + i, chunk));
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
      for (int tn = 0; tn < TN; ++tn)
        acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[tm], b[tn], acc[tm][tn], 0, 0, 0);
  }
}

template <int TM, int TN>
__device__ __forceinline__ void zero_acc(v16f (&acc)[TM][TN]) {
#pragma unroll
  for (int x = 0; x < TM; ++x)
#pragma unroll
    for (int y = 0; y < TN; ++y)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[x][y][r] = 0.f;
}

template <int EPI, int TM, int TN, typename TC>
__device__ __forceinline__ void store_acc(const v16f (&acc)[TM][TN], TC* __restrict__ C, int64_t ldc, int64_t row0,
                                          int col0, int64_t M, int N, float slope, const bf16_t* __restrict__ aux,
                                          int64_t ldaux) {
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int tm = 0; tm < TM; ++tm)
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
      const int col = col0 + tn * 32 + (lane & 31);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int64_t row = row0 + tm * 32 + acc_row(r, lane);
        if (row < M && col < N) {
          float v = acc[tm][tn][r];
          if (EPI == EPI_RELU) v = leaky(v, v > 0.f, slope);
          if (EPI == EPI_MASK) v = leaky(v, bf16_to_float(aux[row * ldaux + col]) > 0.f, slope);
          C[row * ldc + col] = from_f32<TC>(v);
        }
      }
    }
}

// Epilogue of the NT kernel.  A lane's accumulator values sit in one column, so writing them directly gives
// 64-byte row pieces (bfloat16).  Each wave instead passes its 32 x (32 TN) accumulator blocks through its own
// region of LDS and writes whole row pieces with 16-byte stores; the mask operand is read the same way.
// Must be entered by all waves of the block, after the last read of the operand tiles: one block-wide barrier
// separates those reads from the staging writes.  After it a wave touches only its own region, and the LDS
// operations of one wave complete in order, so the passes need no further barrier.
template <int EPI, int TM, int TN, typename TC>
__device__ __forceinline__ void store_rows(const v16f (&acc)[TM][TN], float* __restrict__ lds, TC* __restrict__ C,
                                           int64_t ldc, int64_t row0, int col0, int64_t M, int N, bool c_vec,
                                           float slope, const bf16_t* __restrict__ aux, int64_t ldaux, bool aux_vec) {
  constexpr int W = 32 * TN;          // columns of the wave's block
  constexpr int LD = W + 8;           // row stride in floats: rows 4 apart fall on the other half of the banks
  constexpr int E = 16 / (int)sizeof(TC);    // elements per 16-byte store
  constexpr int CH = W / E;           // 16-byte pieces per row
  const int lane = threadIdx.x & 63;
  float* mine = lds + (threadIdx.x >> 6) * (32 * LD);
  __syncthreads();
#pragma unroll
  for (int tm = 0; tm < TM; ++tm) {
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
      for (int r = 0; r < 16; ++r) mine[acc_row(r, lane) * LD + tn * 32 + (lane & 31)] = acc[tm][tn][r];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");     // keeps the compiler from moving the reads above the writes
    __builtin_amdgcn_wave_barrier();
    static_assert((32 * CH) % 64 == 0, "whole wave passes");
#pragma unroll
    for (int it = 0; it < 32 * CH / 64; ++it) {
      const int p = lane + 64 * it;
      const int rl = p / CH, cl = (p % CH) * E;
      const int64_t row = row0 + tm * 32 + rl;
      const int col = col0 + cl;
      if (row >= M || col >= N) continue;
      float v[E];
#pragma unroll
      for (int q = 0; q < E; ++q) v[q] = mine[rl * LD + cl + q];
      const bool full = col + E <= N;
      if (EPI == EPI_RELU) {
#pragma unroll
        for (int q = 0; q < E; ++q) v[q] = leaky(v[q], v[q] > 0.f, slope);
      }
      if (EPI == EPI_MASK) {
        const bf16_t* ap = aux + row * ldaux + col;
        float m[E];
        if (full && aux_vec && E == 8) {
          load_row_piece<8, bf16_t>(ap, reinterpret_cast<float(&)[8]>(m));
        } else {
#pragma unroll
          for (int q = 0; q < E; ++q) m[q] = col + q < N ? bf16_to_float(ap[q]) : 0.f;
        }
#pragma unroll
        for (int q = 0; q < E; ++q) v[q] = leaky(v[q], m[q] > 0.f, slope);
      }
      TC* cp = C + row * ldc + col;
      if (full && c_vec) {
        if constexpr (sizeof(TC) == 2) {
          uint4 o;
          o.x = (uint32_t)float_to_bf16(v[0]) | ((uint32_t)float_to_bf16(v[1]) << 16);
          o.y = (uint32_t)float_to_bf16(v[2]) | ((uint32_t)float_to_bf16(v[3]) << 16);
          o.z = (uint32_t)float_to_bf16(v[4]) | ((uint32_t)float_to_bf16(v[5]) << 16);
          o.w = (uint32_t)float_to_bf16(v[6]) | ((uint32_t)float_to_bf16(v[7]) << 16);
          *reinterpret_cast<uint4*>(cp) = o;
        } else {
          *reinterpret_cast<float4*>(cp) = make_float4(v[0], v[1], v[2], v[3]);
        }
      } else {
#pragma unroll
        for (int q = 0; q < E; ++q)
          if (col + q < N) cp[q] = from_f32<TC>(v[q]);
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");     // the next pass writes what this one read
    __builtin_amdgcn_wave_barrier();
  }
}

// ---- NT ----------------------------------------------------------------------------------------
// WM x WN waves per block, each owning TM x TN accumulator blocks of 32 x 32: block tile BM x BN =
// (32 WM TM) x (32 WN TN).  Work item = (row tile, column tile) with the column tile fastest, so the blocks
// that share a row tile of A follow each other on one XCD.  Bt has ldb = K rounded up to BK, zero filled.
// Used with 2 x 2 waves of 64 x (32 TN): two or three blocks per CU.  (A 256 x 256 block of 2 x 4 waves on this
// kernel was measured, too: not faster than 128 x 256; the wide outputs have a kernel of their own below.)
// FAST: A may be fetched in aligned 16-byte pieces (16-byte aligned rows; a piece that straddles column K reads
// padding inside the row, which the caller must have declared readable).  Its loads are unconditional (a piece outside the matrix is fetched from the matrix's
// first bytes; what lies outside is zeroed when the piece is staged), so the compiler can count the loads in
// flight and wait only for the oldest tile; the general path waits for all of them.
template <int BK, int WM, int WN, int TM, int TN, int EPI, typename TC, bool FAST>
__global__ __launch_bounds__(64 * WM * WN, WM * WN == 4 ? 2 : 1) void gemm_nt_kernel(
    const bf16_t* __restrict__ A, int64_t lda, const bf16_t* __restrict__ Bt, int64_t ldb, TC* __restrict__ C,
    int64_t ldc, int64_t M, int N, int K, bool a_vec, bool c_vec, float slope, const bf16_t* __restrict__ aux,
    int64_t ldaux, bool aux_vec, int tiles_n, int64_t total) {
  constexpr int MODE = BK == 32 ? kSwz32 : kPadded;
  constexpr int NT = 64 * WM * WN;                           // threads per block
  constexpr int BM = 32 * WM * TM, BN = 32 * WN * TN, LDK = tile_ld<BK, MODE>(), CH = BK / 8;
  constexpr int PA = BM * CH / NT, PB = BN * CH / NT;        // 16-byte pieces per thread and tile
  static_assert(BM * CH % NT == 0 && BN * CH % NT == 0, "whole pieces per thread");
  constexpr int TILE = (BM + BN) * LDK;
  extern __shared__ __align__(16) unsigned char smem_raw[];
  bf16_t* smem = reinterpret_cast<bf16_t*>(smem_raw);        // [2][TILE]: rows 0..BM-1 = A, then BN rows of Bt
  const int t = threadIdx.x, w = t >> 6, wm = w / WN, wn = w % WN;
  const int64_t item = xcd_order(blockIdx.x, total);
  const int64_t row0 = (item / tiles_n) * BM;
  const int col0 = (int)(item % tiles_n) * BN;
  v16f acc[TM][TN];
  zero_acc<TM, TN>(acc);

  constexpr int kDepth = nt_depth<TN>();
  // kDepth tiles are in flight in registers (tile j in slot j % kDepth).
  uint4 ra[kDepth][PA], rb[kDepth][PB];
  auto fetch = [&](uint4 (&a)[PA], uint4 (&b)[PB], int k1) {
#pragma unroll
    for (int j = 0; j < PA; ++j) {
      const int p = t + NT * j;
      const int64_t row = row0 + p / CH;
      const int col = k1 + (p % CH) * 8;
      if (FAST) {
        const bool ok = row < M && col < K;
        a[j] = *reinterpret_cast<const uint4*>(A + (ok ? row * lda + col : 0));
      } else {
        a[j] = load_piece(A, lda, row, M, col, K, a_vec);
      }
    }
#pragma unroll
    for (int j = 0; j < PB; ++j) {                     // Bt is zero padded to whole tiles along k: inside for k1 < K
      const int p = t + NT * j;
      const int r = col0 + p / CH;
      b[j] = *reinterpret_cast<const uint4*>(Bt + (r < N && k1 < K ? (int64_t)r * ldb + k1 + (p % CH) * 8 : 0));
    }
  };
  auto stage = [&](const uint4 (&a)[PA], const uint4 (&b)[PB], bf16_t* tile, int k1) {
#pragma unroll
    for (int j = 0; j < PA; ++j) {
      const int p = t + NT * j;
      const int n_valid = !FAST ? 8 : (row0 + p / CH < M ? K - (k1 + (p % CH) * 8) : 0);
      *reinterpret_cast<uint4*>(tile + tile_off<LDK, MODE>(p / CH, p % CH)) = keep_first(a[j], n_valid);
    }
#pragma unroll
    for (int j = 0; j < PB; ++j) {
      const int p = t + NT * j;
      *reinterpret_cast<uint4*>(tile + BM * LDK + tile_off<LDK, MODE>(p / CH, p % CH)) = keep_if(col0 + p / CH < N, b[j]);
    }
  };
  // The pipeline is free of conditions (fetches past the last tile read the matrix's first bytes, stages past it
  // write a tile nobody reads), so the loads in flight at every wait are known when the kernel is compiled.
  const int n_kt = (K + BK - 1) / BK;
#pragma unroll
  for (int d = 0; d < kDepth; ++d) fetch(ra[d], rb[d], d * BK);
  stage(ra[0], rb[0], smem, 0);
  fetch(ra[0], rb[0], kDepth * BK);
  __syncthreads();
  for (int kt0 = 0; kt0 < n_kt; kt0 += kDepth) {
    bool done = false;
#pragma unroll
    for (int d = 0; d < kDepth; ++d) {
      const int kt = kt0 + d;
      bf16_t* cur = smem + (kt & 1) * TILE;
      bf16_t* nxt = smem + ((kt & 1) ^ 1) * TILE;
      mma_tile<BK, TM, TN, MODE>(cur, cur + BM * LDK, wm * 32 * TM, wn * 32 * TN, acc);
      const int slot = (d + 1) % kDepth;                     // tile kt + 1
      stage(ra[slot], rb[slot], nxt, (kt + 1) * BK);
      fetch(ra[slot], rb[slot], (kt + 1 + kDepth) * BK);
      __syncthreads();
      if (kt + 1 >= n_kt) {                                  // the same for every thread of the block
        done = true;
        break;
      }
    }
    if (done) break;
  }
  store_rows<EPI, TM, TN, TC>(acc, reinterpret_cast<float*>(smem_raw), C, ldc, row0 + wm * 32 * TM, col0 + wn * 32 * TN,
                              M, N, c_vec, slope, aux, ldaux, aux_vec);
}

// ---- NT, wide outputs: operand tiles straight from global memory into LDS ------------------------------------
// The tiles are filled by global_load_lds_dwordx4: a wave instruction moves 64 16-byte pieces from 64 global
// addresses into 1 KB of LDS (the piece of lane l lands at byte 16 l of the region), without passing through
// registers.  A 1 KB region holds 16 tile rows of a 32-deep tile (64-byte rows, layout kSwz32) or 8 rows of a
// 64-deep tile (128-byte rows, whole cache lines, layout kSwz64); the swizzle is applied to the address a lane
// fetches from: the slot at position pos of a row holds chunk pos ^ ((row >> 2) & 3), or pos ^ (row & 7).
// A tile is (BM + BN) / 16 (or / 8) regions, the A part first; wave w moves regions w, w + NW, .. of each part.
// kDmaStages tiles live in LDS; all but one are in flight while one is multiplied: at the top of step kt a wave
// waits until at most stages - 2 tiles' worth of its own loads are outstanding -- tile kt has landed -- then the
// block barrier makes every wave's share of tile kt visible and shows that everyone is done with tile kt - 1,
// whose memory the tile requested next overwrites.  The compiler does not order LDS reads behind these loads; the
// explicit wait counts do.  Steps past the last tile fetch tile 0 again into memory nobody reads, so every step
// issues the same number of loads.
// Conditions (checked by the launcher): K a whole number of 16-byte chunks, 16-byte aligned rows of A and Bt, N >= 256.
// Rows of A past M and rows of Bt past N are fetched from the last valid row; their products land in
// accumulators that the epilogue does not store.  K need not be a whole number of tiles: Bt is zero filled up to
// whole tiles, and a lane whose chunk of A lies past column K fetches the row's first chunk instead (finite data
// times zero).
// Used with 256 x 256 blocks of eight waves (2 x 4 waves of 128 x 64).  Measured on 4.2 M x 512 x 512 (forward):
// two 64-deep tiles 2.95 ms, three 32-deep tiles 3.07 ms, 128 x 256 blocks of four waves (two per CU) with three
// 32-deep tiles 3.17 ms; the register-staged kernel above 3.45 ms.
template <int kDmaBK, int kDmaStages, int WM, int WN, int TM, int TN, int EPI, typename TC>
__global__ __launch_bounds__(64 * WM * WN, WM * WN == 4 ? 2 : 1) void gemm_nt_dma_kernel(
    const bf16_t* __restrict__ A, int64_t lda, const bf16_t* __restrict__ Bt, int64_t ldb, TC* __restrict__ C,
    int64_t ldc, int64_t M, int N, int K, bool c_vec, float slope, const bf16_t* __restrict__ aux, int64_t ldaux,
    bool aux_vec, int tiles_n, int64_t total) {
  constexpr int NW = WM * WN, BM = 32 * WM * TM, BN = 32 * WN * TN;
  constexpr int MODE = kDmaBK == 32 ? kSwz32 : kSwz64;
  constexpr int RR = 512 / kDmaBK;                           // tile rows per 1 KB region (16 or 8)
  constexpr int CPR = kDmaBK / 8;                            // 16-byte chunks per tile row (4 or 8)
  constexpr int RA = BM / RR, RB = BN / RR;                  // 1 KB regions of a tile's A part and Bt part
  constexpr int LA = RA / NW, LB = RB / NW;                  // regions (= loads) per wave and tile
  static_assert(RA % NW == 0 && RB % NW == 0, "whole regions per wave");
  constexpr int TILE = (BM + BN) * kDmaBK;                   // elements of one tile
  extern __shared__ __align__(16) unsigned char smem_raw[];
  bf16_t* smem = reinterpret_cast<bf16_t*>(smem_raw);        // [3][TILE]: rows 0..BM-1 = A, then BN rows of Bt
  const int t = threadIdx.x, w = t >> 6, lane = t & 63, wm = w / WN, wn = w % WN;
  const int64_t item = xcd_order(blockIdx.x, total);
  const int64_t row0 = (item / tiles_n) * BM;
  const int col0 = (int)(item % tiles_n) * BN;
  v16f acc[TM][TN];
  zero_acc<TM, TN>(acc);

  // the rows this lane fetches from (regions w, w + NW, .. of the A part, then of the Bt part) and its chunk in them
  const bf16_t* src[LA + LB];
  int coff[LA + LB];
#pragma unroll
  for (int j = 0; j < LA + LB; ++j) {
    const bool is_a = j < LA;
    const int row = ((is_a ? j : j - LA) * NW + w) * RR + lane / CPR;       // tile row inside its part
    const int chunk = kDmaBK == 32 ? (lane & 3) ^ ((row >> 2) & 3) : (lane & 7) ^ (row & 7);
    coff[j] = chunk * 8;
    if (is_a) {
      const int64_t r = row0 + row < M ? row0 + row : M - 1;
      src[j] = A + r * lda;
    } else {
      const int r = col0 + row < N ? col0 + row : N - 1;
      src[j] = Bt + (int64_t)r * ldb;
    }
  }
  const int n_kt = (K + kDmaBK - 1) / kDmaBK;
  auto issue = [&](int tile) {
    const int koff = (tile < n_kt ? tile : 0) * kDmaBK;
    unsigned char* dst = smem_raw + (tile % kDmaStages) * (TILE * 2) + w * 1024;
#pragma unroll
    for (int j = 0; j < LA + LB; ++j) {
      const int region = j < LA ? j * NW : RA + (j - LA) * NW;       // + w, already in dst
      int col = koff + coff[j];
      if (j < LA && col >= K) col = 0;                               // past the end of A's rows: see above
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src[j] + col),
                                       (__attribute__((address_space(3))) void*)(dst + region * 1024), 16, 0, 0);
    }
  };
#pragma unroll
  for (int d = 0; d < kDmaStages - 1; ++d) issue(d);
  for (int kt = 0; kt < n_kt; ++kt) {
    // vmcnt((stages - 2) tiles): this wave's share of tile kt is in LDS
    __builtin_amdgcn_s_waitcnt(0x0F70 | ((kDmaStages - 2) * (LA + LB)));
    __builtin_amdgcn_s_barrier();
    issue(kt + kDmaStages - 1);
    const bf16_t* cur = smem + (kt % kDmaStages) * TILE;
    mma_tile<kDmaBK, TM, TN, MODE>(cur, cur + BM * kDmaBK, wm * 32 * TM, wn * 32 * TN, acc);
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);                        // vmcnt(0): the two trailing fetches have landed too
  store_rows<EPI, TM, TN, TC>(acc, reinterpret_cast<float*>(smem_raw), C, ldc, row0 + wm * 32 * TM, col0 + wn * 32 * TN,
                              M, N, c_vec, slope, aux, ldaux, aux_vec);
}

// ---- TN ----------------------------------------------------------------------------------------
// Output tile 128 x 128 of K x N; work item = (slab, output tile) with the output tile fastest, so the
// blocks that read the same rows of A and G follow each other on one XCD.  Writes P[slab][K x N] (ld N).
constexpr int TBK = 64;            // rows of A / G per tile (the contraction index)
constexpr int TLDK = TBK + 8;

__device__ __forceinline__ uint32_t dword_of(const uint4& v, int d) { return d == 0 ? v.x : d == 1 ? v.y : d == 2 ? v.z : v.w; }

// in[r] = 8 consecutive columns of row r (r = 0..7)  ->  out[c] = rows 0..7 of column c.
__device__ __forceinline__ void transpose8x8(const uint4 (&in)[8], uint4 (&out)[8]) {
#pragma unroll
  for (int d = 0; d < 4; ++d) {        // dword d of a row holds its columns 2d (low half) and 2d+1 (high half)
    uint32_t lo[4], hi[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const uint32_t x = dword_of(in[2 * j], d), y = dword_of(in[2 * j + 1], d);
      lo[j] = __builtin_amdgcn_perm(y, x, 0x05040100u);   // column 2d   of rows 2j (low half), 2j+1 (high half)
      hi[j] = __builtin_amdgcn_perm(y, x, 0x07060302u);   // column 2d+1 of rows 2j, 2j+1
    }
    out[2 * d] = make_uint4(lo[0], lo[1], lo[2], lo[3]);
    out[2 * d + 1] = make_uint4(hi[0], hi[1], hi[2], hi[3]);
  }
}

// FAST: as for the NT kernel, for both operands (16-byte aligned rows).
template <bool FAST>
__global__ __launch_bounds__(256, 2) void gemm_tn_kernel(const bf16_t* __restrict__ A, int64_t lda,
                                                      const bf16_t* __restrict__ G, int64_t ldg,
                                                      float* __restrict__ P, int64_t M, int K, int N,
                                                      int64_t slab_rows, int tiles_n, int tiles, int64_t total,
                                                      bool a_vec, bool g_vec) {
  constexpr int TILE = 2 * 128 * TLDK;                         // 128 tile rows of A^T, then 128 of G^T
  extern __shared__ __align__(16) unsigned char smem_raw[];
  bf16_t* smem = reinterpret_cast<bf16_t*>(smem_raw);          // [2][TILE]
  const int t = threadIdx.x, w = t >> 6, wm = w >> 1, wn = w & 1;
  const int64_t item = xcd_order(blockIdx.x, total);
  const int tile = (int)(item % tiles);
  const int64_t slab = item / tiles;
  const int k0 = (tile / tiles_n) * 128;    // output row block (columns of A)
  const int n0 = (tile % tiles_n) * 128;    // output column block (columns of G)
  const int64_t m_begin = slab * slab_rows;
  const int64_t m_end = m_begin + slab_rows < M ? m_begin + slab_rows : M;
  v16f acc[2][2];
  zero_acc<2, 2>(acc);

  // threads 0..127 move A, 128..255 move G; unit u = (row group mb of 8 rows, column group cb of 8 columns)
  const bool is_g = t >= 128;
  const int u = t & 127, cb = u & 15, mb = u >> 4;
  const bf16_t* src = is_g ? G : A;
  const int64_t ld = is_g ? ldg : lda;
  const int c0 = (is_g ? n0 : k0) + cb * 8;
  const int n_cols = is_g ? N : K;
  const bool vec = is_g ? g_vec : a_vec;
  const int tile_row0 = (is_g ? 128 : 0) + cb * 8;
  uint4 rin[kTnDepth][8];                     // kTnDepth tiles in flight in registers, tile j in slot j % kTnDepth
  const bool col_ok = c0 < n_cols;
  auto fetch = [&](uint4 (&in)[8], int64_t m1) {
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      const int64_t row = m1 + mb * 8 + r;
      if (FAST)
        in[r] = *reinterpret_cast<const uint4*>(src + (row < m_end && col_ok ? row * ld + c0 : 0));
      else
        in[r] = load_piece(src, ld, row, m_end, c0, n_cols, vec);
    }
  };
  auto stage = [&](const uint4 (&in)[8], bf16_t* tl, int64_t m1) {
    uint4 rin_ok[8], rout[8];
#pragma unroll
    for (int r = 0; r < 8; ++r)
      rin_ok[r] = keep_first(in[r], !FAST ? 8 : (m1 + mb * 8 + r < m_end ? n_cols - c0 : 0));
    transpose8x8(rin_ok, rout);
#pragma unroll
    for (int c = 0; c < 8; ++c)
      *reinterpret_cast<uint4*>(tl + tile_off<TLDK, kSwzTn>(tile_row0 + c, mb)) = rout[c];
  };
  // As in the NT kernel, the pipeline is free of conditions: rows past the slab are fetched as zeros.
  const int64_t n_mt = (m_end - m_begin + TBK - 1) / TBK;
#pragma unroll
  for (int d = 0; d < kTnDepth; ++d) fetch(rin[d], m_begin + d * TBK);
  stage(rin[0], smem, m_begin);
  fetch(rin[0], m_begin + (int64_t)kTnDepth * TBK);
  __syncthreads();
  for (int64_t mt0 = 0; mt0 < n_mt; mt0 += kTnDepth) {
    bool done = false;
#pragma unroll
    for (int d = 0; d < kTnDepth; ++d) {
      const int64_t mt = mt0 + d;
      bf16_t* cur = smem + (mt & 1) * TILE;
      bf16_t* nxt = smem + ((mt & 1) ^ 1) * TILE;
      mma_tile<TBK, 2, 2, kSwzTn>(cur, cur, wm * 64, 128 + wn * 64, acc);
      const int slot = (d + 1) % kTnDepth;                   // tile mt + 1
      stage(rin[slot], nxt, m_begin + (mt + 1) * TBK);
      fetch(rin[slot], m_begin + (mt + 1 + kTnDepth) * TBK);
      __syncthreads();
      if (mt + 1 >= n_mt) {                                  // the same for every thread of the block
        done = true;
        break;
      }
    }
    if (done) break;
  }
  float* Pslab = P + slab * (int64_t)K * N;
  store_acc<EPI_NONE, 2, 2, float>(acc, Pslab, N, k0 + wm * 64, n0 + wn * 64, K, N, 0.f, nullptr, 0);
}

// ---- TN, tiles loaded straight into LDS -----------------------------------------------------------
// Output tile 256 x 256 of K x N by WM x WN waves (used: 2 x 4 of 128 x 64), so that a block reads each row of A and G once
// per 256 output columns / rows instead of once per 128.  A tile is kTwBK rows of A and of G, 256 columns each,
// row-major as in memory: 512-byte rows, the A part first; a 1 KB region is two tile rows, wave w moves regions w,
// w + NW, .. of each part, and kTwStages tiles live in LDS (all but one in flight while that one is multiplied; waits
// as in the NT kernel).  The matrix instruction wants, per lane, 8 consecutive reduction rows of one column; the transposing LDS
// read delivers exactly that from a row-major tile: within 16 lanes, lane t points at the 8 bytes of row t / 4, columns
// 4 (t % 4) .. + 3, and lane i receives column i of those four rows.  Two such reads make one operand.
// Bank conflicts: the 64 lanes of one read touch 4 rows x 2 (reduction halves) x 32 columns, and rows are 512 bytes
// apart, so the 16-byte chunk c of tile row r is kept at position c ^ (4 (r & 3) + 16 ((r >> 3) & 1)) -- applied, as
// in the NT kernel, to the address a lane fetches from; the read then covers all 32 slots of a 512-byte window once.
// Conditions (checked by the launcher): 16-byte aligned rows of A and G, no 16-byte piece reaching past the end of an
// allocated row, slabs of whole tiles.  Rows past the end of the last slab are fetched from row M - 1 and zeroed in
// LDS before they are multiplied; column chunks past K or N are fetched from column 0 and feed only accumulators that
// are not stored.
// Measured on 4.2 M x 512 x 512 (the 128 x 128 kernel above: 4.12 ms): tiles of 64 rows, two in LDS 2.71 ms; tiles of
// 32 rows, two, three or four in LDS 3.01 - 3.03 ms (the number in flight does not matter, the barriers per row do);
// twice as many slabs (two blocks' worth of work per CU instead of one) 2.74 ms; four waves of 128 x 128 (WM = WN = 2:
// 256 accumulator registers per lane, a third fewer operand reads from LDS per matrix instruction, one wave per
// SIMD) 2.77 ms against 2.66 for the eight waves of 128 x 64 in the same run.

typedef short v4s __attribute__((ext_vector_type(4)));

__device__ __forceinline__ bf16x8 read_tr8(const unsigned char* p) {
  // rows r .. r + 3 and r + 4 .. r + 7 of the lane's column: two transposing reads 4 tile rows (2 KB) apart
  const v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s*)(p));
  const v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s*)(p + 4 * 512));
  typedef short v8s __attribute__((ext_vector_type(8)));
  const v8s both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, both);
}

template <int kTwBK, int kTwStages, int WM, int WN>
__global__ __launch_bounds__(64 * WM * WN, 1) void gemm_tn_dma_kernel(const bf16_t* __restrict__ A, int64_t lda,
                                                                      const bf16_t* __restrict__ G, int64_t ldg,
                                                                      float* __restrict__ P, int64_t M, int K, int N,
                                                                      int64_t slab_rows, int tiles_n, int tiles,
                                                                      int64_t total, bool p_vec) {
  constexpr int kTwPart = kTwBK * 256;                       // elements of a tile's A part (and of its G part)
  constexpr int NW = WM * WN, TM = 8 / WM, TN = 8 / WN;      // waves; 32 x 32 accumulator blocks per wave
  constexpr int LP = kTwBK / 2 / NW;                         // regions (= loads) per wave, part and tile
  static_assert(LP * NW * 2 == kTwBK, "whole regions per wave");
  extern __shared__ __align__(16) unsigned char smem_raw[];
  const int t = threadIdx.x, w = t >> 6, lane = t & 63, wm = w / WN, wn = w % WN;
  const int64_t item = xcd_order(blockIdx.x, total);
  const int tile = (int)(item % tiles);
  const int64_t slab = item / tiles;
  const int k0 = (tile / tiles_n) * 256;    // output row block (columns of A)
  const int n0 = (tile % tiles_n) * 256;    // output column block (columns of G)
  const int64_t m_begin = slab * slab_rows;
  const int64_t m_end = m_begin + slab_rows < M ? m_begin + slab_rows : M;
  const int n_mt = (int)((m_end - m_begin + kTwBK - 1) / kTwBK);
  v16f acc[TM][TN];
  zero_acc<TM, TN>(acc);

  // what this lane fetches in load j of a part: tile row 2 (w + NW j) + lane / 32, the chunk that belongs in slot
  // lane % 32 of that row
  auto issue = [&](int mt) {
    const int64_t m0 = m_begin + (int64_t)(mt < n_mt ? mt : 0) * kTwBK;
    unsigned char* dst = smem_raw + (mt % kTwStages) * (2 * kTwPart * 2) + w * 1024;
#pragma unroll
    for (int j = 0; j < 2 * LP; ++j) {
      const bool is_a = j < LP;
      const int jj = is_a ? j : j - LP;
      const int frow = 2 * (jj * NW + w) + (lane >> 5);
      const int fchunk = (lane & 31) ^ (((frow & 3) << 2) | (((frow >> 3) & 1) << 4));
      int col = (is_a ? k0 : n0) + fchunk * 8;
      if (col >= (is_a ? K : N)) col = 0;
      int64_t row = m0 + frow;
      row = row < M ? row : M - 1;
      const bf16_t* src = is_a ? A + row * lda + col : G + row * ldg + col;
      const int region = (is_a ? 0 : kTwBK / 2) + jj * NW;            // + w, already in dst
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                       (__attribute__((address_space(3))) void*)(dst + region * 1024), 16, 0, 0);
    }
  };

  // what this lane reads: see above; g16 = which 16 columns of the 32, kg = which 8 of the 16 reduction rows
  const int t16 = lane & 15, g16 = (lane >> 4) & 1, kg = lane >> 5;
  const int swz = ((t16 >> 2) << 2) | (kg << 4);             // of tile rows 8 kg + t16 / 4 (+ 4, + 16 ks)
  const int low = (2 * g16 + ((t16 & 3) >> 1)) * 16 + (t16 & 1) * 8 + (8 * kg + (t16 >> 2)) * 512;
  int off_a[TM], off_g[TN];                                  // byte offsets inside a part, reduction row 0
#pragma unroll
  for (int tm = 0; tm < TM; ++tm) off_a[tm] = ((((wm * TM + tm) * 32) >> 3) ^ swz) * 16 + low;
#pragma unroll
  for (int tn = 0; tn < TN; ++tn) off_g[tn] = ((((wn * TN + tn) * 32) >> 3) ^ swz) * 16 + low + kTwPart * 2;

#pragma unroll
  for (int d = 0; d < kTwStages - 1; ++d) issue(d);
  for (int mt = 0; mt < n_mt; ++mt) {
    __builtin_amdgcn_s_waitcnt(0x0F70 | ((kTwStages - 2) * 2 * LP));   // this wave's share of tile mt is in LDS
    __builtin_amdgcn_s_barrier();
    unsigned char* cur = smem_raw + (mt % kTwStages) * (2 * kTwPart * 2);
    const int64_t valid = m_end - (m_begin + (int64_t)mt * kTwBK);
    if (valid < kTwBK) {                                     // the same for every thread; only a slab's last tile
      const int first = (int)valid;                          // rows first .. 63 of both parts
      for (int p = t; p < (kTwBK - first) * 32; p += 64 * NW) {
        *reinterpret_cast<uint4*>(cur + first * 512 + p * 16) = make_uint4(0u, 0u, 0u, 0u);
        *reinterpret_cast<uint4*>(cur + kTwPart * 2 + first * 512 + p * 16) = make_uint4(0u, 0u, 0u, 0u);
      }
      __syncthreads();
    }
    issue(mt + kTwStages - 1);
    // the operands of step ks + 1 are read while the matrix instructions of step ks run
    bf16x8 a[2][TM], b[2][TN];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) a[0][tm] = read_tr8(cur + off_a[tm]);
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) b[0][tn] = read_tr8(cur + off_g[tn]);
#pragma unroll
    for (int ks = 0; ks < kTwBK / 16; ++ks) {
      if (ks + 1 < kTwBK / 16) {
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) a[(ks + 1) & 1][tm] = read_tr8(cur + off_a[tm] + (ks + 1) * 16 * 512);
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) b[(ks + 1) & 1][tn] = read_tr8(cur + off_g[tn] + (ks + 1) * 16 * 512);
      }
#pragma unroll
      for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
          acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks & 1][tm], b[ks & 1][tn], acc[tm][tn], 0, 0, 0);
    }
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);                        // the trailing fetch has landed before LDS is reused
  float* Pslab = P + slab * (int64_t)K * N;
  store_rows<EPI_NONE, TM, TN, float>(acc, reinterpret_cast<float*>(smem_raw), Pslab, N, k0 + wm * 32 * TM,
                                      n0 + wn * 32 * TN, K, N, p_vec, 0.f, nullptr, 0, false);
}

// out[r][c] (leading dimension ld_out) = transpose ? W[c][r] : W[r][c], rounded to bfloat16; zero for
// out_cols <= c < ld_out.  W is row-major with w_cols columns.
__global__ void weights_to_bf16(const float* __restrict__ W, int w_cols, bool transpose, bf16_t* __restrict__ out,
                                int out_rows, int out_cols, int ld_out) {
  const int64_t e = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (e >= (int64_t)out_rows * ld_out) return;
  const int r = (int)(e / ld_out), c = (int)(e % ld_out);
  float v = 0.f;
  if (c < out_cols) v = transpose ? W[(int64_t)c * w_cols + r] : W[(int64_t)r * w_cols + c];
  out[e] = float_to_bf16(v);
}

bool vec_ok(const bf16_t* p, int64_t ld) { return (ld % 8 == 0) && ((reinterpret_cast<uintptr_t>(p) & 15u) == 0); }

constexpr int kNtBKmax = 64;

template <int kNtBK, int WM, int WN, int TM, int TN, typename TC>
int launch_nt(const bf16_t* A, int64_t lda, const bf16_t* Bt, int64_t ldb, TC* C, int64_t ldc, int64_t M, int N, int K,
              const Epi& e, hipStream_t s) {
  constexpr int BM = 32 * WM * TM, BN = 32 * WN * TN, NT = 64 * WM * WN;
  constexpr size_t tiles_bytes = 2u * (BM + BN) * (kNtBK == 32 ? 32 : kNtBK + 8) * sizeof(bf16_t);   // two operand tiles
  constexpr size_t stage_bytes = (size_t)(WM * WN) * 32 * (32 * TN + 8) * sizeof(float);    // epilogue staging, reuses them
  constexpr size_t smem = tiles_bytes > stage_bytes ? tiles_bytes : stage_bytes;
  static_assert(smem <= 160 * 1024, "one block's tiles fit the CU's LDS");
  const int tiles_n = (int)ceil_div(N, BN);
  const int64_t total = ceil_div(M, BM) * tiles_n;
  GAD_GRID_CHECK(total, NT);
  const bf16_t* aux = static_cast<const bf16_t*>(e.aux);
  const bool av = vec_ok(A, lda);
  const bool fast = av && (e.full_rows || K % 8 == 0);      // no 16-byte piece may reach past the end of a row
  const bool cv = (ldc % (16 / (int)sizeof(TC)) == 0) && ((reinterpret_cast<uintptr_t>(C) & 15u) == 0);
  const bool xv = aux != nullptr && vec_ok(aux, e.ldaux);
#define GAD_NT_LAUNCH(EPI)                                                                                          \
  {                                                                                                                 \
    auto kern = fast ? gemm_nt_kernel<kNtBK, WM, WN, TM, TN, EPI, TC, true>                                         \
                     : gemm_nt_kernel<kNtBK, WM, WN, TM, TN, EPI, TC, false>;                                       \
    static std::atomic<bool> attr_set[2];          /* set once per kernel; setting it twice is harmless */          \
    if (!attr_set[fast].load(std::memory_order_acquire)) {                                                          \
      GAD_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,  \
                                  (int)smem));                                                                      \
      attr_set[fast].store(true, std::memory_order_release);                                                        \
    }                                                                                                               \
    kern<<<(unsigned)total, NT, smem, s>>>(A, lda, Bt, ldb, C, ldc, M, N, K, av, cv, e.slope, aux, e.ldaux, xv,     \
                                           tiles_n, total);                                                         \
  }
  switch (e.kind) {
    case EPI_NONE: GAD_NT_LAUNCH(EPI_NONE) break;
    case EPI_RELU: GAD_NT_LAUNCH(EPI_RELU) break;
    case EPI_MASK: GAD_NT_LAUNCH(EPI_MASK) break;
    default: return set_error(GAD_ERR_UNSUPPORTED, "unknown epilogue %d", e.kind);
  }
#undef GAD_NT_LAUNCH
  GAD_LAUNCH_CHECK();
  return GAD_OK;
}

template <int kDmaBK, int kDmaStages, int WM, int WN, int TM, int TN, typename TC>
int launch_nt_dma(const bf16_t* A, int64_t lda, const bf16_t* Bt, int64_t ldb, TC* C, int64_t ldc, int64_t M, int N, int K,
                  const Epi& e, hipStream_t s) {
  constexpr int BM = 32 * WM * TM, BN = 32 * WN * TN, NT = 64 * WM * WN;
  constexpr size_t tiles_bytes = (size_t)kDmaStages * (BM + BN) * kDmaBK * sizeof(bf16_t);
  constexpr size_t stage_bytes = (size_t)(WM * WN) * 32 * (32 * TN + 8) * sizeof(float);
  constexpr size_t smem = tiles_bytes > stage_bytes ? tiles_bytes : stage_bytes;
  static_assert((WM * WN == 4 ? 2 : 1) * smem <= 160 * 1024, "the blocks of a CU fit its LDS");
  const int tiles_n = (int)ceil_div(N, BN);
  const int64_t total = ceil_div(M, BM) * tiles_n;
  GAD_GRID_CHECK(total, NT);
  const bf16_t* aux = static_cast<const bf16_t*>(e.aux);
  const bool cv = (ldc % (16 / (int)sizeof(TC)) == 0) && ((reinterpret_cast<uintptr_t>(C) & 15u) == 0);
  const bool xv = aux != nullptr && vec_ok(aux, e.ldaux);
#define GAD_DMA_LAUNCH(EPI)                                                                                         \
  {                                                                                                                 \
    auto kern = gemm_nt_dma_kernel<kDmaBK, kDmaStages, WM, WN, TM, TN, EPI, TC>;                                                        \
    static std::atomic<bool> attr_set;                                                                              \
    if (!attr_set.load(std::memory_order_acquire)) {                                                                \
      GAD_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,  \
                                  (int)smem));                                                                      \
      attr_set.store(true, std::memory_order_release);                                                              \
    }                                                                                                               \
    kern<<<(unsigned)total, NT, smem, s>>>(A, lda, Bt, ldb, C, ldc, M, N, K, cv, e.slope, aux, e.ldaux, xv,         \
                                           tiles_n, total);                                                         \
  }
  switch (e.kind) {
    case EPI_NONE: GAD_DMA_LAUNCH(EPI_NONE) break;
    case EPI_RELU: GAD_DMA_LAUNCH(EPI_RELU) break;
    case EPI_MASK: GAD_DMA_LAUNCH(EPI_MASK) break;
    default: return set_error(GAD_ERR_UNSUPPORTED, "unknown epilogue %d", e.kind);
  }
#undef GAD_DMA_LAUNCH
  GAD_LAUNCH_CHECK();
  return GAD_OK;
}

// GAD_NT_WIDE=0 in the environment keeps outputs of 256 columns or more on the register-staged kernel.
bool nt_wide_direct() {
  static const bool on = [] {
    const char* e = getenv("GAD_NT_WIDE");
    return !(e && e[0] == '0');
  }();
  return on;
}

template <typename TC>
int nt_typed(const bf16_t* A, int64_t lda, const bf16_t* Bt, int64_t ldb, TC* C, int64_t ldc, int64_t M, int N, int K,
             const Epi& e, hipStream_t s) {
  // Narrow outputs: 64-deep tiles staged through registers, two or three blocks per CU.
  if (N <= 64) return launch_nt<64, 2, 2, 2, 1, TC>(A, lda, Bt, ldb, C, ldc, M, N, K, e, s);
  if (N <= 128) return launch_nt<64, 2, 2, 2, 2, TC>(A, lda, Bt, ldb, C, ldc, M, N, K, e, s);
  // Wide outputs: 256 x 256 blocks, tiles loaded straight into LDS -- two 64-deep tiles (three 32-deep ones for
  // K <= 32); unaligned rows, or a K that is not a whole number of 16-byte chunks, stay on the register-staged kernel
  // (128 x 256 blocks, 32-deep tiles).  Bt is zero filled up to a multiple of 64, which covers either tile depth.
  if (N >= 256 && nt_wide_direct() && M >= 1 && K % 8 == 0 && vec_ok(A, lda) && vec_ok(Bt, ldb)) {
    if (K > 32) return launch_nt_dma<64, 2, 2, 4, 4, 2, TC>(A, lda, Bt, ldb, C, ldc, M, N, K, e, s);
    return launch_nt_dma<32, 3, 2, 4, 4, 2, TC>(A, lda, Bt, ldb, C, ldc, M, N, K, e, s);
  }
  return launch_nt<32, 2, 2, 2, 4, TC>(A, lda, Bt, ldb, C, ldc, M, N, K, e, s);
}

}  // namespace

size_t bf16_weight_elems(int n_out, int k) { return (size_t)n_out * (size_t)round_up(k, kNtBKmax); }

int gemm_w_bf16(const void* A, int64_t lda, const float* W, int w_rows, int w_cols, bool trans_w, void* C, int64_t ldc,
                gad_dtype tc, int64_t M, const Epi& e, void* scratch, hipStream_t s) {
  const int N = trans_w ? w_rows : w_cols, K = trans_w ? w_cols : w_rows;
  if (M == 0 || N == 0) return GAD_OK;
  // Bt[n][k] = op(W)[k][n]: W^T when op is the identity, W itself when op is the transpose.
  bf16_t* Bt = static_cast<bf16_t*>(scratch);
  const int ldb = (int)round_up(K, kNtBKmax);
  weights_to_bf16<<<(unsigned)ceil_div((int64_t)N * ldb, 256), 256, 0, s>>>(W, w_cols, !trans_w, Bt, N, K, ldb);
  GAD_LAUNCH_CHECK();
  const bf16_t* a = static_cast<const bf16_t*>(A);
  if (tc == GAD_BF16) return nt_typed<bf16_t>(a, lda, Bt, ldb, static_cast<bf16_t*>(C), ldc, M, N, K, e, s);
  return nt_typed<float>(a, lda, Bt, ldb, static_cast<float*>(C), ldc, M, N, K, e, s);
}

bool gemm_tn_bf16_wide_ok(const void* A, int64_t lda, const void* G, int64_t ldg, int K, int N, bool full_rows) {
  static const bool on = [] {                                // GAD_TN_WIDE=0 keeps every shape on the 128 x 128 kernel
    const char* e = getenv("GAD_TN_WIDE");
    return !(e && e[0] == '0');
  }();
  return on && tn_wide_shape(K, N) && vec_ok(static_cast<const bf16_t*>(A), lda) &&
         vec_ok(static_cast<const bf16_t*>(G), ldg) && (full_rows || (K % 8 == 0 && N % 8 == 0));
}

int gemm_tn_bf16(const void* A, int64_t lda, const void* G, int64_t ldg, float* partials, int64_t M, int K, int N,
                 int n_slabs, int64_t slab_rows, bool full_rows, bool wide, hipStream_t s) {
  const bf16_t* a = static_cast<const bf16_t*>(A);
  const bf16_t* g = static_cast<const bf16_t*>(G);
  if (wide) {
    constexpr int kTwBK = 64, kTwStages = 2;
    constexpr size_t tiles_bytes = (size_t)kTwStages * 2 * kTwBK * 256 * sizeof(bf16_t);
    constexpr size_t kTwSmem = tiles_bytes;                  // the epilogue staging (at most 70 KB) reuses them
    static_assert(kTwSmem <= 160 * 1024 && kTwSmem >= 4u * 32 * (32 * 4 + 8) * sizeof(float), "LDS of one block");
    if (!gemm_tn_bf16_wide_ok(A, lda, G, ldg, K, N, full_rows) || slab_rows % kTwBK != 0 || M < 1)
      return set_error(GAD_ERR_UNSUPPORTED, "the 256 x 256 weight-gradient kernel does not take these operands");
    auto kern = gemm_tn_dma_kernel<kTwBK, kTwStages, 2, 4>;
    constexpr int threads = 512;
    static std::atomic<bool> wide_attr_set;          // set once; setting it twice is harmless
    if (!wide_attr_set.load(std::memory_order_acquire)) {
      GAD_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  (int)kTwSmem));
      wide_attr_set.store(true, std::memory_order_release);
    }
    const int tiles_n = (int)ceil_div(N, 256);
    const int tiles = (int)ceil_div(K, 256) * tiles_n;
    const int64_t total = (int64_t)tiles * n_slabs;
    GAD_GRID_CHECK(total, threads);
    // every slab of the partial products starts on a 16-byte boundary when K N is a multiple of 4
    const bool pv = N % 4 == 0 && (reinterpret_cast<uintptr_t>(partials) & 15u) == 0 && ((int64_t)K * N) % 4 == 0;
    kern<<<(unsigned)total, threads, kTwSmem, s>>>(a, lda, g, ldg, partials, M, K, N, slab_rows, tiles_n, tiles, total, pv);
    GAD_LAUNCH_CHECK();
    return GAD_OK;
  }
  constexpr size_t smem = 2u * 2u * 128u * TLDK * sizeof(bf16_t);
  const bool av = vec_ok(a, lda), gv = vec_ok(g, ldg);
  const bool fast = av && gv && (full_rows || (K % 8 == 0 && N % 8 == 0));   // no piece may reach past a row's end
  auto kern = fast ? gemm_tn_kernel<true> : gemm_tn_kernel<false>;
  static std::atomic<bool> attr_set[2];            // set once per kernel; setting it twice is harmless
  if (!attr_set[fast].load(std::memory_order_acquire)) {
    GAD_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)smem));
    attr_set[fast].store(true, std::memory_order_release);
  }
  const int tiles_n = (int)ceil_div(N, 128);
  const int tiles = (int)ceil_div(K, 128) * tiles_n;
  const int64_t total = (int64_t)tiles * n_slabs;
  GAD_GRID_CHECK(total, 256);
  kern<<<(unsigned)total, 256, smem, s>>>(a, lda, g, ldg, partials, M, K, N, slab_rows, tiles_n, tiles, total, av, gv);
  GAD_LAUNCH_CHECK();
  return GAD_OK;
}

}  // namespace gad
