// Shared device helpers of the float32 matrix-core kernels (gfx950, v_mfma_f32_32x32x2_f32): the LDS tile of one
// k-slice of both operands, the per-tile multiply, and the loaders that stage 8-element row pieces.
// Four wave64s per block in a 2 x 2 arrangement; a wave owns 2 x TNW accumulators of 32 x 32.
#pragma once
#include "dtype.h"

namespace gad {
namespace {

typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int BM = 128, BK = 16;          // block rows; depth of one LDS tile (block columns: 64 TNW)
constexpr int LDS_LD = BM + 4;   // row stride of As / Bs in floats (16-byte aligned rows)

// One k-slice of both operands; TNW = accumulators per wave along N (block tile 128 x 64 TNW).
template <int TNW>
struct Tile {
  float a[BK][LDS_LD];
  float b[BK][64 * TNW + 4];
};

// acc[tm][tn] += As[:, 64*wm + 32*tm .. ]^T Bs[:, 64*wn + 32*tn ..]
// (Measured without gain against this per-k-step form at three blocks per CU: reading all fragments of a tile ahead
// of the matrix instructions, reading the next step's fragments one step ahead, a 32-deep tile at two blocks per
// CU, persistent blocks that fetch the next tile before writing the finished one, starting the three blocks
// of a CU a third of a tile time apart, a 256 x 128 block tile with 4 x 2 accumulators per wave at two blocks per
// CU (slower: 101 against 113 TFLOP/s at long K), and two tiles in flight in registers (the register ring costs
// the fourth wave per SIMD).)
template <int TNW>
__device__ __forceinline__ void mma_tile(const Tile<TNW>& t, int wm, int wn, v16f (&acc)[2][TNW]) {
  const int lane = threadIdx.x & 63;
  const int i = lane & 31, half = lane >> 5;
#pragma unroll
  for (int k0 = 0; k0 < BK; k0 += 2) {
    float a[2], b[TNW];
#pragma unroll
    for (int q = 0; q < 2; ++q) a[q] = t.a[k0 + half][wm * 64 + q * 32 + i];
#pragma unroll
    for (int q = 0; q < TNW; ++q) b[q] = t.b[k0 + half][wn * 32 * TNW + q * 32 + i];
#pragma unroll
    for (int tm = 0; tm < 2; ++tm)
#pragma unroll
      for (int tn = 0; tn < TNW; ++tn)
        acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[tm], b[tn], acc[tm][tn], 0, 0, 0);
  }
}

// Row of accumulator register r of a 32x32 MFMA result held by `lane` (its column is lane % 32).
__device__ __forceinline__ int acc_row(int r, int lane) { return 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3); }

// 8 consecutive elements of row `row` starting at column `col`, zero outside the matrix, widened to float.
// vec_ok: 8 elements may be fetched with 16-byte loads (alignment checked on the host).
template <typename T>
__device__ __forceinline__ void load8(const T* __restrict__ base, int64_t ld, int64_t row, int64_t n_rows, int col,
                                      int n_cols, bool vec_ok, float (&r)[8]) {
  if (row < n_rows && vec_ok && col + 8 <= n_cols) {
    const T* p = base + row * ld + col;
    if constexpr (sizeof(T) == 4) {
      float lo[4], hi[4];
      load_row_piece<4, T>(p, lo);
      load_row_piece<4, T>(p + 4, hi);
#pragma unroll
      for (int q = 0; q < 4; ++q) { r[q] = lo[q]; r[4 + q] = hi[q]; }
    } else {
      load_row_piece<8, T>(p, r);
    }
  } else {
#pragma unroll
    for (int q = 0; q < 8; ++q)
      r[q] = (row < n_rows && col + q < n_cols) ? to_f32<T>(base[row * ld + col + q]) : 0.f;
  }
}

template <int LD>
__device__ __forceinline__ void store_direct(float (*dst)[LD], int kk, int seg, const float (&r)[8]) {
  *reinterpret_cast<float4*>(&dst[kk][seg]) = make_float4(r[0], r[1], r[2], r[3]);
  *reinterpret_cast<float4*>(&dst[kk][seg + 4]) = make_float4(r[4], r[5], r[6], r[7]);
}

__device__ __forceinline__ void store_transposed(float (*dst)[LDS_LD], int i, int kseg, const float (&r)[8]) {
#pragma unroll
  for (int q = 0; q < 8; ++q) dst[kseg + q][i] = r[q];
}

}  // namespace
}  // namespace gad
