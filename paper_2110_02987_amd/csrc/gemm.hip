// Dense contractions of the GCN step on the gfx950 matrix cores (float32 MFMA 32x32x2):
//   NN:  C[M x N] = A[M x K] B[K x N]          -- the feature transform H W of Eq. 7 and the
//                                                  input-gradient product S W^T (B = W^T)
//   TN:  C[K x N] = A[M x K]^T G[M x N]        -- the weight gradient dW = (A~ H)^T G, a reduction
//                                                  over the M = n nodes, split over M in slabs whose
//                                                  partial products are added in slab order.
// (arXiv 2110.02987, Section 3.3: Eq. 7 forward; backward step of Algorithm 2.)
//
// Block tile 128 x 128, four wave64s in a 2 x 2 arrangement, each wave a 64 x 64 sub-tile made of
// 2 x 2 MFMA 32x32 accumulators; outputs of at most 64 columns (the class logits, their gradient) use a
// 128 x 64 block tile (2 x 1 accumulators per wave) so that matrix instructions are not spent on padding.
// Both operands are staged through LDS with the reduction index leading (As[kk][i], Bs[kk][j]) so that a
// fragment read is 64 consecutive floats; the next tile is fetched from global memory into registers while
// the current one is multiplied (double-buffered LDS).
// This file holds the float32 storage path; bfloat16 storage runs on the bfloat16 matrix instruction
// (gemm_bf16.hip).
#include "dtype.h"
#include "gad_internal.h"
#include "mfma_tile.h"
#include "xcd.h"

namespace gad {
namespace {

// Row stride (floats) of a wave's staging block in the epilogue: rows 4 apart, which the two halves of a wave
// write together, fall on different halves of the LDS banks.
template <int TNW>
constexpr int stage_ld() { return 32 * TNW + 8; }

// LDS bytes of a block: the two operand tiles, reused by the epilogue as four staging blocks of 32 rows.
template <int TNW>
constexpr size_t block_lds_bytes() {
  constexpr size_t tiles = 2 * sizeof(Tile<TNW>), stage = 4 * 32 * stage_ld<TNW>() * sizeof(float);
  return tiles > stage ? tiles : stage;
}

// Epilogue: the accumulators of a wave (64 rows x 32 TNW columns, held column-per-lane) go through a
// wave-private LDS block, 32 rows at a time, and leave as 16-byte row pieces, so that a wave instruction writes
// (and, for the mask, reads) whole rows instead of 32-float column strips.  The mask values of a pass are requested
// before the accumulators are staged.  Entered by all four waves after the last read of the operand tiles.
// c_vec / aux_vec: 16-byte accesses allowed at any column that is a multiple of 4 (alignment checked on the host).
template <int EPI, int TNW>
__device__ __forceinline__ void store_acc(const v16f (&acc)[2][TNW], float* __restrict__ lds, float* __restrict__ C,
                                          int64_t ldc, int64_t row0, int col0, int64_t M, int N, int wm, int wn,
                                          float slope, const float* __restrict__ aux, int64_t ldaux, bool c_vec,
                                          bool aux_vec) {
  constexpr int W = 32 * TNW, LD = stage_ld<TNW>();
  constexpr int LPR = W / 4;            // lanes per row, one 16-byte piece each
  constexpr int RPI = 64 / LPR;         // rows per wave instruction
  constexpr int NI = 32 / RPI;          // wave instructions per 32-row pass
  const int lane = threadIdx.x & 63;
  float* mine = lds + (threadIdx.x >> 6) * (32 * LD);
  const int rl = lane / LPR, cl = (lane % LPR) * 4;
  const int col = col0 + wn * W + cl;
  const bool full = col + 4 <= N;
  __syncthreads();                     // every wave is done with the operand tiles; from here on a wave uses only its
                                       // own staging block, and the LDS operations of one wave complete in order
#pragma unroll
  for (int tm = 0; tm < 2; ++tm) {
    const int64_t rbase = row0 + wm * 64 + tm * 32 + rl;
    float m[NI][4];
    if (EPI == EPI_MASK) {
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        const int64_t row = rbase + i * RPI;
        const float* ap = aux + row * ldaux + col;
        if (row < M && full && aux_vec) {
          load_row_piece<4, float>(ap, m[i]);
        } else {
#pragma unroll
          for (int q = 0; q < 4; ++q) m[i][q] = (row < M && col + q < N) ? ap[q] : 0.f;
        }
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");     // the staging writes stay behind the previous pass's reads
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int tn = 0; tn < TNW; ++tn)
#pragma unroll
      for (int r = 0; r < 16; ++r) mine[acc_row(r, lane) * LD + tn * 32 + (lane & 31)] = acc[tm][tn][r];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");     // and ahead of this pass's reads
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int64_t row = rbase + i * RPI;
      const float4 t = *reinterpret_cast<const float4*>(&mine[(rl + i * RPI) * LD + cl]);
      float v[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        if (EPI == EPI_RELU) v[q] = leaky(v[q], v[q] > 0.f, slope);
        if (EPI == EPI_MASK) v[q] = leaky(v[q], m[i][q] > 0.f, slope);
      }
      if (row < M && col < N) {
        float* cp = C + row * ldc + col;
        if (full && c_vec) {
          *reinterpret_cast<float4*>(cp) = make_float4(v[0], v[1], v[2], v[3]);
        } else {
#pragma unroll
          for (int q = 0; q < 4; ++q)
            if (col + q < N) cp[q] = v[q];
        }
      }
    }
  }
}

static_assert(BM * BK / 8 == 256, "one 8-float piece of A per thread and tile");

// ---- NN ----------------------------------------------------------------------------------------
// grid: one block per (row tile of 128 rows, column tile of 64 TNW columns), column tile fastest and renumbered so
// that the column tiles of a row tile run on the same XCD: the rows of A come from HBM once and from that XCD's L2
// for the other column tiles.
template <int EPI, int TNW>
__global__ __launch_bounds__(256) void gemm_nn_kernel(const float* __restrict__ A, int64_t lda,
                                                      const float* __restrict__ B, int64_t ldb, float* __restrict__ C,
                                                      int64_t ldc, int64_t M, int N, int K, bool a_vec, bool b_vec,
                                                      bool c_vec, float slope, const float* __restrict__ aux,
                                                      int64_t ldaux, bool aux_vec, int tiles_n, int64_t total) {
  constexpr int BNW = 64 * TNW, SEGB = BNW / 8;      // block columns; 8-float pieces per B row
  __shared__ __align__(16) unsigned char lds_raw[block_lds_bytes<TNW>()];
  Tile<TNW>* tiles = reinterpret_cast<Tile<TNW>*>(lds_raw);
  const int t = threadIdx.x, w = t >> 6, wm = w >> 1, wn = w & 1;
  const int64_t item = xcd_order(blockIdx.x, total);
  const int64_t row0 = (item / tiles_n) * BM;
  const int col0 = (int)(item % tiles_n) * BNW;
  v16f acc[2][TNW];
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int y = 0; y < TNW; ++y)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[x][y][r] = 0.f;

  // piece t of A: row t / (BK/8), k segment (t % (BK/8)) * 8;  piece t of B (t < BK * SEGB): k row t / SEGB,
  // column segment (t % SEGB) * 8
  const bool has_b = t < BK * SEGB;
  float ra[8], rb[8];
  auto fetch = [&](int k1) {
    load8<float>(A, lda, row0 + t / (BK / 8), M, k1 + (t % (BK / 8)) * 8, K, a_vec, ra);
    if (has_b) load8<float>(B, ldb, k1 + t / SEGB, K, col0 + (t % SEGB) * 8, N, b_vec, rb);
  };
  auto stage = [&](Tile<TNW>& tile) {
    store_transposed(tile.a, t / (BK / 8), (t % (BK / 8)) * 8, ra);
    if (has_b) store_direct(tile.b, t / SEGB, (t % SEGB) * 8, rb);
  };
  fetch(0);
  stage(tiles[0]);
  __syncthreads();
  const int n_kt = (K + BK - 1) / BK;
  for (int kt = 0; kt < n_kt; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < n_kt) fetch((kt + 1) * BK);
    mma_tile<TNW>(tiles[cur], wm, wn, acc);
    if (kt + 1 < n_kt) stage(tiles[cur ^ 1]);
    __syncthreads();
  }
  store_acc<EPI, TNW>(acc, reinterpret_cast<float*>(lds_raw), C, ldc, row0, col0, M, N, wm, wn, slope, aux, ldaux,
                      c_vec, aux_vec);
}

// ---- TN ----------------------------------------------------------------------------------------
// grid: x = output tile (tiles_k * tiles_n) of 128 x 64 TNW, y = slab of M.  Writes P[slab][K x N] (ld N).
template <int TNW>
__global__ __launch_bounds__(256) void gemm_tn_kernel(const float* __restrict__ A, int64_t lda,
                                                      const float* __restrict__ G, int64_t ldg, float* __restrict__ P,
                                                      int64_t M, int K, int N, int64_t slab_rows, int tiles_n,
                                                      bool a_vec, bool g_vec, bool p_vec) {
  constexpr int BNW = 64 * TNW, SEGB = BNW / 8;
  __shared__ __align__(16) unsigned char lds_raw[block_lds_bytes<TNW>()];
  Tile<TNW>* tiles = reinterpret_cast<Tile<TNW>*>(lds_raw);
  const int t = threadIdx.x, w = t >> 6, wm = w >> 1, wn = w & 1;
  const int k0 = (blockIdx.x / tiles_n) * BM;    // output row block (columns of A)
  const int n0 = (blockIdx.x % tiles_n) * BNW;   // output column block (columns of G)
  const int64_t m_begin = (int64_t)blockIdx.y * slab_rows;
  const int64_t m_end = m_begin + slab_rows < M ? m_begin + slab_rows : M;
  v16f acc[2][TNW];
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int y = 0; y < TNW; ++y)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[x][y][r] = 0.f;

  // piece t: reduction row t / 16, column segment (t % 16) * 8 of A; row t / SEGB, segment (t % SEGB) * 8 of G
  const bool has_b = t < BK * SEGB;
  float ra[8], rb[8];
  auto fetch = [&](int64_t m1) {
    load8<float>(A, lda, m1 + t / 16, m_end, k0 + (t % 16) * 8, K, a_vec, ra);
    if (has_b) load8<float>(G, ldg, m1 + t / SEGB, m_end, n0 + (t % SEGB) * 8, N, g_vec, rb);
  };
  auto stage = [&](Tile<TNW>& tile) {
    store_direct(tile.a, t / 16, (t % 16) * 8, ra);
    if (has_b) store_direct(tile.b, t / SEGB, (t % SEGB) * 8, rb);
  };
  fetch(m_begin);
  stage(tiles[0]);
  __syncthreads();
  const int64_t n_mt = (m_end - m_begin + BK - 1) / BK;
  for (int64_t mt = 0; mt < n_mt; ++mt) {
    const int cur = (int)(mt & 1);
    if (mt + 1 < n_mt) fetch(m_begin + (mt + 1) * BK);
    mma_tile<TNW>(tiles[cur], wm, wn, acc);
    if (mt + 1 < n_mt) stage(tiles[cur ^ 1]);
    __syncthreads();
  }
  float* Pslab = P + (int64_t)blockIdx.y * K * N;
  store_acc<EPI_NONE, TNW>(acc, reinterpret_cast<float*>(lds_raw), Pslab, N, k0, n0, K, N, wm, wn, 0.f, nullptr, 0,
                           p_vec, false);
}

// C = sum over the slabs of P[slab], in float64 and in a fixed order: a block owns 32 output elements; its eight
// 32-lane groups each add a contiguous run of slabs (four partial sums per thread keep four loads in flight and are
// combined in a fixed order), then the eight run sums are added in run order.
__global__ __launch_bounds__(256) void reduce_slabs(const float* __restrict__ P, int n_slabs, int64_t elems, int N,
                                                    float* __restrict__ C, int64_t ldc) {
  __shared__ double run_sum[8][32];
  const int l = threadIdx.x & 31, run = threadIdx.x >> 5;
  const int64_t e = blockIdx.x * 32ll + l;
  const int q0 = (int)((int64_t)run * n_slabs / 8), q1 = (int)((int64_t)(run + 1) * n_slabs / 8);
  double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
  if (e < elems) {
    const float* p = P + e;
    int q = q0;
    for (; q + 4 <= q1; q += 4) {
      s0 += (double)p[(int64_t)q * elems];
      s1 += (double)p[(int64_t)(q + 1) * elems];
      s2 += (double)p[(int64_t)(q + 2) * elems];
      s3 += (double)p[(int64_t)(q + 3) * elems];
    }
    for (; q < q1; ++q) s0 += (double)p[(int64_t)q * elems];
  }
  run_sum[run][l] = (s0 + s1) + (s2 + s3);
  __syncthreads();
  if (run == 0 && e < elems) {
    double s = run_sum[0][l];
#pragma unroll
    for (int r = 1; r < 8; ++r) s += run_sum[r][l];
    C[(e / N) * ldc + (e % N)] = (float)s;
  }
}

__global__ void transpose_kernel(const float* __restrict__ in, int rows, int cols, float* __restrict__ out) {
  __shared__ float tile[32][33];
  const int x = blockIdx.x * 32 + threadIdx.x, y0 = blockIdx.y * 32;
  for (int dy = threadIdx.y; dy < 32; dy += blockDim.y)
    if (x < cols && y0 + dy < rows) tile[dy][threadIdx.x] = in[(int64_t)(y0 + dy) * cols + x];
  __syncthreads();
  const int ox = blockIdx.y * 32 + threadIdx.x, oy0 = blockIdx.x * 32;
  for (int dy = threadIdx.y; dy < 32; dy += blockDim.y)
    if (ox < rows && oy0 + dy < cols) out[(int64_t)(oy0 + dy) * rows + ox] = tile[threadIdx.x][dy];
}

// 8 elements of a row can be fetched with 16-byte loads from any column that is a multiple of 8
template <typename T>
bool vec_ok(const T* p, int64_t ld) {
  return (ld % (16 / (int)sizeof(T)) == 0) && ((reinterpret_cast<uintptr_t>(p) & 15u) == 0);
}

// Block columns: 64 when the output has at most 64 columns (a 128-wide tile would spend most of its matrix
// instructions on padding), else 128.
inline int block_cols(int N) { return N <= 64 ? 64 : 128; }

// wide: the bfloat16 kernel with 256 x 256 output tiles, one block per CU.
void tn_split(int64_t M, int K, int N, bool wide, int* n_slabs, int64_t* slab_rows) {
  const int64_t tiles = wide ? ceil_div(K, 256) * ceil_div(N, 256) : ceil_div(K, BM) * ceil_div(N, block_cols(N));
  int64_t want = ceil_div(wide ? 256 : 512, tiles);   // one block (wide) or ~2 blocks per CU over the whole grid
  const int64_t max_slabs = ceil_div(M, 512);         // at least 512 reduction rows per slab
  if (want > max_slabs) want = max_slabs;
  if (want < 1) want = 1;
  *slab_rows = round_up(ceil_div(M, want), 64);       // whole tiles of every kernel (16 or 64 rows)
  *n_slabs = (int)ceil_div(M, *slab_rows);
}

template <int TNW>
int gemm_nn_launch(const float* A, int64_t lda, const float* B, int64_t ldb, float* C, int64_t ldc, int64_t M, int N,
                   int K, const Epi& e, hipStream_t s) {
  const float* aux = static_cast<const float*>(e.aux);
  const int64_t ldaux = e.ldaux;
  const int tiles_n = (int)ceil_div(N, 64 * TNW);
  const int64_t total = ceil_div(M, BM) * tiles_n;
  GAD_GRID_CHECK(total, 256);
  const unsigned grid = (unsigned)total;
  const bool av = vec_ok(A, lda), bv = vec_ok(B, ldb), cv = vec_ok(C, ldc);
  const bool xv = e.kind == EPI_MASK && vec_ok(aux, ldaux);
  switch (e.kind) {
    case EPI_NONE:
      gemm_nn_kernel<EPI_NONE, TNW><<<grid, 256, 0, s>>>(A, lda, B, ldb, C, ldc, M, N, K, av, bv, cv, e.slope, aux, ldaux, xv,
                                                         tiles_n, total);
      break;
    case EPI_RELU:
      gemm_nn_kernel<EPI_RELU, TNW><<<grid, 256, 0, s>>>(A, lda, B, ldb, C, ldc, M, N, K, av, bv, cv, e.slope, aux, ldaux, xv,
                                                         tiles_n, total);
      break;
    case EPI_MASK:
      gemm_nn_kernel<EPI_MASK, TNW><<<grid, 256, 0, s>>>(A, lda, B, ldb, C, ldc, M, N, K, av, bv, cv, e.slope, aux, ldaux, xv,
                                                         tiles_n, total);
      break;
    default:
      return set_error(GAD_ERR_UNSUPPORTED, "unknown epilogue %d", e.kind);
  }
  GAD_LAUNCH_CHECK();
  return GAD_OK;
}

int gemm_nn_f32(const float* A, int64_t lda, const float* B, int64_t ldb, float* C, int64_t ldc, int64_t M, int N, int K,
                const Epi& e, hipStream_t s) {
  if (block_cols(N) == 64) return gemm_nn_launch<1>(A, lda, B, ldb, C, ldc, M, N, K, e, s);
  return gemm_nn_launch<2>(A, lda, B, ldb, C, ldc, M, N, K, e, s);
}

int gemm_tn_f32(const float* A, int64_t lda, const float* G, int64_t ldg, float* C, int64_t ldc, int64_t M, int K, int N,
                float* partials, hipStream_t s) {
  int n_slabs;
  int64_t slab_rows;
  tn_split(M, K, N, false, &n_slabs, &slab_rows);
  const int tiles_n = (int)ceil_div(N, block_cols(N));
  const dim3 grid((unsigned)(ceil_div(K, BM) * tiles_n), (unsigned)n_slabs);
  // every slab of the partial products starts on a 16-byte boundary when K N is a multiple of 4
  const bool pv = vec_ok(partials, N) && ((int64_t)K * N) % 4 == 0;
  if (block_cols(N) == 64)
    gemm_tn_kernel<1><<<grid, 256, 0, s>>>(A, lda, G, ldg, partials, M, K, N, slab_rows, tiles_n, vec_ok(A, lda),
                                           vec_ok(G, ldg), pv);
  else
    gemm_tn_kernel<2><<<grid, 256, 0, s>>>(A, lda, G, ldg, partials, M, K, N, slab_rows, tiles_n, vec_ok(A, lda),
                                           vec_ok(G, ldg), pv);
  GAD_LAUNCH_CHECK();
  const int64_t elems = (int64_t)K * N;
  reduce_slabs<<<(unsigned)ceil_div(elems, 32), 256, 0, s>>>(partials, n_slabs, elems, N, C, ldc);
  GAD_LAUNCH_CHECK();
  return GAD_OK;
}

}  // namespace

size_t gemm_w_scratch_bytes(int w_rows, int w_cols) {
  const size_t f32 = (size_t)w_rows * w_cols * sizeof(float);                       // transposed float32 copy
  const size_t a = bf16_weight_elems(w_cols, w_rows) * sizeof(bf16_t);              // bfloat16 W^T, padded rows
  const size_t b = bf16_weight_elems(w_rows, w_cols) * sizeof(bf16_t);              // bfloat16 W, padded rows
  return f32 > a ? (f32 > b ? f32 : b) : (a > b ? a : b);
}

int gemm_w(const void* A, int64_t lda, gad_dtype ta, const float* W, int w_rows, int w_cols, bool trans_w, void* C,
           int64_t ldc, gad_dtype tc, int64_t M, const Epi& e, void* scratch, hipStream_t s) {
  const int N = trans_w ? w_rows : w_cols, K = trans_w ? w_cols : w_rows;
  if (M == 0 || N == 0) return GAD_OK;
  if (ta == GAD_BF16) return gemm_w_bf16(A, lda, W, w_rows, w_cols, trans_w, C, ldc, tc, M, e, scratch, s);
  if (tc != GAD_F32) return set_error(GAD_ERR_UNSUPPORTED, "GEMM from float32 storage to bfloat16 storage is not implemented");
  const float* B = W;
  if (trans_w) {
    int st = transpose_f32(W, w_rows, w_cols, static_cast<float*>(scratch), s);
    if (st != GAD_OK) return st;
    B = static_cast<const float*>(scratch);
  }
  return gemm_nn_f32((const float*)A, lda, B, N, (float*)C, ldc, M, N, K, e, s);
}

size_t gemm_tn_partial_floats(int64_t M, int K, int N) {
  int n_slabs, n_wide = 0;
  int64_t slab_rows;
  tn_split(M, K, N, false, &n_slabs, &slab_rows);
  if (tn_wide_shape(K, N)) tn_split(M, K, N, true, &n_wide, &slab_rows);   // whichever kernel ends up running
  return (size_t)(n_slabs > n_wide ? n_slabs : n_wide) * (size_t)K * (size_t)N;
}

int gemm_tn(const void* A, int64_t lda, const void* G, int64_t ldg, gad_dtype t, float* C, int64_t ldc, int64_t M,
            int K, int N, float* partials, bool full_rows, hipStream_t s) {
  if (K == 0 || N == 0) return GAD_OK;
  if (t == GAD_F32) return gemm_tn_f32((const float*)A, lda, (const float*)G, ldg, C, ldc, M, K, N, partials, s);
  const bool wide = gemm_tn_bf16_wide_ok(A, lda, G, ldg, K, N, full_rows);
  int n_slabs;
  int64_t slab_rows;
  tn_split(M, K, N, wide, &n_slabs, &slab_rows);
  int st = gemm_tn_bf16(A, lda, G, ldg, partials, M, K, N, n_slabs, slab_rows, full_rows, wide, s);
  if (st != GAD_OK) return st;
  const int64_t elems = (int64_t)K * N;
  reduce_slabs<<<(unsigned)ceil_div(elems, 32), 256, 0, s>>>(partials, n_slabs, elems, N, C, ldc);
  GAD_LAUNCH_CHECK();
  return GAD_OK;
}

int transpose_f32(const float* in, int rows, int cols, float* out, hipStream_t s) {
  if (rows == 0 || cols == 0) return GAD_OK;
  transpose_kernel<<<dim3((unsigned)ceil_div(cols, 32), (unsigned)ceil_div(rows, 32)), dim3(32, 8), 0, s>>>(in, rows,
                                                                                                            cols, out);
  GAD_LAUNCH_CHECK();
  return GAD_OK;
}

}  // namespace gad
