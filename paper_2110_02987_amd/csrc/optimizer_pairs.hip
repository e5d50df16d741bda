// Variance-based subgraph importance with the distance inside the pair sum -- the other reading of Eq. 14
// (arXiv 2110.02987, Section 3.4.1):
//     zeta_pair = sum_{i<j} p_i p_j / (||v_i - v_j||_2 + beta),   p_i = deg_i / sum_k deg_k.
// All n (n - 1) / 2 pairs are visited in 128 x 128 tiles of the upper triangle.  The squared distances of a
// tile come from one matrix product on the float32 matrix cores,
//     ||v_i - v_j||^2 = ||v_i||^2 + ||v_j||^2 - 2 v_i . v_j,
// taken on vectors that were first centred on the subgraph mean (identical vectors then give exactly 0, which the
// paper's worked example needs, and the magnitudes that cancel are as small as they can be).  The difference of
// large numbers loses accuracy only for pairs that are close compared with their norms; where that loss could
// show in the pair's term (see kGramErr / kTermTol) the squared distance is recomputed from the coordinate
// differences.
// The tile epilogue applies 1 / (sqrt(d^2) + beta) and the degree product; tile sums are float64 and are added
// in a fixed order (per block, then over blocks), so the result is reproducible bit for bit.
#include <math.h>

#include "gad_internal.h"
#include "mfma_tile.h"

namespace gad {
namespace {

// A squared distance from the Gram tile carries an absolute error of about kGramErr (||v_i||^2 + ||v_j||^2); it is
// recomputed from coordinate differences when that error could move the pair's term by more than kTermTol of
// its value (the error of d is at most delta / (d + sqrt(delta)); the term is 1 / (d + beta)).
constexpr float kGramErr = 1e-6f;
constexpr float kTermTol = 2e-5f;

// Vc[i][c] = float(v_ic - mean_c) for c < F, 0 for F <= c < ldv;  nrm[i] = sum_c Vc[i][c]^2 (of the rounded
// values, so that the norm and the matrix product describe the same vectors);  degf[i] = float(deg_i).
// A 16-lane group owns one row.
template <typename T>
__global__ __launch_bounds__(256) void centre_rows(const T* __restrict__ V, int64_t n, int F,
                                                   const double* __restrict__ mean, const int32_t* __restrict__ deg,
                                                   float* __restrict__ Vc, int64_t ldv, float* __restrict__ nrm,
                                                   float* __restrict__ degf) {
  const int grp = threadIdx.x >> 4, l = threadIdx.x & 15;
  const int64_t i = (int64_t)blockIdx.x * 16 + grp;
  double s = 0.0;
  if (i < n) {
    for (int c = l; c < (int)ldv; c += 16) {
      float v = 0.f;
      if (c < F) v = (float)((double)to_f32<T>(V[i * F + c]) - mean[c]);
      Vc[i * ldv + c] = v;
      s += (double)v * (double)v;
    }
  }
#pragma unroll
  for (int o = 8; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
  if (i < n && l == 0) {
    nrm[i] = (float)s;
    degf[i] = (float)deg[i];
  }
}

// Block partial sums of deg and deg^2 (exact 64-bit integers).
__global__ __launch_bounds__(256) void degree_partials(const int32_t* __restrict__ deg, int64_t n,
                                                       unsigned long long* __restrict__ part) {
  __shared__ unsigned long long s1[256], s2[256];
  unsigned long long a = 0, b = 0;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const unsigned long long d = (unsigned long long)deg[i];
    a += d;
    b += d * d;
  }
  s1[threadIdx.x] = a;
  s2[threadIdx.x] = b;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) {
      s1[threadIdx.x] += s1[threadIdx.x + o];
      s2[threadIdx.x] += s2[threadIdx.x + o];
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    part[2 * blockIdx.x] = s1[0];
    part[2 * blockIdx.x + 1] = s2[0];
  }
}

// Tile b of the upper triangle (row-major, T tiles per side) -> (ti, tj), ti <= tj.
__device__ __forceinline__ void tile_of(int64_t b, int64_t T, int* ti, int* tj) {
  // row ti starts at offset ti * T - ti (ti - 1) / 2
  const double t2 = 2.0 * (double)T + 1.0;
  int64_t r = (int64_t)((t2 - sqrt(t2 * t2 - 8.0 * (double)b)) * 0.5);
  if (r < 0) r = 0;
  if (r > T - 1) r = T - 1;
  while (r > 0 && r * T - r * (r - 1) / 2 > b) --r;
  while (r + 1 < T && (r + 1) * T - (r + 1) * r / 2 <= b) ++r;
  *ti = (int)r;
  *tj = (int)(r + (b - (r * T - r * (r - 1) / 2)));
}

__global__ __launch_bounds__(256) void pair_tiles(const float* __restrict__ Vc, int64_t ldv,
                                                  const float* __restrict__ nrm, const float* __restrict__ degf,
                                                  int64_t n, int64_t T, int64_t n_tiles, float beta,
                                                  double* __restrict__ tile_sum) {
  __shared__ Tile<2> tiles[2];
  __shared__ float info[4][BM];          // ||v_i||^2, deg_i of the tile's rows; ||v_j||^2, deg_j of its columns
  __shared__ double red[256];
  const int t = threadIdx.x, w = t >> 6, wm = w >> 1, wn = w & 1, lane = t & 63;
  const int64_t tile = (int64_t)blockIdx.y * gridDim.x + blockIdx.x;     // the grid is folded into two dimensions
  if (tile >= n_tiles) return;                                          // (whole blocks leave)
  int ti, tj;
  tile_of(tile, T, &ti, &tj);
  const int64_t i0 = (int64_t)ti * BM, j0 = (int64_t)tj * BM;
  {
    const int64_t r = (t < BM ? i0 : j0 - BM) + t;
    const bool ok = r < n;
    info[t < BM ? 0 : 2][t & (BM - 1)] = ok ? nrm[r] : 0.f;
    info[t < BM ? 1 : 3][t & (BM - 1)] = ok ? degf[r] : 0.f;
  }
  v16f acc[2][2];
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int y = 0; y < 2; ++y)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[x][y][r] = 0.f;

  // piece t of either operand: row t / (BK/8) of the tile, k segment (t % (BK/8)) * 8; Vc is zero padded to ldv
  const int K = (int)ldv;
  float ra[8], rb[8];
  auto fetch = [&](int k1) {
    load8<float>(Vc, ldv, i0 + t / (BK / 8), n, k1 + (t % (BK / 8)) * 8, K, true, ra);
    load8<float>(Vc, ldv, j0 + t / (BK / 8), n, k1 + (t % (BK / 8)) * 8, K, true, rb);
  };
  auto stage = [&](Tile<2>& tile) {
    store_transposed(tile.a, t / (BK / 8), (t % (BK / 8)) * 8, ra);
    store_transposed(tile.b, t / (BK / 8), (t % (BK / 8)) * 8, rb);
  };
  fetch(0);
  stage(tiles[0]);
  __syncthreads();
  const int n_kt = K / BK;               // ldv is a multiple of BK
  for (int kt = 0; kt < n_kt; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < n_kt) fetch((kt + 1) * BK);
    mma_tile<2>(tiles[cur], wm, wn, acc);
    if (kt + 1 < n_kt) stage(tiles[cur ^ 1]);
    __syncthreads();
  }

  // 64 pairs per lane.  Square root and reciprocal are the hardware's one-instruction forms (1 ulp; the library
  // forms cost ten times the instructions and this loop bounds the kernel for short vectors); a squared distance
  // below the smallest normal float counts as 0.  Rows and columns past n carry degree 0.
  // First pass: every pair from the Gram tile; a pair whose lost digits would show adds nothing here and sets its
  // bit.  Second pass: those pairs, from coordinate differences.  Keeping the rare path
  // out of the unrolled loop keeps the kernel's code small.
  float sum = 0.f;
  uint32_t redo[2] = {0u, 0u};                         // redo[tm], bit 16 tn + r
#pragma unroll
  for (int tm = 0; tm < 2; ++tm)
#pragma unroll
    for (int tn = 0; tn < 2; ++tn) {
      const int cl = wn * 64 + tn * 32 + (lane & 31);
      const int64_t gj = j0 + cl;
      const float nj = info[2][cl], dj = info[3][cl];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int rl = wm * 64 + tm * 32 + acc_row(r, lane);
        const bool valid = (i0 + rl < gj) & (gj < n);                 // (bitwise: no branches in this loop)
        const float s2 = info[0][rl] + nj;
        const float d2 = fmaxf(s2 - 2.f * acc[tm][tn][r], 0.f);
        const float d = __builtin_amdgcn_sqrtf(d2);
        const float delta = kGramErr * s2;
        const bool close = valid & (delta > kTermTol * (d + __builtin_amdgcn_sqrtf(delta)) * (d + beta));
        redo[tm] |= (close ? 1u : 0u) << (16 * tn + r);
        const float w = (valid & !close) ? info[1][rl] * dj : 0.f;
        sum = fmaf(w, __builtin_amdgcn_rcpf(d + beta), sum);
      }
    }
  uint64_t todo = ((uint64_t)redo[1] << 32) | redo[0];
  while (todo != 0) {
    const int bit = __ffsll((unsigned long long)todo) - 1;
    todo &= todo - 1;
    const int tm = bit >> 5, tn = (bit >> 4) & 1, r = bit & 15;
    const int rl = wm * 64 + tm * 32 + acc_row(r, lane);
    const int cl = wn * 64 + tn * 32 + (lane & 31);
    const float4* a = reinterpret_cast<const float4*>(Vc + (i0 + rl) * ldv);
    const float4* b = reinterpret_cast<const float4*>(Vc + (j0 + cl) * ldv);
    float e = 0.f;
    for (int c = 0; c < K / 4; ++c) {
      const float4 x = a[c], y = b[c];
      const float d0 = x.x - y.x, d1 = x.y - y.y, d2 = x.z - y.z, d3 = x.w - y.w;
      e = fmaf(d0, d0, e);
      e = fmaf(d1, d1, e);
      e = fmaf(d2, d2, e);
      e = fmaf(d3, d3, e);
    }
    sum = fmaf(info[1][rl] * info[3][cl], __builtin_amdgcn_rcpf(__builtin_amdgcn_sqrtf(e) + beta), sum);
  }
  red[t] = (double)sum;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if (t < o) red[t] += red[t + o];
    __syncthreads();
  }
  if (t == 0) tile_sum[tile] = red[0];
}

static_assert(BM == 128 && 2 * BM == 256, "the info loader maps one thread to one row or column of the tile");

// part[b] = sum of block b's contiguous share of the tile sums (fixed shares, fixed order inside a share).
__global__ __launch_bounds__(256) void sum_tiles(const double* __restrict__ tile_sum, int64_t n_tiles, int64_t share,
                                                 double* __restrict__ part) {
  __shared__ double sm[256];
  const int64_t b = (int64_t)blockIdx.x * share;
  const int64_t e = b + share < n_tiles ? b + share : n_tiles;
  double s = 0.0;
  for (int64_t k = b + threadIdx.x; k < e; k += 256) s += tile_sum[k];
  sm[threadIdx.x] = s;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) sm[threadIdx.x] += sm[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) part[blockIdx.x] = sm[0];
}

__global__ __launch_bounds__(256) void finalize_pairs(const double* __restrict__ tile_sum, int64_t n_tiles,
                                                      const unsigned long long* __restrict__ dpart, int n_dpart,
                                                      double* __restrict__ out2) {
  __shared__ double sm[256];
  double s = 0.0;
  for (int64_t k = threadIdx.x; k < n_tiles; k += 256) s += tile_sum[k];
  sm[threadIdx.x] = s;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) sm[threadIdx.x] += sm[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    unsigned long long s1 = 0, s2 = 0;
    for (int b = 0; b < n_dpart; ++b) {
      s1 += dpart[2 * b];
      s2 += dpart[2 * b + 1];
    }
    double zeta = 0.0, spp = 0.0;
    if (s1 != 0) {
      const double sq = (double)s1 * (double)s1;
      zeta = sm[0] / sq;
      spp = 0.5 * (1.0 - (double)s2 / sq);
    }
    out2[0] = zeta;
    out2[1] = spp;
  }
}

constexpr int kDegBlocks = 256;
constexpr int kSumBlocks = 1024;
constexpr size_t kAlign = 256;

struct Layout {
  size_t vc, nrm, degf, mean, colpart, tiles, tilepart, dpart, total;
  int64_t ldv, T, n_tiles;
};

Layout layout(int64_t n, int F) {
  Layout L;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    size_t o = off;
    off += (bytes + kAlign - 1) / kAlign * kAlign;
    return o;
  };
  L.ldv = round_up(F, BK);
  L.T = ceil_div(n, BM);
  L.n_tiles = L.T * (L.T + 1) / 2;
  L.vc = take((size_t)n * L.ldv * sizeof(float));
  L.nrm = take((size_t)n * sizeof(float));
  L.degf = take((size_t)n * sizeof(float));
  L.mean = take((size_t)F * sizeof(double));
  L.colpart = take((size_t)kVarBlocks * F * sizeof(double));
  L.tiles = take((size_t)L.n_tiles * sizeof(double));
  L.tilepart = take((size_t)kSumBlocks * sizeof(double));
  L.dpart = take((size_t)2 * kDegBlocks * sizeof(unsigned long long));
  L.total = off;
  return L;
}

}  // namespace

size_t pair_importance_workspace_bytes(int64_t n, int F) { return layout(n, F).total; }

int pair_importance(const gad_graph* g, const void* V, int F, gad_dtype dtype, double beta, double* out2, void* ws,
                    hipStream_t s) {
  const int64_t n = g->n;
  const Layout L = layout(n, F);
  constexpr int64_t kGridX = 1 << 20;                                   // tiles per row of the folded grid
  const int64_t grid_y = ceil_div(L.n_tiles, kGridX);
  if (grid_y > 65535) return set_error(GAD_ERR_SHAPE, "n = %lld has too many pair tiles for one launch", (long long)n);
  char* base = static_cast<char*>(ws);
  float* Vc = reinterpret_cast<float*>(base + L.vc);
  float* nrm = reinterpret_cast<float*>(base + L.nrm);
  float* degf = reinterpret_cast<float*>(base + L.degf);
  double* mean = reinterpret_cast<double*>(base + L.mean);
  double* colpart = reinterpret_cast<double*>(base + L.colpart);
  double* tile_sum = reinterpret_cast<double*>(base + L.tiles);
  double* tile_part = reinterpret_cast<double*>(base + L.tilepart);
  unsigned long long* dpart = reinterpret_cast<unsigned long long*>(base + L.dpart);
  int st = column_means_f64(V, n, F, dtype, colpart, mean, s);
  if (st != GAD_OK) return st;
  GAD_GRID_CHECK(ceil_div(n, 16), 256);
  const unsigned row_blocks = (unsigned)ceil_div(n, 16);
  if (dtype == GAD_F32)
    centre_rows<float><<<row_blocks, 256, 0, s>>>(static_cast<const float*>(V), n, F, mean, g->deg, Vc, L.ldv, nrm, degf);
  else
    centre_rows<bf16_t><<<row_blocks, 256, 0, s>>>(static_cast<const bf16_t*>(V), n, F, mean, g->deg, Vc, L.ldv, nrm, degf);
  GAD_LAUNCH_CHECK();
  const int dblocks = (int)(ceil_div(n, 256) < kDegBlocks ? ceil_div(n, 256) : kDegBlocks);
  degree_partials<<<dblocks, 256, 0, s>>>(g->deg, n, dpart);
  GAD_LAUNCH_CHECK();
  const dim3 grid((unsigned)(L.n_tiles < kGridX ? L.n_tiles : kGridX), (unsigned)grid_y);
  pair_tiles<<<grid, 256, 0, s>>>(Vc, L.ldv, nrm, degf, n, L.T, L.n_tiles, (float)beta, tile_sum);
  GAD_LAUNCH_CHECK();
  // tile sums -> kSumBlocks partial sums -> one sum: the shares depend on the tile count alone
  const int64_t share = ceil_div(L.n_tiles, kSumBlocks);
  const int64_t n_part = ceil_div(L.n_tiles, share);
  sum_tiles<<<(unsigned)n_part, 256, 0, s>>>(tile_sum, L.n_tiles, share, tile_part);
  GAD_LAUNCH_CHECK();
  finalize_pairs<<<1, 256, 0, s>>>(tile_part, n_part, dpart, dblocks, out2);
  GAD_LAUNCH_CHECK();
  return GAD_OK;
}

}  // namespace gad
