// Normalised sparse aggregation  out = A~ T,  A~ = D~^-1/2 (A + I) D~^-1/2  (the A~ H of Eq. 7,
// arXiv 2110.02987; also the backward product A~^T G = A~ G since A~ is symmetric).
//
// out_i = dinv_i * sum_{j in row i} dinv_j * T_j.  One wave64 owns one row.  The wave is cut into
// 64/LPR groups of LPR lanes; a group gathers one neighbour row at a time, each lane holding V
// consecutive columns (16-byte loads: V = 4 float32 or 8 bfloat16), so a gathered row is read as one
// contiguous burst.  Groups walk the neighbour list interleaved and are combined with wave shuffles at
// the end.  Accumulation is float32 whatever the storage type.  Only the 4-byte column index is read per
// edge; dinv_j comes from a 4n-byte array that stays in L2.
// Rows longer than kLongRow are cut into chunks, one wave per chunk (the first blocks of the same
// launch), whose raw sums go to a partial buffer and are added in chunk order by a second kernel
// (deterministic: no floating-point atomics).
#include "dtype.h"
#include "gad_internal.h"

namespace gad {
namespace {

// Sum over the neighbour positions [begin, end) of dinv_j * T_j for this lane's V columns starting at
// column c (if `active`), combined over the wave's groups.  All lanes return the combined value.
template <int LPR, int V, typename TI>
__device__ __forceinline__ void gather_sum(const int32_t* __restrict__ colidx, const float* __restrict__ dinv,
                                           const TI* __restrict__ T, int64_t ldt, int64_t begin, int64_t end, int c,
                                           bool active, float (&acc)[V]) {
  constexpr int G = 64 / LPR;
  const int lane = threadIdx.x & 63;
  const int grp = lane / LPR;
#pragma unroll
  for (int k = 0; k < V; ++k) acc[k] = 0.f;
  int64_t p = begin + grp;
  // four neighbours in flight per group
  for (; p + 3 * G < end; p += 4 * G) {
    const int32_t j0 = colidx[p], j1 = colidx[p + G], j2 = colidx[p + 2 * G], j3 = colidx[p + 3 * G];
    const float d0 = dinv[j0], d1 = dinv[j1], d2 = dinv[j2], d3 = dinv[j3];
    if (active) {
      float t0[V], t1[V], t2[V], t3[V];
      load_row_piece<V, TI>(T + (int64_t)j0 * ldt + c, t0);
      load_row_piece<V, TI>(T + (int64_t)j1 * ldt + c, t1);
      load_row_piece<V, TI>(T + (int64_t)j2 * ldt + c, t2);
      load_row_piece<V, TI>(T + (int64_t)j3 * ldt + c, t3);
#pragma unroll
      for (int k = 0; k < V; ++k) {
        acc[k] = fmaf(d0, t0[k], acc[k]);
        acc[k] = fmaf(d1, t1[k], acc[k]);
        acc[k] = fmaf(d2, t2[k], acc[k]);
        acc[k] = fmaf(d3, t3[k], acc[k]);
      }
    }
  }
  for (; p < end; p += G) {
    const int32_t j = colidx[p];
    const float d = dinv[j];
    if (active) {
      float t[V];
      load_row_piece<V, TI>(T + (int64_t)j * ldt + c, t);
#pragma unroll
      for (int k = 0; k < V; ++k) acc[k] = fmaf(d, t[k], acc[k]);
    }
  }
#pragma unroll
  for (int off = LPR; off < 64; off <<= 1) {
#pragma unroll
    for (int k = 0; k < V; ++k) acc[k] += __shfl_xor(acc[k], off, 64);
  }
}

template <typename TI, typename TO>
__device__ __forceinline__ void store_elem(TO* __restrict__ out, int64_t ldo, int64_t i, int c, float v, int epi,
                                           float slope, const TI* __restrict__ aux, int64_t ldaux) {
  if (epi == EPI_RELU) v = leaky(v, v > 0.f, slope);
  if (epi == EPI_MASK) v = leaky(v, to_f32<TI>(aux[i * ldaux + c]) > 0.f, slope);
  out[i * ldo + c] = from_f32<TO>(v);
}

// One launch covers the whole product.  grid.y: column slab of LPR*V columns.  grid.x: the first
// `chunk_blocks` blocks take the chunks of the long rows (4 per block, one per wave; the longest work
// starts first), the remaining blocks take 4 rows each (one per wave) and skip the long rows.
// Chunk sums go to partial[chunk][column - col0] for columns in [col0, col0 + kPartialWidth).
template <int LPR, int V, typename TI, typename TO>
__global__ __launch_bounds__(256) void spmm_kernel(const int64_t* __restrict__ rowptr, const int32_t* __restrict__ colidx,
                                                   const float* __restrict__ dinv, const TI* __restrict__ T,
                                                   int64_t ldt, TO* __restrict__ out, int64_t ldo, int width, int col0,
                                                   int64_t n, int epi, float slope, const TI* __restrict__ aux,
                                                   int64_t ldaux, int chunk_blocks, const int32_t* __restrict__ chunk_row,
                                                   const int32_t* __restrict__ chunk_begin, int n_chunks,
                                                   float* __restrict__ partial) {
  const int lane = threadIdx.x & 63;
  const int rel = blockIdx.y * (LPR * V) + (lane % LPR) * V;
  const int c = col0 + rel;
  float acc[V];
  if ((int)blockIdx.x < chunk_blocks) {
    const int ch = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (ch >= n_chunks) return;
    const int64_t i = chunk_row[ch];
    const int64_t begin = rowptr[i] + chunk_begin[ch];
    const int64_t row_end = rowptr[i + 1];
    const int64_t end = begin + kLongRow < row_end ? begin + kLongRow : row_end;
    const bool active = c < width && rel < kPartialWidth;
    gather_sum<LPR, V, TI>(colidx, dinv, T, ldt, begin, end, c, active, acc);
    if (active && lane < LPR) {
#pragma unroll
      for (int k = 0; k < V; ++k)
        if (c + k < width) partial[(int64_t)ch * kPartialWidth + rel + k] = acc[k];
    }
    return;
  }
  const int64_t i = (int64_t)(blockIdx.x - chunk_blocks) * 4 + (threadIdx.x >> 6);
  if (i >= n) return;
  const int64_t begin = rowptr[i], end = rowptr[i + 1];
  if (end - begin > kLongRow) return;   // summed by the chunk blocks + spmm_long_reduce
  const bool active = c < width;
  gather_sum<LPR, V, TI>(colidx, dinv, T, ldt, begin, end, c, active, acc);
  if (active && lane < LPR) {
    const float di = dinv[i];
#pragma unroll
    for (int k = 0; k < V; ++k)
      if (c + k < width) store_elem<TI, TO>(out, ldo, i, c + k, di * acc[k], epi, slope, aux, ldaux);
  }
}

// One thread per (long row, column): adds the row's partial sums in chunk order.
template <typename TI, typename TO>
__global__ __launch_bounds__(256) void spmm_long_reduce(const int64_t* __restrict__ rowptr,
                                                        const float* __restrict__ dinv,
                                                        const int32_t* __restrict__ long_row,
                                                        const int32_t* __restrict__ long_first,
                                                        const float* __restrict__ partial, int col0, int ncols,
                                                        TO* __restrict__ out, int64_t ldo, int epi, float slope,
                                                        const TI* __restrict__ aux, int64_t ldaux) {
  const int slot = blockIdx.x;
  const int64_t i = long_row[slot];
  const int first = long_first[slot];
  const int k = (int)((rowptr[i + 1] - rowptr[i] + kLongRow - 1) / kLongRow);
  const float di = dinv[i];
  for (int rel = threadIdx.x; rel < ncols; rel += blockDim.x) {
    float s = 0.f;
    for (int q = 0; q < k; ++q) s += partial[(int64_t)(first + q) * kPartialWidth + rel];
    store_elem<TI, TO>(out, ldo, i, col0 + rel, di * s, epi, slope, aux, ldaux);
  }
}

template <int LPR, int V, typename TI, typename TO>
int launch(const gad_graph* g, const TI* T, int64_t ldt, TO* out, int64_t ldo, int width, const Epi& e, hipStream_t s) {
  const int epi = e.kind;
  const float slope = e.slope;
  const TI* aux = static_cast<const TI*>(e.aux);
  const int64_t ldaux = e.ldaux;
  constexpr int slab = LPR * V;
  const unsigned row_blocks = (unsigned)ceil_div(g->n, 4);
  const unsigned chunk_blocks = (unsigned)ceil_div(g->n_chunks, 4);
  // Columns are covered kPartialWidth at a time: one pass for every width the GCN step uses.
  for (int col0 = 0; col0 < width; col0 += kPartialWidth) {
    const int ncols = width - col0 < kPartialWidth ? width - col0 : kPartialWidth;
    const dim3 grid(chunk_blocks + row_blocks, (unsigned)ceil_div(ncols, slab));
    spmm_kernel<LPR, V, TI, TO><<<grid, 256, 0, s>>>(g->rowptr, g->colidx, g->dinv, T, ldt, out, ldo, col0 + ncols, col0,
                                                     g->n, epi, slope, aux, ldaux, (int)chunk_blocks, g->chunk_row,
                                                     g->chunk_begin, g->n_chunks, g->partial);
    GAD_LAUNCH_CHECK();
    if (g->n_long > 0) {
      spmm_long_reduce<TI, TO><<<(unsigned)g->n_long, 256, 0, s>>>(g->rowptr, g->dinv, g->long_row, g->long_first,
                                                                   g->partial, col0, ncols, out, ldo, epi, slope, aux,
                                                                   ldaux);
      GAD_LAUNCH_CHECK();
    }
  }
  return GAD_OK;
}

template <typename TI, typename TO>
int spmm_typed(const gad_graph* g, const TI* T, int64_t ldt, TO* out, int64_t ldo, int width, const Epi& e,
               hipStream_t s) {
  constexpr int VEC = 16 / (int)sizeof(TI);      // elements per 16-byte load
  const bool vec = (ldt % VEC == 0) && ((reinterpret_cast<uintptr_t>(T) & 15u) == 0);
  const int lanes = vec ? (width + VEC - 1) / VEC : width;
#define GAD_SPMM_CASE(L)                                                                                   \
  if (lanes <= L)                                                                                          \
    return vec ? launch<L, VEC, TI, TO>(g, T, ldt, out, ldo, width, e, s)                  \
               : launch<L, 1, TI, TO>(g, T, ldt, out, ldo, width, e, s);
  GAD_SPMM_CASE(4)
  GAD_SPMM_CASE(8)
  GAD_SPMM_CASE(16)
  GAD_SPMM_CASE(32)
#undef GAD_SPMM_CASE
  return vec ? launch<64, VEC, TI, TO>(g, T, ldt, out, ldo, width, e, s)
             : launch<64, 1, TI, TO>(g, T, ldt, out, ldo, width, e, s);
}

}  // namespace

int spmm(const gad_graph* g, const void* T, int64_t ldt, gad_dtype t_in, void* out, int64_t ldo, gad_dtype t_out,
         int width, const Epi& e, hipStream_t s) {
  if (g->n == 0 || width == 0) return GAD_OK;
  if (t_in == GAD_F32 && t_out == GAD_F32)
    return spmm_typed<float, float>(g, (const float*)T, ldt, (float*)out, ldo, width, e, s);
  if (t_in == GAD_BF16 && t_out == GAD_BF16)
    return spmm_typed<bf16_t, bf16_t>(g, (const bf16_t*)T, ldt, (bf16_t*)out, ldo, width, e, s);
  if (t_in == GAD_BF16 && t_out == GAD_F32)
    return spmm_typed<bf16_t, float>(g, (const bf16_t*)T, ldt, (float*)out, ldo, width, e, s);
  return set_error(GAD_ERR_UNSUPPORTED, "SpMM from float32 storage to bfloat16 storage is not implemented");
}

}  // namespace gad
