// Normalised sparse aggregation  out = A~ T,  A~ = D~^-1/2 (A + I) D~^-1/2  (the A~ H of Eq. 7,
// arXiv 2110.02987; also the backward product A~^T G = A~ G since A~ is symmetric).
//
// out_i = dinv_i * sum_{j in row i} dinv_j * T_j.  One wave64 owns one row.  The wave is cut into
// 64/LPR groups of LPR lanes; a group gathers one neighbour row at a time, each lane holding V
// consecutive columns (16-byte loads: V = 4 float32 or 8 bfloat16), so a gathered row is read as one
// contiguous burst.  Groups walk the neighbour list interleaved and are combined with wave shuffles at
// the end.  Accumulation is float32 whatever the storage type.  Per edge the 4-byte column index and the 4-byte
// factor dinv_j are read, both streamed in edge order (ew[p] = dinv[colidx[p]] is stored with the graph: gathering
// dinv[j] instead, a second access that depends on the index, cost 7 % of the kernel at width 256 and 17 - 24 % at
// widths 47 - 64; one packed 8-byte entry per edge instead of the two arrays measured within 1 - 3 % either way).
// Rows longer than kLongRow are cut into chunks, one wave per chunk (the first blocks of the same
// launch), whose raw sums go to a partial buffer and are added in a fixed order by a second kernel
// (deterministic: no floating-point atomics).
// Scheduling (arrays prepared once per graph): the chunks run ordered by the first column they gather.  A
// row's columns ascend, so chunks that run side by side read the same region of T and the rows of T that many
// long rows share are fetched from HBM once and then found in the caches; on a power-law graph most
// non-zeros sit in long rows, which is where this pays.  Short rows run longest class first, so that a
// wave's neighbours in dispatch order do similar amounts of work and wave slots are not left idle behind a
// few long waves.
#include "dtype.h"
#include "gad_internal.h"

namespace gad {
namespace {

// Sum over the neighbour positions [begin, end) of ew_p * T_j (ew_p = dinv_j) for this lane's V columns starting at
// column c (if `active`), combined over the wave's groups.  All lanes return the combined value.
template <int LPR, int V, typename TI>
__device__ __forceinline__ void gather_sum(const int32_t* __restrict__ colidx, const float* __restrict__ ew,
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
    const float d0 = ew[p], d1 = ew[p + G], d2 = ew[p + 2 * G], d3 = ew[p + 3 * G];
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
    const float d = ew[p];
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
// `chunk_blocks` blocks take the chunks of the long rows in their scheduling order (4 per block, one per wave;
// the longest work starts first), the remaining blocks take the short rows in class order (one per wave).
// Chunk sums go to partial[chunk id][column] (leading dimension ldp).
template <int LPR, int V, typename TI, typename TO>
__global__ __launch_bounds__(256) void spmm_kernel(const int64_t* __restrict__ rowptr, const int32_t* __restrict__ colidx,
                                                   const float* __restrict__ ew, const float* __restrict__ dinv,
                                                   const TI* __restrict__ T,
                                                   int64_t ldt, TO* __restrict__ out, int64_t ldo, int width,
                                                   int64_t n_short, const int32_t* __restrict__ row_order, int epi,
                                                   float slope, const TI* __restrict__ aux, int64_t ldaux,
                                                   int chunk_blocks, const int32_t* __restrict__ chunk_perm,
                                                   const int32_t* __restrict__ chunk_row,
                                                   const int32_t* __restrict__ chunk_begin, int n_chunks,
                                                   float* __restrict__ partial, int64_t ldp) {
  const int lane = threadIdx.x & 63;
  const int c = blockIdx.y * (LPR * V) + (lane % LPR) * V;
  const bool active = c < width;
  float acc[V];
  if ((int)blockIdx.x < chunk_blocks) {
    const int e = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (e >= n_chunks) return;
    const int ch = chunk_perm[e];
    const int64_t i = chunk_row[ch];
    const int64_t begin = rowptr[i] + chunk_begin[ch];
    const int64_t row_end = rowptr[i + 1];
    const int64_t end = begin + kLongRow < row_end ? begin + kLongRow : row_end;
    gather_sum<LPR, V, TI>(colidx, ew, T, ldt, begin, end, c, active, acc);
    if (active && lane < LPR) {
#pragma unroll
      for (int k = 0; k < V; ++k)
        if (c + k < width) partial[(int64_t)ch * ldp + c + k] = acc[k];
    }
    return;
  }
  const int64_t slot = (int64_t)(blockIdx.x - chunk_blocks) * 4 + (threadIdx.x >> 6);
  if (slot >= n_short) return;
  const int64_t i = row_order[slot];
  gather_sum<LPR, V, TI>(colidx, ew, T, ldt, rowptr[i], rowptr[i + 1], c, active, acc);
  if (active && lane < LPR) {
    const float di = dinv[i];
#pragma unroll
    for (int k = 0; k < V; ++k)
      if (c + k < width) store_elem<TI, TO>(out, ldo, i, c + k, di * acc[k], epi, slope, aux, ldaux);
  }
}

// Adds the chunk sums of the long rows; the order of the additions depends only on the row's chunk count k.
// Rows with k <= kWaveReduce: one wave per (row, slab of 256 columns) adds the chunks in chunk order.
// Rows with more chunks: one block per (row, slab of 64 columns); the chunks are cut into four contiguous runs,
// one per wave, each added in chunk order, then the four run sums are added in run order.
template <typename TI, typename TO>
__global__ __launch_bounds__(256) void spmm_reduce_few(const int64_t* __restrict__ rowptr,
                                                       const float* __restrict__ dinv,
                                                       const int32_t* __restrict__ long_row,
                                                       const int32_t* __restrict__ long_first, int n_long,
                                                       const float* __restrict__ partial, int64_t ldp, int width,
                                                       TO* __restrict__ out, int64_t ldo, int epi, float slope,
                                                       const TI* __restrict__ aux, int64_t ldaux) {
  const int slot = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (slot >= n_long) return;
  const int64_t i = long_row[slot];
  const int64_t k = (rowptr[i + 1] - rowptr[i] + kLongRow - 1) / kLongRow;
  if (k > kWaveReduce) return;
  const int c = blockIdx.y * 256 + (threadIdx.x & 63) * 4;
  if (c >= width) return;
  const float* p = partial + (int64_t)long_first[slot] * ldp + c;      // ldp is a multiple of 4: 16-byte aligned
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  int64_t q = 0;
  for (; q + 8 <= k; q += 8) {
    float4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = *reinterpret_cast<const float4*>(p + (q + u) * ldp);
#pragma unroll
    for (int u = 0; u < 8; ++u) { s.x += v[u].x; s.y += v[u].y; s.z += v[u].z; s.w += v[u].w; }
  }
  for (; q < k; ++q) {
    const float4 v = *reinterpret_cast<const float4*>(p + q * ldp);
    s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
  }
  const float di = dinv[i];
  const float r[4] = {s.x, s.y, s.z, s.w};
#pragma unroll
  for (int u = 0; u < 4; ++u)
    if (c + u < width) store_elem<TI, TO>(out, ldo, i, c + u, di * r[u], epi, slope, aux, ldaux);
}

template <typename TI, typename TO>
__global__ __launch_bounds__(256) void spmm_reduce_many(const int64_t* __restrict__ rowptr,
                                                        const float* __restrict__ dinv,
                                                        const int32_t* __restrict__ long_row,
                                                        const int32_t* __restrict__ long_first,
                                                        const int32_t* __restrict__ many_slot,
                                                        const float* __restrict__ partial, int64_t ldp, int width,
                                                        TO* __restrict__ out, int64_t ldo, int epi, float slope,
                                                        const TI* __restrict__ aux, int64_t ldaux) {
  __shared__ float run_sum[4][64];
  const int slot = many_slot[blockIdx.x];             // only the rows of more than kWaveReduce chunks are launched
  const int64_t i = long_row[slot];
  const int64_t k = (rowptr[i + 1] - rowptr[i] + kLongRow - 1) / kLongRow;
  const int64_t first = long_first[slot];
  const int lane = threadIdx.x & 63, run = threadIdx.x >> 6;
  const int64_t q0 = first + run * k / 4, q1 = first + (run + 1) * k / 4;
  const int c = blockIdx.y * 64 + lane;
  float s = 0.f;
  if (c < width) {
    const float* p = partial + c;
    int64_t q = q0;
    for (; q + 8 <= q1; q += 8) {
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = p[(q + u) * ldp];
#pragma unroll
      for (int u = 0; u < 8; ++u) s += v[u];
    }
    for (; q < q1; ++q) s += p[q * ldp];
  }
  run_sum[run][lane] = s;
  __syncthreads();
  if (run == 0 && c < width) {
    const float v = ((run_sum[0][lane] + run_sum[1][lane]) + run_sum[2][lane]) + run_sum[3][lane];
    store_elem<TI, TO>(out, ldo, i, c, dinv[i] * v, epi, slope, aux, ldaux);
  }
}

constexpr unsigned kCapLdsBytes = 32000;      // five blocks (20 waves) per CU out of 160 KB

template <int LPR, int V, typename TI, typename TO>
int launch(const gad_graph* g, const TI* T, int64_t ldt, TO* out, int64_t ldo, int width, const Epi& e, float* partial,
           hipStream_t s) {
  const TI* aux = static_cast<const TI*>(e.aux);
  const int64_t ldp = round_up(width, 4);
  GAD_GRID_CHECK(ceil_div(g->n_short, 4) + ceil_div(g->n_chunks, 4), 256);
  const unsigned row_blocks = (unsigned)ceil_div(g->n_short, 4);
  const unsigned chunk_blocks = (unsigned)ceil_div(g->n_chunks, 4);
  const dim3 grid(chunk_blocks + row_blocks, (unsigned)ceil_div(width, LPR * V));
  // float32 rows of 129 - 256 columns (1 KB per gathered row): 20 waves per CU finish sooner than the 32 that fit,
  // presumably because fewer rows in flight push each other out of L2 less often (products_part 4.33 -> 4.21 ms,
  // whole_graph 16.68 -> 16.50, reddit_part 0.322 -> 0.312; 16 waves: 4.30, 12 waves: 4.62).  Narrower rows need every
  // slot (width 100: 2.12 -> 2.21 ms at 20 waves), bfloat16 rows of 1 KB gain nothing (30.3 -> 30.9 ms), and two
  // column slabs lose 0.5 %.  The cap is a reservation of LDS the kernel never touches; it is left off when another
  // kernel that needs LDS shares the GPU (the weight gradient beside a backward product would have to wait).
  const unsigned cap_lds = sizeof(TI) == 4 && LPR == 64 && width <= 256 && !e.shares_gpu ? kCapLdsBytes : 0u;
  spmm_kernel<LPR, V, TI, TO><<<grid, 256, cap_lds, s>>>(g->rowptr, g->colidx, g->ew, g->dinv, T, ldt, out, ldo, width,
                                                         g->n_short, g->row_order, e.kind, e.slope, aux, e.ldaux,
                                                         (int)chunk_blocks, g->chunk_perm, g->chunk_row, g->chunk_begin,
                                                         g->n_chunks, partial, ldp);
  GAD_LAUNCH_CHECK();
  if (g->n_long > 0) {
    spmm_reduce_few<TI, TO><<<dim3((unsigned)ceil_div(g->n_long, 4), (unsigned)ceil_div(width, 256)), 256, 0, s>>>(
        g->rowptr, g->dinv, g->long_row, g->long_first, g->n_long, partial, ldp, width, out, ldo, e.kind, e.slope, aux,
        e.ldaux);
    GAD_LAUNCH_CHECK();
    if (g->n_many > 0) {
      spmm_reduce_many<TI, TO><<<dim3((unsigned)g->n_many, (unsigned)ceil_div(width, 64)), 256, 0, s>>>(
          g->rowptr, g->dinv, g->long_row, g->long_first, g->many_slot, partial, ldp, width, out, ldo, e.kind, e.slope,
          aux, e.ldaux);
      GAD_LAUNCH_CHECK();
    }
  }
  return GAD_OK;
}

template <typename TI, typename TO>
int spmm_typed(const gad_graph* g, const TI* T, int64_t ldt, TO* out, int64_t ldo, int width, const Epi& e,
               float* partial, hipStream_t s) {
  constexpr int VEC = 16 / (int)sizeof(TI);      // elements per 16-byte load
  const bool vec = (ldt % VEC == 0) && ((reinterpret_cast<uintptr_t>(T) & 15u) == 0);
  const int lanes = vec ? (width + VEC - 1) / VEC : width;
#define GAD_SPMM_CASE(L)                                                                                   \
  if (lanes <= L)                                                                                          \
    return vec ? launch<L, VEC, TI, TO>(g, T, ldt, out, ldo, width, e, partial, s)                  \
               : launch<L, 1, TI, TO>(g, T, ldt, out, ldo, width, e, partial, s);
  GAD_SPMM_CASE(4)
  GAD_SPMM_CASE(8)
  GAD_SPMM_CASE(16)
  GAD_SPMM_CASE(32)
#undef GAD_SPMM_CASE
  return vec ? launch<64, VEC, TI, TO>(g, T, ldt, out, ldo, width, e, partial, s)
             : launch<64, 1, TI, TO>(g, T, ldt, out, ldo, width, e, partial, s);
}

}  // namespace

size_t spmm_partial_floats(const gad_graph* g, int width) { return (size_t)g->n_chunks * (size_t)round_up(width, 4); }

int spmm(const gad_graph* g, const void* T, int64_t ldt, gad_dtype t_in, void* out, int64_t ldo, gad_dtype t_out,
         int width, const Epi& e, float* partial, hipStream_t s) {
  if (g->n == 0 || width == 0) return GAD_OK;
  if (g->n_chunks > 0 && !partial) return set_error(GAD_ERR_NULL, "SpMM needs a buffer for the chunk sums of the long rows");
  if (t_in == GAD_F32 && t_out == GAD_F32)
    return spmm_typed<float, float>(g, (const float*)T, ldt, (float*)out, ldo, width, e, partial, s);
  if (t_in == GAD_BF16 && t_out == GAD_BF16)
    return spmm_typed<bf16_t, bf16_t>(g, (const bf16_t*)T, ldt, (bf16_t*)out, ldo, width, e, partial, s);
  if (t_in == GAD_BF16 && t_out == GAD_F32)
    return spmm_typed<bf16_t, float>(g, (const bf16_t*)T, ldt, (float*)out, ldo, width, e, partial, s);
  return set_error(GAD_ERR_UNSUPPORTED, "SpMM from float32 storage to bfloat16 storage is not implemented");
}

}  // namespace gad
