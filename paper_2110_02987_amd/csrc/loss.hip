// Row softmax, cross-entropy loss and the gradient seed of the backward pass
// (arXiv 2110.02987, Eq. 8: y^ = softmax(Z); Eq. 9 read as softmax cross-entropy summed over the
// masked nodes; Eq. 10 through the softmax: G = scale * mask * (y^ - onehot(label))).
//
// A 16-lane group owns one row (four rows per wave64); max and sum go through wave shuffles.
// The loss is summed in float64: per block in a fixed order, then over blocks in a fixed order.
#include <math.h>

#include "dtype.h"
#include "gad_internal.h"

namespace gad {
namespace {

constexpr int kGroup = 16;                 // lanes per row
constexpr int kRowsPerBlock = 256 / kGroup;

__device__ __forceinline__ float group_max(float v) {
#pragma unroll
  for (int o = kGroup / 2; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float group_sum(float v) {
#pragma unroll
  for (int o = kGroup / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

template <typename TG>
__global__ __launch_bounds__(256) void softmax_xent_kernel(const float* __restrict__ Z, int64_t ldz,
                                                           const int32_t* __restrict__ labels,
                                                           const uint8_t* __restrict__ mask, float scale,
                                                           const float* __restrict__ row_scale, int64_t n, int C,
                                                           TG* __restrict__ G, int64_t ldg,
                                                           double* __restrict__ block_partials) {
  __shared__ double row_loss[kRowsPerBlock];
  const int grp = threadIdx.x / kGroup, l = threadIdx.x % kGroup;
  const int64_t i = (int64_t)blockIdx.x * kRowsPerBlock + grp;
  double my_loss = 0.0;
  if (i < n) {
    const float* z = Z + i * ldz;
    float m = -INFINITY;
    for (int c = l; c < C; c += kGroup) m = fmaxf(m, z[c]);
    m = group_max(m);
    float se = 0.f;
    for (int c = l; c < C; c += kGroup) se += expf(z[c] - m);
    se = group_sum(se);
    const int32_t y = labels[i];
    const bool on = (mask == nullptr || mask[i] != 0) && y >= 0 && y < C;
    const float sc = row_scale ? scale * row_scale[i] : scale;       // per-node weight of the loss (NULL = 1)
    const float g_scale = on ? sc : 0.f;
    const float inv = 1.f / se;
    for (int c = l; c < C; c += kGroup) {
      const float p = expf(z[c] - m) * inv;
      G[i * ldg + c] = from_f32<TG>(g_scale * (p - (c == y ? 1.f : 0.f)));
    }
    if (on && l == 0) my_loss = (double)sc * ((double)logf(se) + (double)m - (double)z[y]);
  }
  if (l == 0) row_loss[grp] = my_loss;
  __syncthreads();
  if (threadIdx.x == 0) {
    double s = 0.0;
    for (int r = 0; r < kRowsPerBlock; ++r) s += row_loss[r];
    block_partials[blockIdx.x] = s;
  }
}

// Single block: sums `count` doubles in a fixed order (strided per thread, then a fixed tree).
__global__ __launch_bounds__(256) void sum_doubles(const double* __restrict__ v, int64_t count,
                                                   double* __restrict__ out) {
  __shared__ double sm[256];
  double s = 0.0;
  for (int64_t k = threadIdx.x; k < count; k += 256) s += v[k];
  sm[threadIdx.x] = s;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) sm[threadIdx.x] += sm[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) out[0] = sm[0];
}

template <typename TI>
__global__ void copy_rows_kernel(const TI* __restrict__ in, int64_t ldi, float* __restrict__ out, int64_t ldo,
                                 int64_t n, int width) {
  const int64_t e = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (e >= n * width) return;
  const int64_t i = e / width;
  const int c = (int)(e % width);
  out[i * ldo + c] = to_f32<TI>(in[i * ldi + c]);
}

}  // namespace

size_t softmax_partial_doubles(int64_t n) { return (size_t)ceil_div(n, kRowsPerBlock) + 1; }

int softmax_xent(const float* Z, int64_t ldz, const int32_t* labels, const uint8_t* mask, float scale,
                 const float* row_scale, int64_t n, int C, void* G, int64_t ldg, gad_dtype tg, double* block_partials, double* loss_out, hipStream_t s) {
  if (n == 0) return GAD_OK;
  const int64_t blocks = ceil_div(n, kRowsPerBlock);
  if (tg == GAD_F32)
    softmax_xent_kernel<float><<<(unsigned)blocks, 256, 0, s>>>(Z, ldz, labels, mask, scale, row_scale, n, C, (float*)G,
                                                                ldg, block_partials);
  else
    softmax_xent_kernel<bf16_t><<<(unsigned)blocks, 256, 0, s>>>(Z, ldz, labels, mask, scale, row_scale, n, C,
                                                                 (bf16_t*)G, ldg, block_partials);
  GAD_LAUNCH_CHECK();
  if (loss_out) {
    sum_doubles<<<1, 256, 0, s>>>(block_partials, blocks, loss_out);
    GAD_LAUNCH_CHECK();
  }
  return GAD_OK;
}

int copy_rows(const void* in, int64_t ldi, gad_dtype ti, float* out, int64_t ldo, int64_t n, int width, hipStream_t s) {
  if (n == 0 || width == 0) return GAD_OK;
  const unsigned blocks = (unsigned)ceil_div(n * width, 256);
  if (ti == GAD_F32)
    copy_rows_kernel<float><<<blocks, 256, 0, s>>>((const float*)in, ldi, out, ldo, n, width);
  else
    copy_rows_kernel<bf16_t><<<blocks, 256, 0, s>>>((const bf16_t*)in, ldi, out, ldo, n, width);
  GAD_LAUNCH_CHECK();
  return GAD_OK;
}

}  // namespace gad
