// Row softmax, cross-entropy loss and the gradient seed of the backward pass
// (arXiv 2110.02987, Eq. 8: y^ = softmax(Z); Eq. 9 read as softmax cross-entropy summed over the
// masked nodes; Eq. 10 through the softmax: G = scale * mask * (y^ - onehot(label))).
//
// A 16-lane group owns one row at a time (four rows per wave64 and pass); max and sum go through wave shuffles.
// The loss is summed in float64: per block in a fixed order, then over blocks in a fixed order.
#include <math.h>

#include "dtype.h"
#include "gad_internal.h"

namespace gad {
namespace {

constexpr int kGroup = 16;                 // lanes per row
constexpr int kPasses = 4;                 // rows per group
constexpr int kRowsPerBlock = kPasses * 256 / kGroup;

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

// ITEMS > 0: C <= 16 ITEMS and a lane keeps its logits (and their exponentials) in registers, so a row is read
// once and exponentiated once; ITEMS = 0: any C, the row is re-read from memory (cache) for each of the three sweeps.
template <typename TG, int ITEMS>
__global__ __launch_bounds__(256) void softmax_xent_kernel(const float* __restrict__ Z, int64_t ldz,
                                                           const int32_t* __restrict__ labels,
                                                           const uint8_t* __restrict__ mask, float scale,
                                                           const float* __restrict__ row_scale, int64_t n, int C,
                                                           TG* __restrict__ G, int64_t ldg,
                                                           double* __restrict__ block_partials) {
  __shared__ double row_loss[kRowsPerBlock];
  const int grp = threadIdx.x / kGroup, l = threadIdx.x % kGroup;
  for (int pass = 0; pass < kPasses; ++pass) {
    const int rl = pass * (256 / kGroup) + grp;
    const int64_t i = (int64_t)blockIdx.x * kRowsPerBlock + rl;
    double my_loss = 0.0;
    if (i < n) {
      const float* z = Z + i * ldz;
      const int32_t y = labels[i];
      const bool on = (mask == nullptr || mask[i] != 0) && y >= 0 && y < C;
      const float sc = row_scale ? scale * row_scale[i] : scale;       // per-node weight of the loss (NULL = 1)
      const float g_scale = on ? sc : 0.f;
      float m = -INFINITY, se = 0.f;
      if (ITEMS > 0) {
        float zv[ITEMS > 0 ? ITEMS : 1];
#pragma unroll
        for (int k = 0; k < ITEMS; ++k) {
          const int c = l + k * kGroup;
          zv[k] = c < C ? z[c] : -INFINITY;
          m = fmaxf(m, zv[k]);
        }
        m = group_max(m);
#pragma unroll
        for (int k = 0; k < ITEMS; ++k) {
          zv[k] = expf(zv[k] - m);            // exp(-inf) = 0 for the columns past C
          se += zv[k];
        }
        se = group_sum(se);
        const float inv = 1.f / se;
#pragma unroll
        for (int k = 0; k < ITEMS; ++k) {
          const int c = l + k * kGroup;
          if (c < C) G[i * ldg + c] = from_f32<TG>(g_scale * (zv[k] * inv - (c == y ? 1.f : 0.f)));
        }
      } else {
        for (int c = l; c < C; c += kGroup) m = fmaxf(m, z[c]);
        m = group_max(m);
        for (int c = l; c < C; c += kGroup) se += expf(z[c] - m);
        se = group_sum(se);
        const float inv = 1.f / se;
        for (int c = l; c < C; c += kGroup) {
          const float p = expf(z[c] - m) * inv;
          G[i * ldg + c] = from_f32<TG>(g_scale * (p - (c == y ? 1.f : 0.f)));
        }
      }
      if (on && l == 0) my_loss = (double)sc * ((double)logf(se) + (double)m - (double)z[y]);
    }
    if (l == 0) row_loss[rl] = my_loss;
  }
  __syncthreads();
  if (threadIdx.x < 64) {                  // lane t adds its row; a fixed shuffle tree adds the lanes
    static_assert(kRowsPerBlock == 64, "one row per lane of the first wave");
    double s = row_loss[threadIdx.x];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    if (threadIdx.x == 0) block_partials[blockIdx.x] = s;
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
  const int64_t total = n * width, stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t e = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; e < total; e += stride) {
    const int64_t i = e / width;
    const int c = (int)(e % width);
    out[i * ldo + c] = to_f32<TI>(in[i * ldi + c]);
  }
}

}  // namespace

size_t softmax_partial_doubles(int64_t n) { return (size_t)ceil_div(n, kRowsPerBlock) + 1; }

int softmax_xent(const float* Z, int64_t ldz, const int32_t* labels, const uint8_t* mask, float scale,
                 const float* row_scale, int64_t n, int C, void* G, int64_t ldg, gad_dtype tg, double* block_partials, double* loss_out, hipStream_t s) {
  if (n == 0) return GAD_OK;
  const int64_t blocks = ceil_div(n, kRowsPerBlock);
  GAD_GRID_CHECK(blocks, 256);
#define GAD_SOFTMAX(TG, ITEMS)                                                                                    \
  softmax_xent_kernel<TG, ITEMS><<<(unsigned)blocks, 256, 0, s>>>(Z, ldz, labels, mask, scale, row_scale, n, C, \
                                                                  static_cast<TG*>(G), ldg, block_partials)
#define GAD_SOFTMAX_C(TG)                                                                                  \
  do {                                                                                                     \
    if (C <= 16) GAD_SOFTMAX(TG, 1); else if (C <= 32) GAD_SOFTMAX(TG, 2); else if (C <= 64) GAD_SOFTMAX(TG, 4); \
    else if (C <= 128) GAD_SOFTMAX(TG, 8); else GAD_SOFTMAX(TG, 0);                                        \
  } while (0)
  if (tg == GAD_F32) GAD_SOFTMAX_C(float); else GAD_SOFTMAX_C(bf16_t);
#undef GAD_SOFTMAX_C
#undef GAD_SOFTMAX
  GAD_LAUNCH_CHECK();
  if (loss_out) {
    sum_doubles<<<1, 256, 0, s>>>(block_partials, blocks, loss_out);
    GAD_LAUNCH_CHECK();
  }
  return GAD_OK;
}

int copy_rows(const void* in, int64_t ldi, gad_dtype ti, float* out, int64_t ldo, int64_t n, int width, hipStream_t s) {
  if (n == 0 || width == 0) return GAD_OK;
  const int64_t want = ceil_div(n * width, 256);
  const unsigned blocks = (unsigned)(want < (1 << 22) ? want : (1 << 22));      // the kernel strides over the rest
  if (ti == GAD_F32)
    copy_rows_kernel<float><<<blocks, 256, 0, s>>>((const float*)in, ldi, out, ldo, n, width);
  else
    copy_rows_kernel<bf16_t><<<blocks, 256, 0, s>>>((const bf16_t*)in, ldi, out, ldo, n, width);
  GAD_LAUNCH_CHECK();
  return GAD_OK;
}

}  // namespace gad
