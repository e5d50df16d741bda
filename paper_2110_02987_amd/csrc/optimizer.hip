// GAD-Optimizer reductions (arXiv 2110.02987, Section 3.4):
//   * variance-based subgraph importance zeta(g'), Eq. 14 and its worked example:
//       zeta = S_pp / (D + beta),  S_pp = sum_{i<j} p_i p_j = (S1^2 - S2) / (2 S1^2) with
//       S1 = sum deg, S2 = sum deg^2 (exact 64-bit integers),  D = sqrt(2 var),
//       var = (1/n) sum_i ||v_i - mean(v)||^2;
//   * weighted global consensus, Eq. 15 (Eq. 11 when all zeta are equal):
//       out = sum_k (zeta_k / sum_j zeta_j) B_k.
// All floating-point reductions are float64 and ordered (per thread, per block, then over blocks), so
// results are reproducible from run to run; the degree sums are exact 64-bit integer sums.
#include <math.h>

#include <mutex>

#include "gad_internal.h"

namespace gad {
namespace {

template <typename T>
__device__ __forceinline__ float to_float(T v);
template <>
__device__ __forceinline__ float to_float<float>(float v) { return v; }
template <>
__device__ __forceinline__ float to_float<uint16_t>(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }  // bfloat16

// Column sums of V[rows x F] over this block's slab of rows -> part[block][F].
// Thread t owns column (t % CW) of row lane (t / CW); CW columns are covered per sweep.
template <typename T, int CW>
__global__ __launch_bounds__(256) void column_sums(const T* __restrict__ V, int64_t n, int F, int64_t slab,
                                                   double* __restrict__ part) {
  constexpr int RL = 256 / CW;
  __shared__ double sm[256];
  const int cl = threadIdx.x % CW, rl = threadIdx.x / CW;
  const int64_t r0 = (int64_t)blockIdx.x * slab;
  const int64_t r1 = r0 + slab < n ? r0 + slab : n;
  for (int c0 = 0; c0 < F; c0 += CW) {
    const int c = c0 + cl;
    double s = 0.0;
    if (c < F) {
      // four independent partial sums keep four loads in flight; they are combined in a fixed order
      double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
      int64_t r = r0 + rl;
      for (; r + 3 * RL < r1; r += 4 * RL) {
        s0 += (double)to_float<T>(V[r * F + c]);
        s1 += (double)to_float<T>(V[(r + RL) * F + c]);
        s2 += (double)to_float<T>(V[(r + 2 * RL) * F + c]);
        s3 += (double)to_float<T>(V[(r + 3 * RL) * F + c]);
      }
      for (; r < r1; r += RL) s0 += (double)to_float<T>(V[r * F + c]);
      s = (s0 + s1) + (s2 + s3);
    }
    sm[threadIdx.x] = s;
    __syncthreads();
    if (rl == 0 && c < F) {
      double tot = 0.0;
      for (int k = 0; k < RL; ++k) tot += sm[k * CW + cl];
      part[(int64_t)blockIdx.x * F + c] = tot;
    }
    __syncthreads();
  }
}

// One wave per column: lane l adds the partial sums of slabs l, l + 64, ..., then a fixed shuffle tree.
__global__ __launch_bounds__(256) void column_means(const double* __restrict__ part, int n_blocks, int F, int64_t n,
                                                    double* __restrict__ mean) {
  const int c = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (c >= F) return;                     // whole waves leave together
  double s = 0.0;
  for (int b = lane; b < n_blocks; b += 64) s += part[(int64_t)b * F + c];
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
  if (lane == 0) mean[c] = s / (double)n;
}

// r_i = ||v_i - mean||^2 (16-lane group per row, kDevRows rows per block in passes of 16), block sums of r_i in
// row order, and the integer degree sums.
constexpr int kDevRows = 256;

template <typename T>
__global__ __launch_bounds__(256) void deviations(const T* __restrict__ V, int64_t n, int F,
                                                  const double* __restrict__ mean, const int32_t* __restrict__ deg,
                                                  float* __restrict__ per_node, double* __restrict__ block_r,
                                                  unsigned long long* __restrict__ block_d1,
                                                  unsigned long long* __restrict__ block_d2) {
  __shared__ double sm_r[kDevRows];
  __shared__ unsigned long long sm_d1[4], sm_d2[4];
  const int grp = threadIdx.x >> 4, l = threadIdx.x & 15;
  const int64_t base = (int64_t)blockIdx.x * kDevRows;
  for (int pass = 0; pass < kDevRows / 16; ++pass) {
    const int64_t i = base + pass * 16 + grp;
    double r = 0.0;
    if (i < n) {
      for (int c = l; c < F; c += 16) {
        const double d = (double)to_float<T>(V[i * F + c]) - mean[c];
        r += d * d;
      }
    }
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) r += __shfl_xor(r, o, 64);
    if (l == 0) {
      sm_r[pass * 16 + grp] = i < n ? r : 0.0;
      if (i < n && per_node) per_node[i] = (float)r;
    }
  }
  // degree sums: thread t takes row base + t (exact integers: the order does not matter)
  unsigned long long d1 = 0, d2 = 0;
  {
    const int64_t j = base + threadIdx.x;
    if (j < n) {
      const unsigned long long d = (unsigned long long)deg[j];
      d1 = d;
      d2 = d * d;
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    d1 += __shfl_xor(d1, o, 64);
    d2 += __shfl_xor(d2, o, 64);
  }
  if ((threadIdx.x & 63) == 0) {
    sm_d1[threadIdx.x >> 6] = d1;
    sm_d2[threadIdx.x >> 6] = d2;
  }
  __syncthreads();
  if (threadIdx.x < 64) {                 // row sums: lane t adds rows t, t + 64, ..., then a fixed shuffle tree
    double s = (sm_r[threadIdx.x] + sm_r[threadIdx.x + 64]) + (sm_r[threadIdx.x + 128] + sm_r[threadIdx.x + 192]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    if (threadIdx.x == 0) {
      block_r[blockIdx.x] = s;
      block_d1[blockIdx.x] = sm_d1[0] + sm_d1[1] + sm_d1[2] + sm_d1[3];
      block_d2[blockIdx.x] = sm_d2[0] + sm_d2[1] + sm_d2[2] + sm_d2[3];
    }
  }
}

static_assert(kDevRows == 256, "one degree per thread and four rows per lane in the block sum");

__global__ __launch_bounds__(256) void finalize_zeta(const double* __restrict__ block_r, int64_t n_blocks, int64_t n,
                                                     const unsigned long long* __restrict__ block_d1,
                                                     const unsigned long long* __restrict__ block_d2, double beta,
                                                     double* __restrict__ out3) {
  __shared__ double sm[256];
  __shared__ unsigned long long sd1[256], sd2[256];
  double s = 0.0;
  unsigned long long a1 = 0, a2 = 0;
  for (int64_t k = threadIdx.x; k < n_blocks; k += 256) {
    s += block_r[k];
    a1 += block_d1[k];
    a2 += block_d2[k];
  }
  sm[threadIdx.x] = s;
  sd1[threadIdx.x] = a1;
  sd2[threadIdx.x] = a2;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) {
      sm[threadIdx.x] += sm[threadIdx.x + o];
      sd1[threadIdx.x] += sd1[threadIdx.x + o];
      sd2[threadIdx.x] += sd2[threadIdx.x + o];
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const double var = sm[0] / (double)n;
    const unsigned long long s1 = sd1[0], s2 = sd2[0];
    double spp = 0.0;
    if (s1 != 0) {
      const double sq = (double)s1 * (double)s1;
      spp = 0.5 * (1.0 - (double)s2 / sq);
    }
    out3[0] = spp / (sqrt(2.0 * var) + beta);
    out3[1] = spp;
    out3[2] = var;
  }
}

struct ConsensusArgs {
  const float* buf[kMaxConsensus];
  double w[kMaxConsensus];
};

// `out` may alias any of the inputs: every element is read from all buffers before it is written.
__global__ __launch_bounds__(256) void consensus_kernel(ConsensusArgs a, int K, int64_t n, float* out) {
  const int64_t e = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (e >= n) return;
  double s = 0.0;
  for (int k = 0; k < K; ++k) s += a.w[k] * (double)a.buf[k][e];
  out[e] = (float)s;
}

// Eq. 15 followed by the update of Eq. 16: params <- params - eta * sum_k w_k g_k; the averaged gradient itself goes
// to avg_out when it is not NULL.
__global__ __launch_bounds__(256) void consensus_update_kernel(ConsensusArgs a, int K, int64_t n, float eta,
                                                               float* __restrict__ params, float* avg_out) {
  const int64_t e = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (e >= n) return;
  double s = 0.0;
  for (int k = 0; k < K; ++k) s += a.w[k] * (double)a.buf[k][e];
  if (avg_out) avg_out[e] = (float)s;
  params[e] = (float)((double)params[e] - (double)eta * s);
}

// `red`: reduction buffer of at least kVarBlocks * F + F + 3 * ceil(n / kDevRows) 8-byte words.  Every word that a
// kernel reads is written by an earlier kernel of the same call, so the buffer needs no clearing between calls.
template <typename T>
int variance_t(const gad_graph* g, const T* V, int F, double beta, double* out3, float* per_node, double* red,
               hipStream_t s) {
  const int64_t n = g->n;
  // scratch layout (8-byte words): part[kVarBlocks x F] | mean[F] | block_r[nb] | block_d1[nb] | block_d2[nb], nb = ceil(n / kDevRows)
  double* part = red;
  double* mean = part + (int64_t)kVarBlocks * F;
  double* block_r = mean + F;
  const int64_t r_blocks = ceil_div(n, kDevRows);
  unsigned long long* block_d1 = reinterpret_cast<unsigned long long*>(block_r + r_blocks);
  unsigned long long* block_d2 = block_d1 + r_blocks;
  int st = column_means_f64(V, n, F, sizeof(T) == 4 ? GAD_F32 : GAD_BF16, part, mean, s);
  if (st != GAD_OK) return st;
  deviations<T><<<(unsigned)r_blocks, 256, 0, s>>>(V, n, F, mean, g->deg, per_node, block_r, block_d1, block_d2);
  GAD_LAUNCH_CHECK();
  finalize_zeta<<<1, 256, 0, s>>>(block_r, r_blocks, n, block_d1, block_d2, beta, out3);
  GAD_LAUNCH_CHECK();
  return GAD_OK;
}

}  // namespace

int column_means_f64(const void* V, int64_t n, int F, gad_dtype dtype, double* part, double* mean, hipStream_t s) {
  int n_blocks = (int)(n < kVarBlocks ? n : kVarBlocks);
  const int64_t slab = ceil_div(n, n_blocks);
  n_blocks = (int)ceil_div(n, slab);
#define GAD_COLSUM(T, CW) column_sums<T, CW><<<n_blocks, 256, 0, s>>>(static_cast<const T*>(V), n, F, slab, part)
  if (dtype == GAD_F32) {
    if (F <= 32) GAD_COLSUM(float, 32); else if (F <= 64) GAD_COLSUM(float, 64);
    else if (F <= 128) GAD_COLSUM(float, 128); else GAD_COLSUM(float, 256);
  } else {
    if (F <= 32) GAD_COLSUM(uint16_t, 32); else if (F <= 64) GAD_COLSUM(uint16_t, 64);
    else if (F <= 128) GAD_COLSUM(uint16_t, 128); else GAD_COLSUM(uint16_t, 256);
  }
#undef GAD_COLSUM
  GAD_LAUNCH_CHECK();
  column_means<<<(unsigned)ceil_div(F, 4), 256, 0, s>>>(part, n_blocks, F, n, mean);
  GAD_LAUNCH_CHECK();
  return GAD_OK;
}

size_t variance_scratch_doubles(int64_t n) {
  return (size_t)kVarBlocks * kMaxWidth + kMaxWidth + 3 * (size_t)ceil_div(n, kDevRows) + 4;
}

int subgraph_variance(const gad_graph* g, const void* V, int F, gad_dtype dtype, double beta, double* out3,
                      float* per_node, hipStream_t s) {
  double* red = g->red_scratch;
  if (dtype == GAD_F32) return variance_t<float>(g, static_cast<const float*>(V), F, beta, out3, per_node, red, s);
  return variance_t<uint16_t>(g, static_cast<const uint16_t*>(V), F, beta, out3, per_node, red, s);
}

// ---- the same reduction for callers that cannot allocate -----------------------------------------------------
// The reduction buffer is a file-scope device array instead of memory of the graph.  Each device that loads the
// library holds its own copy of the array until the process ends; the array's name is only a host-side stand-in, so
// its device address is looked up once per device (with that device current) and every launch takes that address.
namespace {
constexpr size_t kStaticDoubles = (size_t)kVarBlocks * kStaticVarMaxF + kStaticVarMaxF +
                                  3 * (size_t)(kStaticVarMaxN / kDevRows) + 4;     // 4.8 MB
static __device__ __align__(256) double scratch[kStaticDoubles];
constexpr int kMaxDevices = 64;
std::mutex g_static_mu;
double* g_static_ptr[kMaxDevices] = {};     // device address of `scratch` on each device, null until first use there
}  // namespace

int subgraph_variance_static(const gad_graph* g, const void* V, int F, gad_dtype dtype, double beta, double* out3,
                             float* per_node, hipStream_t s) {
  if (F > kStaticVarMaxF || g->n > kStaticVarMaxN)
    return set_error(GAD_ERR_SHAPE, "F = %d or n = %lld beyond what the static reduction buffer holds (F <= %d, n <= %lld)",
                     F, (long long)g->n, kStaticVarMaxF, (long long)kStaticVarMaxN);
  int dev = 0;
  GAD_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return set_error(GAD_ERR_UNSUPPORTED, "device ordinal %d out of range", dev);
  if (dev != g->device) return set_error(GAD_ERR_STATE, "the graph lives on device %d, the current device is %d", g->device, dev);
  double* red = nullptr;
  {
    std::lock_guard<std::mutex> lk(g_static_mu);
    if (!g_static_ptr[dev]) {
      void* p = nullptr;
      GAD_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
      if (!p) return set_error(GAD_ERR_HIP, "the static reduction buffer has no address on device %d", dev);
      g_static_ptr[dev] = static_cast<double*>(p);
    }
    red = g_static_ptr[dev];
  }
  if (dtype == GAD_F32) return variance_t<float>(g, static_cast<const float*>(V), F, beta, out3, per_node, red, s);
  return variance_t<uint16_t>(g, static_cast<const uint16_t*>(V), F, beta, out3, per_node, red, s);
}

int weighted_consensus(const float* const* bufs, int K, const double* w, int64_t n, float* out, hipStream_t s) {
  if (n == 0) return GAD_OK;
  ConsensusArgs a;
  for (int k = 0; k < K; ++k) {
    a.buf[k] = bufs[k];
    a.w[k] = w[k];
  }
  for (int k = K; k < kMaxConsensus; ++k) {
    a.buf[k] = nullptr;
    a.w[k] = 0.0;
  }
  consensus_kernel<<<(unsigned)ceil_div(n, 256), 256, 0, s>>>(a, K, n, out);
  GAD_LAUNCH_CHECK();
  return GAD_OK;
}

int consensus_update(const float* const* bufs, int K, const double* w, int64_t n, float eta, float* params,
                     float* avg_out, hipStream_t s) {
  if (n == 0) return GAD_OK;
  ConsensusArgs a;
  for (int k = 0; k < kMaxConsensus; ++k) {
    a.buf[k] = k < K ? bufs[k] : nullptr;
    a.w[k] = k < K ? w[k] : 0.0;
  }
  consensus_update_kernel<<<(unsigned)ceil_div(n, 256), 256, 0, s>>>(a, K, n, eta, params, avg_out);
  GAD_LAUNCH_CHECK();
  return GAD_OK;
}

}  // namespace gad
