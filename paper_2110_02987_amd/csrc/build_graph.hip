// Augmented-subgraph CSR build and normalisation on the GPU (gfx950).
//
// g' = (v + v', e + e') -- Algorithm 1 (last step) and Algorithm 2 (Require) of arXiv 2110.02987 --
// becomes the CSR of A + I, A being the induced simple undirected graph on local ++ halo nodes.
// Steps: id -> row lookup table; every kept pair emits the two 64-bit keys (row << bits | col) and
// (col << bits | row), every row emits its self-loop key; an LSD radix sort (8-bit digits, stable
// ranking by wave ballots) orders the keys; adjacent-unique + exclusive scan compacts them into
// colidx and marks row starts in rowptr.  The result depends only on the *set* of keys, so the
// unordered atomic append of the emit step does not affect it: the CSR is deterministic.
#include <math.h>

#include <vector>

#include "gad_internal.h"

namespace gad {
namespace {

constexpr int kThreads = 256;
constexpr int kItems = 16;                      // keys per thread in a radix / scan tile
constexpr int kTile = kThreads * kItems;        // 4096

__device__ __forceinline__ uint64_t lanemask_lt() {
  return (1ull << (threadIdx.x & 63)) - 1ull;
}

// ------------------------------------------------------------------------------------------------
// exclusive scan of a uint32 array (three kernels: tile sums, scan of tile sums, apply)
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v) {
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    uint32_t o = __shfl_up(v, d, 64);
    if (lane >= d) v += o;
  }
  return v;
}

// Block-wide exclusive scan of one value per thread (256 threads); returns the exclusive prefix and
// the block total through `total`.
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* total, uint32_t* smem /*[5]*/) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  uint32_t inc = wave_inclusive_scan(v);
  if (lane == 63) smem[w] = inc;
  __syncthreads();
  uint32_t base = 0, tot = 0;
#pragma unroll
  for (int k = 0; k < kThreads / 64; ++k) {
    uint32_t s = smem[k];
    if (k < w) base += s;
    tot += s;
  }
  __syncthreads();
  *total = tot;
  return base + inc - v;
}

__global__ __launch_bounds__(kThreads) void scan_tile_sums(const uint32_t* __restrict__ in, uint32_t n,
                                                          uint32_t* __restrict__ tile_sum) {
  __shared__ uint32_t smem[8];
  const uint32_t base = blockIdx.x * (uint32_t)kTile + threadIdx.x * kItems;
  uint32_t s = 0;
#pragma unroll
  for (int i = 0; i < kItems; ++i)
    if (base + i < n) s += in[base + i];
  uint32_t tot;
  block_exclusive_scan(s, &tot, smem);
  if (threadIdx.x == 0) tile_sum[blockIdx.x] = tot;
}

// One block scans the tile sums in place (exclusive) and writes the grand total to total_out[0].
__global__ __launch_bounds__(kThreads) void scan_of_tile_sums(uint32_t* __restrict__ tile_sum, uint32_t n_tiles,
                                                             uint32_t* __restrict__ total_out) {
  __shared__ uint32_t smem[8];
  uint32_t carry = 0;
  for (uint32_t s = 0; s < n_tiles; s += kThreads) {
    uint32_t i = s + threadIdx.x;
    uint32_t v = i < n_tiles ? tile_sum[i] : 0u;
    uint32_t tot;
    uint32_t ex = block_exclusive_scan(v, &tot, smem);
    if (i < n_tiles) tile_sum[i] = carry + ex;
    carry += tot;
  }
  if (threadIdx.x == 0) total_out[0] = carry;
}

__global__ __launch_bounds__(kThreads) void scan_apply(uint32_t* __restrict__ data, uint32_t n,
                                                      const uint32_t* __restrict__ tile_excl) {
  __shared__ uint32_t smem[8];
  const uint32_t base = blockIdx.x * (uint32_t)kTile + threadIdx.x * kItems;
  uint32_t v[kItems];
  uint32_t s = 0;
#pragma unroll
  for (int i = 0; i < kItems; ++i) {
    v[i] = base + i < n ? data[base + i] : 0u;
    s += v[i];
  }
  uint32_t tot;
  uint32_t ex = block_exclusive_scan(s, &tot, smem) + tile_excl[blockIdx.x];
#pragma unroll
  for (int i = 0; i < kItems; ++i) {
    if (base + i < n) data[base + i] = ex;
    ex += v[i];
  }
}

// data[0..n) <- exclusive scan; total_out[0] <- sum.  tile_tmp must hold ceil(n / kTile) uint32.
int exclusive_scan_u32(uint32_t* data, uint32_t n, uint32_t* tile_tmp, uint32_t* total_out, hipStream_t s) {
  const uint32_t n_tiles = (uint32_t)ceil_div(n, kTile);
  if (n_tiles == 0) {
    GAD_HIP(hipMemsetAsync(total_out, 0, sizeof(uint32_t), s));
    return GAD_OK;
  }
  scan_tile_sums<<<n_tiles, kThreads, 0, s>>>(data, n, tile_tmp);
  GAD_LAUNCH_CHECK();
  scan_of_tile_sums<<<1, kThreads, 0, s>>>(tile_tmp, n_tiles, total_out);
  GAD_LAUNCH_CHECK();
  scan_apply<<<n_tiles, kThreads, 0, s>>>(data, n, tile_tmp);
  GAD_LAUNCH_CHECK();
  return GAD_OK;
}

// ------------------------------------------------------------------------------------------------
// id lookup table and key emission
// ------------------------------------------------------------------------------------------------
__global__ void fill_i32(int32_t* p, int64_t n, int32_t v) {
  int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// flags[0]: an id out of range; flags[1]: an id seen twice
__global__ void assign_rows(const int64_t* __restrict__ local_ids, int64_t n_local,
                            const int64_t* __restrict__ halo_ids, int64_t n_halo, int64_t n_global,
                            int32_t* __restrict__ lut, uint32_t* __restrict__ flags) {
  int64_t k = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (k >= n_local + n_halo) return;
  int64_t id = k < n_local ? local_ids[k] : halo_ids[k - n_local];
  if (id < 0 || id >= n_global) {
    flags[0] = 1u;
    return;
  }
  int32_t old = atomicCAS(&lut[id], -1, (int32_t)k);
  if (old != -1) flags[1] = 1u;
}

// keys[0..n) = self loops; kept pairs are appended behind them (two keys each) through counter[0].
// A block takes kEmitItems * kThreads consecutive pairs and reserves the room for all its keys with ONE atomic add
// (an add per wave made the single counter the bottleneck: 2 M serialised atomics for 134 M pairs).  Where a pair's
// keys land depends on the order of those adds; the sort that follows makes the result independent of it.
constexpr int kEmitItems = 8;

__global__ __launch_bounds__(kThreads) void emit_keys(const int64_t* __restrict__ src, const int64_t* __restrict__ dst,
                                                     int64_t n_edges, int64_t n_global,
                                                     const int32_t* __restrict__ lut, int64_t n, int bits,
                                                     uint64_t* __restrict__ keys, uint32_t* __restrict__ counter) {
  static_assert(kThreads == 256, "four waves per block");
  __shared__ uint32_t wave_count[kEmitItems][4];
  __shared__ uint32_t block_base;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t first = (int64_t)blockIdx.x * (kEmitItems * kThreads);
  uint64_t r[kEmitItems], c[kEmitItems];
  uint32_t rank[kEmitItems];                 // position among the kept pairs of this wave and item
  bool valid[kEmitItems];
#pragma unroll
  for (int i = 0; i < kEmitItems; ++i) {
    const int64_t e = first + (int64_t)i * kThreads + threadIdx.x;
    if (e < n) keys[e] = ((uint64_t)e << bits) | (uint64_t)e;
    valid[i] = false;
    r[i] = c[i] = 0;
    if (e < n_edges) {
      const int64_t a = src[e], b = dst[e];
      if (a >= 0 && a < n_global && b >= 0 && b < n_global) {
        const int32_t ra = lut[a], rb = lut[b];
        valid[i] = ra >= 0 && rb >= 0 && ra != rb;
        r[i] = (uint64_t)(uint32_t)ra;
        c[i] = (uint64_t)(uint32_t)rb;
      }
    }
    const uint64_t m = __ballot(valid[i]);
    rank[i] = (uint32_t)__popcll(m & lanemask_lt());
    if (lane == 0) wave_count[i][wave] = (uint32_t)__popcll(m);
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t total = 0;
#pragma unroll
    for (int i = 0; i < kEmitItems; ++i)
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const uint32_t cnt = wave_count[i][w];
        wave_count[i][w] = total;            // exclusive offset of (item, wave) inside the block
        total += cnt;
      }
    block_base = total ? atomicAdd(counter, 2u * total) : 0u;
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < kEmitItems; ++i) {
    if (valid[i]) {
      uint64_t* o = keys + n + block_base + 2u * (wave_count[i][wave] + rank[i]);
      o[0] = (r[i] << bits) | c[i];
      o[1] = (c[i] << bits) | r[i];
    }
  }
}

// ------------------------------------------------------------------------------------------------
// LSD radix sort of uint64 keys, 8 bits per pass
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void radix_histogram(const uint64_t* __restrict__ keys, uint32_t n_keys,
                                                           int shift, uint32_t n_tiles, uint32_t* __restrict__ hist) {
  __shared__ uint32_t h[256];
  h[threadIdx.x] = 0;
  __syncthreads();
  const uint32_t base = blockIdx.x * (uint32_t)kTile;
#pragma unroll
  for (int i = 0; i < kItems; ++i) {
    uint32_t idx = base + i * kThreads + threadIdx.x;
    if (idx < n_keys) atomicAdd(&h[(uint32_t)(keys[idx] >> shift) & 255u], 1u);
  }
  __syncthreads();
  hist[threadIdx.x * n_tiles + blockIdx.x] = h[threadIdx.x];   // digit-major: scan order = (digit, tile)
}

__global__ __launch_bounds__(kThreads) void radix_scatter(const uint64_t* __restrict__ in, uint64_t* __restrict__ out,
                                                         uint32_t n_keys, int shift, uint32_t n_tiles,
                                                         const uint32_t* __restrict__ offs) {
  __shared__ uint32_t running[256];          // next free output slot of each digit for this tile
  __shared__ uint32_t wcnt[kThreads / 64][256];
  const int t = threadIdx.x, w = t >> 6;
  running[t] = offs[t * n_tiles + blockIdx.x];
#pragma unroll
  for (int k = 0; k < kThreads / 64; ++k) wcnt[k][t] = 0;
  __syncthreads();
  const uint32_t base = blockIdx.x * (uint32_t)kTile;
  const uint64_t lt = lanemask_lt();
  for (int i = 0; i < kItems; ++i) {
    const uint32_t idx = base + i * kThreads + t;
    const bool valid = idx < n_keys;
    const uint64_t key = valid ? in[idx] : 0ull;
    const uint32_t d = (uint32_t)(key >> shift) & 255u;
    // lanes of this wave holding the same digit
    uint64_t peers = __ballot(valid);
#pragma unroll
    for (int b = 0; b < 8; ++b) {
      const bool bit = (d >> b) & 1u;
      const uint64_t bal = __ballot(valid && bit);
      peers &= bit ? bal : ~bal;
    }
    const uint32_t rank = (uint32_t)__popcll(peers & lt);
    const uint32_t cnt = (uint32_t)__popcll(peers);
    const bool leader = valid && rank == 0;
    if (leader) wcnt[w][d] = cnt;
    __syncthreads();
    if (valid) {
      uint32_t pos = running[d] + rank;
      for (int k = 0; k < w; ++k) pos += wcnt[k][d];
      out[pos] = key;
    }
    __syncthreads();
    if (leader) {
      atomicAdd(&running[d], cnt);
      wcnt[w][d] = 0;
    }
  }
}

// ------------------------------------------------------------------------------------------------
// unique + CSR assembly
// ------------------------------------------------------------------------------------------------
__global__ void mark_first(const uint64_t* __restrict__ keys, uint32_t n_keys, uint32_t* __restrict__ flag) {
  uint32_t p = blockIdx.x * blockDim.x + threadIdx.x;
  if (p < n_keys) flag[p] = (p == 0 || keys[p] != keys[p - 1]) ? 1u : 0u;
}

__global__ void assemble_csr(const uint64_t* __restrict__ keys, uint32_t n_keys, const uint32_t* __restrict__ pos,
                             int bits, int64_t n, int64_t nnz, int64_t* __restrict__ rowptr,
                             int32_t* __restrict__ colidx) {
  uint32_t p = blockIdx.x * blockDim.x + threadIdx.x;
  if (p == 0) rowptr[n] = nnz;
  if (p >= n_keys) return;
  const uint64_t k = keys[p];
  const uint64_t prev = p ? keys[p - 1] : ~0ull;
  if (p == 0 || k != prev) {
    const uint32_t q = pos[p];
    colidx[q] = (int32_t)(k & ((1ull << bits) - 1ull));
    if (p == 0 || (k >> bits) != (prev >> bits)) rowptr[k >> bits] = (int64_t)q;   // every row has its self loop
  }
}

__global__ void degree_norm(const int64_t* __restrict__ rowptr, int64_t n, int32_t* __restrict__ deg,
                            float* __restrict__ dinv) {
  int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (i >= n) return;
  const int64_t len = rowptr[i + 1] - rowptr[i];
  deg[i] = (int32_t)(len - 1);
  dinv[i] = (float)(1.0 / sqrt((double)len));     // d~ = deg + 1 = row length
}

// ------------------------------------------------------------------------------------------------
// SpMM schedule (see gad_graph): classes of short rows, chunks of long rows
// ------------------------------------------------------------------------------------------------
// Short rows (1 .. kLongRow non-zeros) fall into classes by ceil(log2(length)), longest class first
// (class 0); long rows form the last class.  key = class << 32 | row: one stable radix pass on the class
// byte orders the rows by class and, inside a class, by row id.
__global__ void classify_rows(const int64_t* __restrict__ rowptr, int64_t n, uint32_t* __restrict__ chunks_of,
                              uint32_t* __restrict__ is_long, uint64_t* __restrict__ key) {
  int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (i >= n) return;
  const int64_t len = rowptr[i + 1] - rowptr[i];
  const bool lng = len > kLongRow;
  chunks_of[i] = lng ? (uint32_t)((len + kLongRow - 1) / kLongRow) : 0u;
  is_long[i] = lng ? 1u : 0u;
  int lg = 0;
  while ((1ll << lg) < len) ++lg;                 // ceil(log2(len)), len >= 1
  int top = 0;
  while ((1 << top) < kLongRow) ++top;            // class of the longest short rows
  const uint64_t cls = lng ? (uint64_t)(top + 1) : (uint64_t)(top - lg);
  key[i] = (cls << 32) | (uint64_t)i;
}

__global__ void take_low32(const uint64_t* __restrict__ key, int64_t n, int32_t* __restrict__ out) {
  int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (i < n) out[i] = (int32_t)(uint32_t)key[i];
}

// chunk_first / long_slot: exclusive scans of chunks_of / is_long.
__global__ void fill_long_rows(int64_t n, const uint32_t* __restrict__ chunk_first,
                               const uint32_t* __restrict__ long_slot, const uint32_t* __restrict__ is_long,
                               int32_t* __restrict__ long_row, int32_t* __restrict__ long_first) {
  int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (i >= n || !is_long[i]) return;
  long_row[long_slot[i]] = (int32_t)i;
  long_first[long_slot[i]] = (int32_t)chunk_first[i];
}

// is_many[i] = 1 iff row i has more than kWaveReduce chunks
__global__ void flag_many(int64_t n, const uint32_t* __restrict__ chunks_of, uint32_t* __restrict__ is_many) {
  int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (i < n) is_many[i] = chunks_of[i] > (uint32_t)kWaveReduce ? 1u : 0u;
}

// many_pos: exclusive scan of is_many; long_slot: position of row i among the long rows.
__global__ void fill_many(int64_t n, const uint32_t* __restrict__ is_many, const uint32_t* __restrict__ many_pos,
                          const uint32_t* __restrict__ long_slot, int32_t* __restrict__ many_slot) {
  int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (i < n && is_many[i]) many_slot[many_pos[i]] = (int32_t)long_slot[i];
}

// One block per long row: its chunks, and for each the key (first gathered column << 32 | chunk id).
__global__ __launch_bounds__(256) void fill_chunks(const int64_t* __restrict__ rowptr, const int32_t* __restrict__ colidx,
                                                   const int32_t* __restrict__ long_row,
                                                   const int32_t* __restrict__ long_first,
                                                   int32_t* __restrict__ chunk_row, int32_t* __restrict__ chunk_begin,
                                                   uint64_t* __restrict__ chunk_key) {
  const int64_t i = long_row[blockIdx.x];
  const int64_t begin = rowptr[i], len = rowptr[i + 1] - begin;
  const int64_t k = (len + kLongRow - 1) / kLongRow;
  const int64_t first = long_first[blockIdx.x];
  for (int64_t c = threadIdx.x; c < k; c += blockDim.x) {
    chunk_row[first + c] = (int32_t)i;
    chunk_begin[first + c] = (int32_t)(c * kLongRow);
    chunk_key[first + c] = ((uint64_t)(uint32_t)colidx[begin + c * kLongRow] << 32) | (uint64_t)(first + c);
  }
}

// One stable pass of the LSD radix sort on the 8-bit digit at `shift`: in -> out.
int radix_pass(const uint64_t* in, uint64_t* out, uint32_t n_keys, int shift, uint32_t* hist, uint32_t* tile_tmp,
               uint32_t* total_out, hipStream_t s) {
  const uint32_t n_tiles = (uint32_t)ceil_div(n_keys, kTile);
  if (n_tiles == 0) return GAD_OK;
  radix_histogram<<<n_tiles, kThreads, 0, s>>>(in, n_keys, shift, n_tiles, hist);
  GAD_LAUNCH_CHECK();
  int st = exclusive_scan_u32(hist, 256u * n_tiles, tile_tmp, total_out, s);
  if (st != GAD_OK) return st;
  radix_scatter<<<n_tiles, kThreads, 0, s>>>(in, out, n_keys, shift, n_tiles, hist);
  GAD_LAUNCH_CHECK();
  return GAD_OK;
}

struct Scratch {   // frees whatever was allocated when it goes out of scope
  std::vector<void*> ptrs;
  ~Scratch() {
    for (void* p : ptrs) (void)hipFree(p);
  }
  template <typename T>
  hipError_t alloc(T** p, size_t count) {
    hipError_t e = hipMalloc((void**)p, sizeof(T) * (count ? count : 1));
    if (e == hipSuccess) ptrs.push_back(*p);
    return e;
  }
};

}  // namespace

// The scan and the radix pass are also used by the augmentation (augment.hip).
int scan_u32(uint32_t* data, uint32_t n, uint32_t* tile_tmp, uint32_t* total_out, hipStream_t s) {
  return exclusive_scan_u32(data, n, tile_tmp, total_out, s);
}
int sort_pass_u64(const uint64_t* in, uint64_t* out, uint32_t n_keys, int shift, uint32_t* hist, uint32_t* tile_tmp,
                  uint32_t* total_out, hipStream_t s) {
  return radix_pass(in, out, n_keys, shift, hist, tile_tmp, total_out, s);
}
size_t sort_hist_len(uint32_t n_keys) { return (size_t)256 * (size_t)ceil_div(n_keys, kTile); }
size_t scan_tmp_len(size_t n) { return (size_t)ceil_div((int64_t)n, kTile) + 1; }

// SpMM schedule of a graph whose rowptr / colidx are in place (see gad_graph).  Allocates the schedule arrays of
// `g` (freed by gad_graph_destroy, also after a failure here) and synchronises the stream.
namespace {
// ew[p] = dinv[colidx[p]]: the factor D~^-1/2 of the gathered row, stored beside its column index
__global__ void edge_weights(const int32_t* __restrict__ colidx, const float* __restrict__ dinv, int64_t nnz,
                             float* __restrict__ ew) {
  const int64_t p = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (p < nnz) ew[p] = dinv[colidx[p]];
}
}  // namespace

int build_schedule(gad_graph* g, hipStream_t s) {
  const int64_t n = g->n;
  if (g->nnz > 0) {
    GAD_HIP(hipMalloc((void**)&g->ew, sizeof(float) * (size_t)g->nnz));
    GAD_GRID_CHECK(ceil_div(g->nnz, 256), 256);
    edge_weights<<<(unsigned)ceil_div(g->nnz, 256), 256, 0, s>>>(g->colidx, g->dinv, g->nnz, g->ew);
    GAD_LAUNCH_CHECK();
  }
  int bits = 1;
  while ((1ll << bits) < n) ++bits;
  Scratch scratch;
  uint32_t *chunks_of = nullptr, *is_long = nullptr, *chunk_first = nullptr, *long_slot = nullptr;
  uint32_t *flags = nullptr, *hist = nullptr, *tile_tmp = nullptr;      // flags: [0] scan totals, [1] long rows, [2] chunks
  uint64_t *key_a = nullptr, *key_b = nullptr;
  // keys: one per row, or one per chunk (a long row of len entries has at most len / kLongRow + 1 <= 2 len / kLongRow)
  const size_t max_chunks = (size_t)(2 * g->nnz / kLongRow + 1);
  const size_t max_keys = (size_t)n > max_chunks ? (size_t)n : max_chunks;
  GAD_HIP(scratch.alloc(&chunks_of, (size_t)n));
  GAD_HIP(scratch.alloc(&is_long, (size_t)n));
  GAD_HIP(scratch.alloc(&chunk_first, (size_t)n));
  GAD_HIP(scratch.alloc(&long_slot, (size_t)n));
  GAD_HIP(scratch.alloc(&flags, 4));
  GAD_HIP(scratch.alloc(&key_a, max_keys));
  GAD_HIP(scratch.alloc(&key_b, max_keys));
  const size_t hist_len = (size_t)256 * (size_t)ceil_div((int64_t)max_keys, kTile);
  GAD_HIP(scratch.alloc(&hist, hist_len));
  GAD_HIP(scratch.alloc(&tile_tmp, (size_t)ceil_div((int64_t)(hist_len > (size_t)n ? hist_len : (size_t)n), kTile) + 1));
  GAD_HIP(hipMemsetAsync(flags, 0, 4 * sizeof(uint32_t), s));
  classify_rows<<<(unsigned)ceil_div(n, 256), 256, 0, s>>>(g->rowptr, n, chunks_of, is_long, key_a);
  GAD_LAUNCH_CHECK();
  GAD_HIP(hipMalloc((void**)&g->row_order, sizeof(int32_t) * (size_t)n));
  int st = radix_pass(key_a, key_b, (uint32_t)n, 32, hist, tile_tmp, flags, s);
  if (st != GAD_OK) return st;
  take_low32<<<(unsigned)ceil_div(n, 256), 256, 0, s>>>(key_b, n, g->row_order);
  GAD_LAUNCH_CHECK();
  // exclusive scans: first chunk id and slot of every long row; totals -> flags[2], flags[1]
  GAD_HIP(hipMemcpyAsync(chunk_first, chunks_of, sizeof(uint32_t) * (size_t)n, hipMemcpyDeviceToDevice, s));
  if ((st = exclusive_scan_u32(chunk_first, (uint32_t)n, tile_tmp, flags + 2, s)) != GAD_OK) return st;
  GAD_HIP(hipMemcpyAsync(long_slot, is_long, sizeof(uint32_t) * (size_t)n, hipMemcpyDeviceToDevice, s));
  if ((st = exclusive_scan_u32(long_slot, (uint32_t)n, tile_tmp, flags + 1, s)) != GAD_OK) return st;
  uint32_t h[4];
  GAD_HIP(hipMemcpyAsync(h, flags, 4 * sizeof(uint32_t), hipMemcpyDeviceToHost, s));
  GAD_HIP(hipStreamSynchronize(s));
  g->n_long = (int32_t)h[1];
  g->n_chunks = (int32_t)h[2];
  g->n_short = n - g->n_long;
  if (g->n_long > 0) {
    GAD_HIP(hipMalloc((void**)&g->long_row, sizeof(int32_t) * (size_t)g->n_long));
    GAD_HIP(hipMalloc((void**)&g->long_first, sizeof(int32_t) * (size_t)g->n_long));
    GAD_HIP(hipMalloc((void**)&g->chunk_row, sizeof(int32_t) * (size_t)g->n_chunks));
    GAD_HIP(hipMalloc((void**)&g->chunk_begin, sizeof(int32_t) * (size_t)g->n_chunks));
    GAD_HIP(hipMalloc((void**)&g->chunk_perm, sizeof(int32_t) * (size_t)g->n_chunks));
    fill_long_rows<<<(unsigned)ceil_div(n, 256), 256, 0, s>>>(n, chunk_first, long_slot, is_long, g->long_row,
                                                              g->long_first);
    GAD_LAUNCH_CHECK();
    uint64_t *ck = key_a, *ck_alt = key_b;
    fill_chunks<<<(unsigned)g->n_long, 256, 0, s>>>(g->rowptr, g->colidx, g->long_row, g->long_first, g->chunk_row,
                                                    g->chunk_begin, ck);
    GAD_LAUNCH_CHECK();
    for (int shift = 32; shift < 32 + bits; shift += 8) {      // order the chunks by their first column
      if ((st = radix_pass(ck, ck_alt, (uint32_t)g->n_chunks, shift, hist, tile_tmp, flags, s)) != GAD_OK) return st;
      uint64_t* t = ck;
      ck = ck_alt;
      ck_alt = t;
    }
    take_low32<<<(unsigned)ceil_div(g->n_chunks, 256), 256, 0, s>>>(ck, g->n_chunks, g->chunk_perm);
    GAD_LAUNCH_CHECK();
    // the rows whose chunk sums a whole block adds (is_long and chunk_first are free again: reused as flag and scan)
    GAD_HIP(hipMalloc((void**)&g->many_slot, sizeof(int32_t) * (size_t)g->n_long));
    flag_many<<<(unsigned)ceil_div(n, 256), 256, 0, s>>>(n, chunks_of, is_long);
    GAD_LAUNCH_CHECK();
    GAD_HIP(hipMemcpyAsync(chunk_first, is_long, sizeof(uint32_t) * (size_t)n, hipMemcpyDeviceToDevice, s));
    if ((st = exclusive_scan_u32(chunk_first, (uint32_t)n, tile_tmp, flags + 3, s)) != GAD_OK) return st;
    fill_many<<<(unsigned)ceil_div(n, 256), 256, 0, s>>>(n, is_long, chunk_first, long_slot, g->many_slot);
    GAD_LAUNCH_CHECK();
    GAD_HIP(hipMemcpyAsync(h, flags, 4 * sizeof(uint32_t), hipMemcpyDeviceToHost, s));
    GAD_HIP(hipStreamSynchronize(s));
    g->n_many = (int32_t)h[3];
  }
  GAD_HIP(hipStreamSynchronize(s));
  return GAD_OK;
}

// ------------------------------------------------------------------------------------------------
// Block-diagonal union of graphs: block k keeps its rows, shifted by the rows of the blocks before it.
// ------------------------------------------------------------------------------------------------
namespace {
__global__ void shift_block(const int64_t* __restrict__ rowptr_in, const int32_t* __restrict__ colidx_in,
                            const int32_t* __restrict__ deg_in, const float* __restrict__ dinv_in, int64_t n, int64_t nnz,
                            int64_t row_off, int64_t nnz_off, int64_t* __restrict__ rowptr, int32_t* __restrict__ colidx,
                            int32_t* __restrict__ deg, float* __restrict__ dinv) {
  const int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (i < n) {
    rowptr[row_off + i] = rowptr_in[i] + nnz_off;
    deg[row_off + i] = deg_in[i];
    dinv[row_off + i] = dinv_in[i];
  }
  if (i < nnz) colidx[nnz_off + i] = colidx_in[i] + (int32_t)row_off;
}
__global__ void set_i64(int64_t* p, int64_t v) { *p = v; }
}  // namespace

int graph_concat(const gad_graph* const* graphs, int K, hipStream_t s, gad_graph** out) {
  int64_t n = 0, nnz = 0, n_local = 0;
  for (int k = 0; k < K; ++k) {
    n += graphs[k]->n;
    nnz += graphs[k]->nnz;
    n_local += graphs[k]->n_local;
  }
  if (n > 2147483646ll || nnz >= 2147483648ll)
    return set_error(GAD_ERR_SHAPE, "the union has %lld rows and %lld non-zeros: beyond 31 bits", (long long)n, (long long)nnz);
  gad_graph* g = new gad_graph();
  g->n = n;
  g->n_local = n_local;
  g->nnz = nnz;
  auto fail = [&](int st) {
    gad_graph_destroy(g);
    return st;
  };
#define GAD_HIP_G(expr)                                                                                    \
  do {                                                                                                     \
    hipError_t _e = (expr);                                                                                \
    if (_e != hipSuccess) return fail(set_error(GAD_ERR_HIP, "%s failed: %s", #expr, hipGetErrorString(_e))); \
  } while (0)
  GAD_HIP_G(hipGetDevice(&g->device));
  GAD_HIP_G(hipMalloc((void**)&g->rowptr, sizeof(int64_t) * (size_t)(n + 1)));
  GAD_HIP_G(hipMalloc((void**)&g->colidx, sizeof(int32_t) * (size_t)nnz));
  GAD_HIP_G(hipMalloc((void**)&g->deg, sizeof(int32_t) * (size_t)n));
  GAD_HIP_G(hipMalloc((void**)&g->dinv, sizeof(float) * (size_t)n));
  GAD_HIP_G(hipMalloc((void**)&g->red_scratch, sizeof(double) * variance_scratch_doubles(n)));
  int64_t row_off = 0, nnz_off = 0;
  for (int k = 0; k < K; ++k) {
    const gad_graph* b = graphs[k];
    const int64_t work = b->nnz > b->n ? b->nnz : b->n;
    shift_block<<<(unsigned)ceil_div(work, 256), 256, 0, s>>>(b->rowptr, b->colidx, b->deg, b->dinv, b->n, b->nnz, row_off,
                                                              nnz_off, g->rowptr, g->colidx, g->deg, g->dinv);
    GAD_HIP_G(hipGetLastError());
    row_off += b->n;
    nnz_off += b->nnz;
  }
  set_i64<<<1, 1, 0, s>>>(g->rowptr + n, nnz);
  GAD_HIP_G(hipGetLastError());
#undef GAD_HIP_G
  int st = build_schedule(g, s);
  if (st != GAD_OK) return fail(st);
  *out = g;
  return GAD_OK;
}

int build_subgraph(const int64_t* src, const int64_t* dst, int64_t n_edges, int64_t n_global, const int64_t* local_ids,
                   int64_t n_local, const int64_t* halo_ids, int64_t n_halo, hipStream_t s, gad_graph** out) {
  const int64_t n = n_local + n_halo;
  const int64_t max_keys = 2 * n_edges + n;
  int bits = 1;
  while ((1ll << bits) < n) ++bits;

  Scratch scratch;
  int32_t* lut = nullptr;
  uint32_t* flags = nullptr;   // [0] range, [1] dup, [2] emitted key count, [3] scan totals (nnz), [4] long rows, [5] chunks
  uint64_t *keys_a = nullptr, *keys_b = nullptr;
  uint32_t *hist = nullptr, *tile_tmp = nullptr, *pos = nullptr;
  GAD_HIP(scratch.alloc(&lut, (size_t)n_global));
  GAD_HIP(scratch.alloc(&flags, 8));
  GAD_HIP(hipMemsetAsync(flags, 0, 8 * sizeof(uint32_t), s));
  fill_i32<<<(unsigned)ceil_div(n_global, 256), 256, 0, s>>>(lut, n_global, -1);
  GAD_LAUNCH_CHECK();
  assign_rows<<<(unsigned)ceil_div(n, 256), 256, 0, s>>>(local_ids, n_local, halo_ids, n_halo, n_global, lut, flags);
  GAD_LAUNCH_CHECK();
  uint32_t h_flags[8];
  GAD_HIP(hipMemcpyAsync(h_flags, flags, 2 * sizeof(uint32_t), hipMemcpyDeviceToHost, s));
  GAD_HIP(hipStreamSynchronize(s));
  if (h_flags[0]) return set_error(GAD_ERR_ID_RANGE, "a local or halo id lies outside [0, n_global)");
  if (h_flags[1]) return set_error(GAD_ERR_ID_DUP, "an id occurs more than once in local_ids ++ halo_ids");

  GAD_HIP(scratch.alloc(&keys_a, (size_t)max_keys));
  GAD_HIP(scratch.alloc(&keys_b, (size_t)max_keys));
  {
    const int64_t work = n_edges > n ? n_edges : n;
    emit_keys<<<(unsigned)ceil_div(work, kEmitItems * kThreads), kThreads, 0, s>>>(src, dst, n_edges, n_global, lut, n, bits, keys_a,
                                                                      flags + 2);
    GAD_LAUNCH_CHECK();
  }
  GAD_HIP(hipMemcpyAsync(h_flags + 2, flags + 2, sizeof(uint32_t), hipMemcpyDeviceToHost, s));
  GAD_HIP(hipStreamSynchronize(s));
  const uint32_t n_keys = (uint32_t)n + h_flags[2];

  const uint32_t n_tiles = (uint32_t)ceil_div(n_keys, kTile);
  const size_t hist_len = (size_t)256 * n_tiles;
  GAD_HIP(scratch.alloc(&hist, hist_len));
  GAD_HIP(scratch.alloc(&tile_tmp, (size_t)ceil_div((int64_t)(hist_len > n_keys ? hist_len : n_keys), kTile) + 1));
  GAD_HIP(scratch.alloc(&pos, (size_t)n_keys));
  uint64_t *cur = keys_a, *alt = keys_b;
  for (int shift = 0; shift < 2 * bits; shift += 8) {
    int st = radix_pass(cur, alt, n_keys, shift, hist, tile_tmp, flags + 3, s);
    if (st != GAD_OK) return st;
    uint64_t* t = cur;
    cur = alt;
    alt = t;
  }
  mark_first<<<(unsigned)ceil_div(n_keys, 256), 256, 0, s>>>(cur, n_keys, pos);
  GAD_LAUNCH_CHECK();
  {
    int st = exclusive_scan_u32(pos, n_keys, tile_tmp, flags + 3, s);
    if (st != GAD_OK) return st;
  }
  GAD_HIP(hipMemcpyAsync(h_flags + 3, flags + 3, sizeof(uint32_t), hipMemcpyDeviceToHost, s));
  GAD_HIP(hipStreamSynchronize(s));
  const int64_t nnz = h_flags[3];

  gad_graph* g = new gad_graph();
  g->n = n;
  g->n_local = n_local;
  g->nnz = nnz;
  auto fail = [&](int st) {
    gad_graph_destroy(g);
    return st;
  };
#define GAD_HIP_G(expr)                                                                                    \
  do {                                                                                                     \
    hipError_t _e = (expr);                                                                                \
    if (_e != hipSuccess) return fail(set_error(GAD_ERR_HIP, "%s failed: %s", #expr, hipGetErrorString(_e))); \
  } while (0)
  GAD_HIP_G(hipGetDevice(&g->device));
  GAD_HIP_G(hipMalloc((void**)&g->rowptr, sizeof(int64_t) * (size_t)(n + 1)));
  GAD_HIP_G(hipMalloc((void**)&g->colidx, sizeof(int32_t) * (size_t)nnz));
  GAD_HIP_G(hipMalloc((void**)&g->deg, sizeof(int32_t) * (size_t)n));
  GAD_HIP_G(hipMalloc((void**)&g->dinv, sizeof(float) * (size_t)n));
  GAD_HIP_G(hipMalloc((void**)&g->red_scratch, sizeof(double) * variance_scratch_doubles(n)));
  assemble_csr<<<(unsigned)ceil_div(n_keys, 256), 256, 0, s>>>(cur, n_keys, pos, bits, n, nnz, g->rowptr, g->colidx);
  GAD_HIP_G(hipGetLastError());
  degree_norm<<<(unsigned)ceil_div(n, 256), 256, 0, s>>>(g->rowptr, n, g->deg, g->dinv);
  GAD_HIP_G(hipGetLastError());
  {
    int st = build_schedule(g, s);       // synchronises the stream
    if (st != GAD_OK) return fail(st);
  }
#undef GAD_HIP_G
  *out = g;
  return GAD_OK;
}

}  // namespace gad
