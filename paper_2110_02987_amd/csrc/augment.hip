// Importance-based subgraph augmentation on the GPU (arXiv 2110.02987, Section 3.2.2): the boundary nodes B(g)
// of a partition (Definition 2), Monte-Carlo importance I(v) of the candidate replication nodes from random walks
// of length l on the original graph (Eq. 3, Property 1), the number of walks from the Monte-Carlo error (Eq. 4),
// and the depth-first selection of whole walks in descending score until the replica budget is met (Algorithm 1).
//
// Everything is integer work, so the result is exact and reproducible: walk j is a pure function of
// (seed, j) through a counter-based generator (a splitmix64 finaliser of the mixed counter; multiply-shift range
// reduction), visit counts are integer atomics, walks are ordered by (score descending, walk number) with a stable
// radix sort, and "the first `budget` distinct nodes met when the walks are read in that order" is computed as the
// nodes with the smallest first position (atomicMin), sorted by that position.  Walks are never stored: the
// scoring and selection passes regenerate them from their number.
#include <math.h>

#include <vector>

#include "gad_internal.h"

namespace gad {
namespace {

constexpr int kMaxWalkLen = 16;

__device__ __forceinline__ uint32_t draw(uint64_t seed, uint64_t walk, uint64_t step) {
  uint64_t x = seed ^ (walk * 0x9E3779B97F4A7C15ull) ^ (step * 0xD1B54A32D192ED03ull);
  x += 0x9E3779B97F4A7C15ull;
  x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
  x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
  x ^= x >> 31;
  return (uint32_t)(x >> 32);
}
__device__ __forceinline__ uint32_t below(uint32_t r, uint32_t m) { return (uint32_t)(((uint64_t)r * m) >> 32); }

__global__ void fill_u32(uint32_t* p, int64_t n, uint32_t v) {
  int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// mark[v] = 1 + position of v in `part` (0: not in the partition).
// flags[0]: a row outside [0, N); flags[1]: a row listed twice
__global__ void mark_part(const int64_t* __restrict__ part, int64_t n_part, int64_t N, uint32_t* __restrict__ mark,
                          uint32_t* __restrict__ flags) {
  int64_t p = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (p >= n_part) return;
  const int64_t v = part[p];
  if (v < 0 || v >= N) {
    flags[0] = 1u;
    return;
  }
  if (atomicExch(&mark[v], (uint32_t)p + 1u) != 0u) flags[1] = 1u;
}

// is_b[p] = 1 iff part[p] has a neighbour outside the partition.  A 16-lane group owns one row and looks at 64
// of its entries per step (columns ascend, so the members of a partition made of low ids all come first: one
// thread per row would walk half of every hub row alone).  Rows longer than kLongRow entries get 0 here and are
// decided chunk by chunk in boundary_flags_long.
__global__ __launch_bounds__(256) void boundary_flags(const int64_t* __restrict__ part, int64_t n_part,
                                                      const int64_t* __restrict__ rowptr,
                                                      const int32_t* __restrict__ colidx,
                                                      const uint32_t* __restrict__ mark, uint32_t* __restrict__ is_b) {
  const int l = threadIdx.x & 15;
  const int64_t p = (blockIdx.x * (int64_t)blockDim.x + threadIdx.x) >> 4;
  const bool live = p < n_part;                      // all lanes of a wave stay in the loop's shuffles
  int64_t b = 0, e = 0;
  if (live) {
    const int64_t v = part[p];
    b = rowptr[v];
    e = rowptr[v + 1];
    if (e - b > kLongRow) e = b;                     // a long row: left to the chunk pass
  }
  int out = 0;
  for (int64_t q0 = b; ; q0 += 64) {
    const int more = (q0 < e && !out) ? 1 : 0;
    // the wave leaves the loop together: when none of its four groups has entries left to look at
    if (__ballot(more) == 0ull) break;
    if (more) {
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int64_t q = q0 + u * 16 + l;
        if (q < e && mark[colidx[q]] == 0u) out = 1;   // the self loop is inside
      }
    }
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) out |= __shfl_xor(out, o, 16);
  }
  if (live && l == 0) is_b[p] = out ? 1u : 0u;
}

// The rows of more than kLongRow entries, by the graph's own chunk list (kLongRow entries per chunk): a 16-lane group
// owns one chunk of a row of the partition and raises the row's flag when the chunk holds an outside neighbour.
__global__ __launch_bounds__(256) void boundary_flags_long(const int32_t* __restrict__ chunk_row,
                                                           const int32_t* __restrict__ chunk_begin, int64_t n_chunks,
                                                           const int64_t* __restrict__ rowptr,
                                                           const int32_t* __restrict__ colidx,
                                                           const uint32_t* __restrict__ mark,
                                                           uint32_t* __restrict__ is_b) {
  const int l = threadIdx.x & 15;
  const int64_t c = (blockIdx.x * (int64_t)blockDim.x + threadIdx.x) >> 4;
  uint32_t m = 0;
  int64_t b = 0, e = 0;
  if (c < n_chunks) {
    const int64_t row = chunk_row[c];
    m = mark[row];
    if (m != 0u) {
      b = rowptr[row] + chunk_begin[c];
      e = rowptr[row + 1];
      if (e > b + kLongRow) e = b + kLongRow;
    }
  }
  int out = 0;
  for (int64_t q = b + l; q < e; q += 16)
    if (mark[colidx[q]] == 0u) out = 1;
#pragma unroll
  for (int o = 8; o > 0; o >>= 1) out |= __shfl_xor(out, o, 16);
  if (m != 0u && out && l == 0) atomicOr(&is_b[m - 1u], 1u);
}

// deg_b[p] = degree of part[p] if it is a boundary node, else 0
__global__ void boundary_degrees(const int64_t* __restrict__ part, int64_t n_part, const int64_t* __restrict__ rowptr,
                                 const uint32_t* __restrict__ is_b, uint32_t* __restrict__ deg_b) {
  const int64_t p = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (p >= n_part) return;
  const int64_t v = part[p];
  deg_b[p] = is_b[p] ? (uint32_t)(rowptr[v + 1] - rowptr[v] - 1) : 0u;
}

__global__ void compact_boundary(const int64_t* __restrict__ part, int64_t n_part, const uint32_t* __restrict__ is_b,
                                 const uint32_t* __restrict__ pos, int32_t* __restrict__ B) {
  int64_t p = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (p < n_part && is_b[p]) B[pos[p]] = (int32_t)part[p];
}

// Walk number j: seq[0] = start, seq[1..l] = the steps.  A node without neighbours stays where it is.
__device__ __forceinline__ void walk(const int64_t* __restrict__ rowptr, const int32_t* __restrict__ colidx,
                                     const int32_t* __restrict__ B, uint32_t n_b, int l, uint64_t seed, uint64_t j,
                                     int32_t (&seq)[kMaxWalkLen + 1]) {
  int32_t cur = B[below(draw(seed, j, 0), n_b)];
  seq[0] = cur;
  for (int t = 1; t <= l; ++t) {
    const int64_t b = rowptr[cur];
    const uint32_t d = (uint32_t)(rowptr[cur + 1] - b - 1);
    if (d > 0) {
      const uint32_t k = below(draw(seed, j, (uint64_t)t), d);
      int32_t u = colidx[b + k];
      if (u >= cur) u = colidx[b + k + 1];        // columns ascend: skip the self loop
      cur = u;
    }
    seq[t] = cur;
  }
}

// Eq. 3: cnt[v] += 1 for every node v outside the partition that walk j meets (once per walk).
__global__ void count_walks(const int64_t* __restrict__ rowptr, const int32_t* __restrict__ colidx,
                            const int32_t* __restrict__ B, uint32_t n_b, int l, uint64_t seed, int64_t j0, int64_t j1,
                            const uint32_t* __restrict__ mark, uint32_t* __restrict__ cnt) {
  const int64_t j = j0 + blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (j >= j1) return;
  int32_t seq[kMaxWalkLen + 1];
  walk(rowptr, colidx, B, n_b, l, seed, (uint64_t)j, seq);
  for (int t = 1; t <= l; ++t) {
    const int32_t v = seq[t];
    if (mark[v]) continue;
    bool again = false;
    for (int q = 1; q < t; ++q) again = again || seq[q] == v;
    if (!again) atomicAdd(&cnt[v], 1u);
  }
}

// stats[0] = visited candidates, stats[1] = sum cnt, stats[2] = sum cnt^2
__global__ __launch_bounds__(256) void count_stats(const uint32_t* __restrict__ cnt, int64_t N,
                                                   unsigned long long* __restrict__ stats) {
  __shared__ unsigned long long sm[3][256];
  unsigned long long m = 0, s1 = 0, s2 = 0;
  for (int64_t v = blockIdx.x * 256ll + threadIdx.x; v < N; v += (int64_t)gridDim.x * 256) {
    const unsigned long long c = cnt[v];
    m += c > 0;
    s1 += c;
    s2 += c * c;
  }
  sm[0][threadIdx.x] = m;
  sm[1][threadIdx.x] = s1;
  sm[2][threadIdx.x] = s2;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o)
      for (int k = 0; k < 3; ++k) sm[k][threadIdx.x] += sm[k][threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x < 3) atomicAdd(&stats[threadIdx.x], sm[threadIdx.x][0]);
}

// key[j] = (0xFFFFFFFF - score_j) << 32 | j, score_j = sum over the steps outside the partition of cnt
__global__ void score_walks(const int64_t* __restrict__ rowptr, const int32_t* __restrict__ colidx,
                            const int32_t* __restrict__ B, uint32_t n_b, int l, uint64_t seed, int64_t n_walks,
                            const uint32_t* __restrict__ mark, const uint32_t* __restrict__ cnt,
                            uint64_t* __restrict__ key) {
  const int64_t j = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (j >= n_walks) return;
  int32_t seq[kMaxWalkLen + 1];
  walk(rowptr, colidx, B, n_b, l, seed, (uint64_t)j, seq);
  uint32_t score = 0;
  for (int t = 1; t <= l; ++t)
    if (!mark[seq[t]]) score += cnt[seq[t]];
  key[j] = ((uint64_t)(0xFFFFFFFFu - score) << 32) | (uint64_t)j;
}

// first[v] = smallest (rank of the walk) * (l + 1) + step at which v is met
__global__ void first_positions(const int64_t* __restrict__ rowptr, const int32_t* __restrict__ colidx,
                                const int32_t* __restrict__ B, uint32_t n_b, int l, uint64_t seed, int64_t n_walks,
                                const uint64_t* __restrict__ sorted_key, const uint32_t* __restrict__ mark,
                                uint32_t* __restrict__ first) {
  const int64_t r = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (r >= n_walks) return;
  int32_t seq[kMaxWalkLen + 1];
  walk(rowptr, colidx, B, n_b, l, seed, sorted_key[r] & 0xFFFFFFFFull, seq);
  for (int t = 1; t <= l; ++t)
    if (!mark[seq[t]]) atomicMin(&first[seq[t]], (uint32_t)(r * (l + 1) + t));
}

__global__ void candidate_flags(const uint32_t* __restrict__ first, int64_t N, uint32_t* __restrict__ flag) {
  int64_t v = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (v < N) flag[v] = first[v] != 0xFFFFFFFFu ? 1u : 0u;
}

__global__ void candidate_keys(const uint32_t* __restrict__ first, int64_t N, const uint32_t* __restrict__ pos,
                               uint64_t* __restrict__ key) {
  int64_t v = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (v < N && first[v] != 0xFFFFFFFFu) key[pos[v]] = ((uint64_t)first[v] << 32) | (uint64_t)v;
}

__global__ void take_nodes(const uint64_t* __restrict__ key, int64_t n, int64_t* __restrict__ out) {
  int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
  if (i < n) out[i] = (int64_t)(key[i] & 0xFFFFFFFFull);
}

struct Scratch {
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

inline unsigned blocks(int64_t n) { return (unsigned)ceil_div(n > 0 ? n : 1, 256); }

// Eq. 4 solved for n at E = 0.05, z_c = 1.96:  n = ceil((z_c / E)^2 (m S2 - S1^2) / S1^2), evaluated exactly:
// (z_c / E)^2 = 38416 / 25, and the ceiling is that of an integer quotient.  S1 <= walks * steps <= 2^30,
// S2 <= S1 * walks <= 2^56 and m <= S1, so 38416 * m * S2 stays below 2^102.
int64_t walk_count(unsigned long long m, unsigned long long s1, unsigned long long s2) {
  if (m == 0 || s1 == 0) return 0;
  const unsigned __int128 num = (unsigned __int128)m * s2 - (unsigned __int128)s1 * s1;     // >= 0 (Cauchy-Schwarz)
  const unsigned __int128 den = (unsigned __int128)s1 * s1;
  const unsigned __int128 a = 38416u * num, b = 25u * den;
  return (int64_t)((a + b - 1) / b);
}

}  // namespace

int augment_subgraph(const gad_graph* G, const int64_t* part, int64_t n_part, int walk_len, int64_t budget, uint64_t seed,
                     int64_t max_walks, int64_t* halo_out, int64_t* n_halo_out, int64_t* n_walks_out, hipStream_t s) {
  const int64_t N = G->n;
  const int l = walk_len;
  *n_halo_out = 0;
  if (n_walks_out) *n_walks_out = 0;
  Scratch scratch;
  uint32_t *mark = nullptr, *cnt = nullptr, *first = nullptr, *is_b = nullptr, *deg_b = nullptr, *pos = nullptr;
  uint32_t *flags = nullptr, *tile_tmp = nullptr, *hist = nullptr;   // flags: [0] range, [1] dup, [2] |B|, [3] n0, [4] scan totals
  unsigned long long* stats = nullptr;
  int32_t* B = nullptr;
  GAD_HIP(scratch.alloc(&mark, (size_t)N));
  GAD_HIP(scratch.alloc(&cnt, (size_t)N));
  GAD_HIP(scratch.alloc(&first, (size_t)N));
  GAD_HIP(scratch.alloc(&is_b, (size_t)n_part));
  GAD_HIP(scratch.alloc(&deg_b, (size_t)n_part));
  GAD_HIP(scratch.alloc(&pos, (size_t)(N > n_part ? N : n_part)));
  GAD_HIP(scratch.alloc(&flags, 8));
  GAD_HIP(scratch.alloc(&stats, 4));
  GAD_HIP(scratch.alloc(&B, (size_t)n_part));
  GAD_HIP(hipMemsetAsync(flags, 0, 8 * sizeof(uint32_t), s));
  GAD_HIP(hipMemsetAsync(stats, 0, 4 * sizeof(unsigned long long), s));
  GAD_HIP(hipMemsetAsync(mark, 0, (size_t)N * sizeof(uint32_t), s));
  GAD_HIP(hipMemsetAsync(cnt, 0, (size_t)N * sizeof(uint32_t), s));
  mark_part<<<blocks(n_part), 256, 0, s>>>(part, n_part, N, mark, flags);
  GAD_LAUNCH_CHECK();
  uint32_t h_flags[8];
  GAD_HIP(hipMemcpyAsync(h_flags, flags, 2 * sizeof(uint32_t), hipMemcpyDeviceToHost, s));
  GAD_HIP(hipStreamSynchronize(s));
  if (h_flags[0]) return set_error(GAD_ERR_ID_RANGE, "a partition row lies outside [0, n)");
  if (h_flags[1]) return set_error(GAD_ERR_ID_DUP, "a partition row is listed twice");

  // boundary set, in the order of `part`; first batch of walks = sum of the boundary degrees
  const size_t max_items = (size_t)(N > n_part ? N : n_part);
  GAD_HIP(scratch.alloc(&tile_tmp, scan_tmp_len(max_items > sort_hist_len((uint32_t)max_walks) ? max_items
                                                                                                : sort_hist_len((uint32_t)max_walks))));
  GAD_GRID_CHECK(ceil_div(n_part * 16, 256), 256);
  GAD_GRID_CHECK(ceil_div((int64_t)G->n_chunks * 16, 256), 256);
  boundary_flags<<<blocks(n_part * 16), 256, 0, s>>>(part, n_part, G->rowptr, G->colidx, mark, is_b);
  GAD_LAUNCH_CHECK();
  if (G->n_chunks > 0) {
    boundary_flags_long<<<blocks((int64_t)G->n_chunks * 16), 256, 0, s>>>(G->chunk_row, G->chunk_begin, G->n_chunks,
                                                                          G->rowptr, G->colidx, mark, is_b);
    GAD_LAUNCH_CHECK();
  }
  boundary_degrees<<<blocks(n_part), 256, 0, s>>>(part, n_part, G->rowptr, is_b, deg_b);
  GAD_LAUNCH_CHECK();
  GAD_HIP(hipMemcpyAsync(pos, is_b, (size_t)n_part * sizeof(uint32_t), hipMemcpyDeviceToDevice, s));
  int st = scan_u32(pos, (uint32_t)n_part, tile_tmp, flags + 2, s);
  if (st != GAD_OK) return st;
  compact_boundary<<<blocks(n_part), 256, 0, s>>>(part, n_part, is_b, pos, B);
  GAD_LAUNCH_CHECK();
  st = scan_u32(deg_b, (uint32_t)n_part, tile_tmp, flags + 3, s);
  if (st != GAD_OK) return st;
  GAD_HIP(hipMemcpyAsync(h_flags + 2, flags + 2, 2 * sizeof(uint32_t), hipMemcpyDeviceToHost, s));
  GAD_HIP(hipStreamSynchronize(s));
  const uint32_t n_b = h_flags[2];
  if (n_b == 0 || budget <= 0) return GAD_OK;            // nothing leaves the partition: no candidates
  int64_t n0 = h_flags[3];
  if (n0 < 1) n0 = 1;
  if (n0 > max_walks) n0 = max_walks;

  // Eq. 3 on the first batch, Eq. 4 for the total, then the rest of the walks
  count_walks<<<blocks(n0), 256, 0, s>>>(G->rowptr, G->colidx, B, n_b, l, seed, 0, n0, mark, cnt);
  GAD_LAUNCH_CHECK();
  count_stats<<<256, 256, 0, s>>>(cnt, N, stats);
  GAD_LAUNCH_CHECK();
  unsigned long long h_stats[3];
  GAD_HIP(hipMemcpyAsync(h_stats, stats, 3 * sizeof(unsigned long long), hipMemcpyDeviceToHost, s));
  GAD_HIP(hipStreamSynchronize(s));
  int64_t n_walks = walk_count(h_stats[0], h_stats[1], h_stats[2]);
  if (n_walks < n0) n_walks = n0;
  if (n_walks > max_walks) n_walks = max_walks;
  if (n_walks > n0) {
    count_walks<<<blocks(n_walks - n0), 256, 0, s>>>(G->rowptr, G->colidx, B, n_b, l, seed, n0, n_walks, mark, cnt);
    GAD_LAUNCH_CHECK();
  }
  if (n_walks_out) *n_walks_out = n_walks;

  // walks in descending score (ties: walk number), first position of every candidate in that order
  uint64_t *key_a = nullptr, *key_b = nullptr;
  const size_t n_keys_max = (size_t)(n_walks > N ? n_walks : N);
  GAD_HIP(scratch.alloc(&key_a, n_keys_max));
  GAD_HIP(scratch.alloc(&key_b, n_keys_max));
  GAD_HIP(scratch.alloc(&hist, sort_hist_len((uint32_t)n_keys_max)));
  score_walks<<<blocks(n_walks), 256, 0, s>>>(G->rowptr, G->colidx, B, n_b, l, seed, n_walks, mark, cnt, key_a);
  GAD_LAUNCH_CHECK();
  uint64_t *cur = key_a, *alt = key_b;
  for (int shift = 32; shift < 64; shift += 8) {
    st = sort_pass_u64(cur, alt, (uint32_t)n_walks, shift, hist, tile_tmp, flags + 4, s);
    if (st != GAD_OK) return st;
    uint64_t* t = cur;
    cur = alt;
    alt = t;
  }
  fill_u32<<<blocks(N), 256, 0, s>>>(first, N, 0xFFFFFFFFu);
  GAD_LAUNCH_CHECK();
  first_positions<<<blocks(n_walks), 256, 0, s>>>(G->rowptr, G->colidx, B, n_b, l, seed, n_walks, cur, mark, first);
  GAD_LAUNCH_CHECK();

  // candidates ordered by first position; the first `budget` of them are the replication nodes
  candidate_flags<<<blocks(N), 256, 0, s>>>(first, N, pos);
  GAD_LAUNCH_CHECK();
  st = scan_u32(pos, (uint32_t)N, tile_tmp, flags + 5, s);
  if (st != GAD_OK) return st;
  GAD_HIP(hipMemcpyAsync(h_flags + 5, flags + 5, sizeof(uint32_t), hipMemcpyDeviceToHost, s));
  GAD_HIP(hipStreamSynchronize(s));
  const int64_t n_cand = h_flags[5];
  candidate_keys<<<blocks(N), 256, 0, s>>>(first, N, pos, key_a);
  GAD_LAUNCH_CHECK();
  cur = key_a;
  alt = key_b;
  for (int shift = 32; shift < 64; shift += 8) {
    st = sort_pass_u64(cur, alt, (uint32_t)n_cand, shift, hist, tile_tmp, flags + 4, s);
    if (st != GAD_OK) return st;
    uint64_t* t = cur;
    cur = alt;
    alt = t;
  }
  const int64_t n_halo = n_cand < budget ? n_cand : budget;
  take_nodes<<<blocks(n_halo), 256, 0, s>>>(cur, n_halo, halo_out);
  GAD_LAUNCH_CHECK();
  GAD_HIP(hipStreamSynchronize(s));
  *n_halo_out = n_halo;
  return GAD_OK;
}

}  // namespace gad
