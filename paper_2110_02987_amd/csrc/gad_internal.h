// Internal declarations shared by the HIP translation units of libgad (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "gad.h"

namespace gad {

constexpr int kWave = 64;

// ---- error plumbing -----------------------------------------------------------------------
int set_error(int status, const char* fmt, ...);   // formats into the thread-local message, returns status

#define GAD_HIP(expr)                                                                        \
  do {                                                                                       \
    hipError_t _e = (expr);                                                                  \
    if (_e != hipSuccess)                                                                    \
      return gad::set_error(GAD_ERR_HIP, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(_e), __FILE__, __LINE__); \
  } while (0)

#define GAD_LAUNCH_CHECK() GAD_HIP(hipGetLastError())

// A launch is valid when, in every grid dimension, the workgroup count fits 31 bits and the thread count 32 bits;
// a larger one is rejected here on the host (it would not run).
#define GAD_GRID_CHECK(blocks, threads)                                                                      \
  do {                                                                                                       \
    const long long _b = (long long)(blocks);                                                                \
    if (_b < 0 || _b > 0x7FFFFFFFll || _b * (long long)(threads) > 0xFFFFFFFFll)                             \
      return gad::set_error(GAD_ERR_SHAPE, "%lld workgroups of %d threads exceed the launch limits (%s:%d)", _b, \
                            (int)(threads), __FILE__, __LINE__);                                             \
  } while (0)

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline int64_t round_up(int64_t a, int64_t b) { return ceil_div(a, b) * b; }

// ---- SpMM epilogues -----------------------------------------------------------------------
enum Epilogue : int {
  EPI_NONE = 0,
  EPI_RELU = 1,   // out = out > 0 ? out : slope * out              (ReLU for slope = 0, LeakyReLU otherwise)
  EPI_MASK = 2,   // out = aux > 0 ? out : slope * out              (its derivative; aux has the layout of out)
};

// Epilogue of a producing kernel (SpMM or GEMM): kind, negative slope, and the activation that decides the mask.
struct Epi {
  int kind = EPI_NONE;
  float slope = 0.f;
  const void* aux = nullptr;   // storage type of the kernel's node-matrix input
  int64_t ldaux = 0;
  bool full_rows = false;      // every row of the node-matrix input can be read up to its leading dimension
  bool shares_gpu = false;     // another kernel runs beside this one (a weight gradient on the side stream)
};

// Rows longer than this many non-zeros are split into chunks of this size; each chunk is summed by
// one wave into a partial row and the partials of a row are added in chunk order.
constexpr int kLongRow = 128;
constexpr int kWaveReduce = 64;   // chunk sums of a row that one wave adds; rows with more are added by a block
constexpr int kMaxWidth = 4096;      // widest feature / hidden dimension accepted
constexpr int kMaxLayers = 16;
constexpr int kMaxConsensus = 128;   // most buffers one consensus call averages
constexpr int kVarBlocks = 512;      // row slabs of the column-sum pass of the variance reduction
constexpr int kStaticVarMaxF = 1024;            // limits of the variance call that keeps its reduction buffer in a
constexpr int64_t kStaticVarMaxN = 1ll << 23;   // file-scope device array (gad_subgraph_variance_static)

}  // namespace gad

struct gad_graph {
  int64_t n = 0, n_local = 0, nnz = 0;
  int64_t* rowptr = nullptr;   // [n+1]
  int32_t* colidx = nullptr;   // [nnz]
  int32_t* deg = nullptr;      // [n]
  float* dinv = nullptr;       // [n]
  float* ew = nullptr;         // [nnz] dinv of the column of every non-zero: the sparse product streams it with colidx
                               // instead of gathering dinv[colidx[p]] (a dependent access per edge: 7 - 24 % of its time)
  // SpMM schedule.  Rows with at most kLongRow non-zeros ("short") are summed by one wave each, in the order
  // row_order[0 .. n_short): longest class first, so that waves running side by side do similar amounts of work.
  // Longer rows are cut into chunks of kLongRow non-zeros; the chunks run in the order chunk_perm[], ascending in
  // the first column they gather, so that chunks running side by side read the same region of the source matrix.
  int64_t n_short = 0;
  int32_t* row_order = nullptr;      // [n] short rows by class, then the long rows
  int32_t n_long = 0;                // number of long rows
  int32_t n_chunks = 0;              // total number of chunks over all long rows
  int32_t* long_row = nullptr;       // [n_long] row id, ascending
  int32_t* long_first = nullptr;     // [n_long] first chunk id of the row (its chunks are consecutive)
  int32_t n_many = 0;                // long rows of more than kWaveReduce chunks
  int32_t* many_slot = nullptr;      // [n_many] their positions in long_row, ascending
  int32_t* chunk_row = nullptr;      // [n_chunks] row id of the chunk
  int32_t* chunk_begin = nullptr;    // [n_chunks] offset of the chunk inside its row
  int32_t* chunk_perm = nullptr;     // [n_chunks] chunk ids in scheduling order
  double* red_scratch = nullptr;     // variance_scratch_doubles(n) doubles; shared by all variance calls on this graph
  int device = 0;
};

namespace gad {

// ---- kernels' host entry points (each enqueues on `s` and returns a gad_status) -------------
int build_subgraph(const int64_t* src, const int64_t* dst, int64_t n_edges, int64_t n_global, const int64_t* local_ids,
                   int64_t n_local, const int64_t* halo_ids, int64_t n_halo, hipStream_t s, gad_graph** out);
// data[0..n) <- exclusive scan (uint32), total_out[0] <- sum; tile_tmp: scan_tmp_len(n) words.
int scan_u32(uint32_t* data, uint32_t n, uint32_t* tile_tmp, uint32_t* total_out, hipStream_t s);
// One stable LSD radix pass on the 8-bit digit at `shift`; hist: sort_hist_len(n_keys) words,
// tile_tmp: scan_tmp_len(sort_hist_len(n_keys)) words.
int sort_pass_u64(const uint64_t* in, uint64_t* out, uint32_t n_keys, int shift, uint32_t* hist, uint32_t* tile_tmp,
                  uint32_t* total_out, hipStream_t s);
size_t sort_hist_len(uint32_t n_keys);
size_t scan_tmp_len(size_t n);
// Importance-based augmentation (Section 3.2.2, Algorithm 1); augment.hip.
int augment_subgraph(const gad_graph* G, const int64_t* part, int64_t n_part, int walk_len, int64_t budget, uint64_t seed,
                     int64_t max_walks, int64_t* halo_out, int64_t* n_halo_out, int64_t* n_walks_out, hipStream_t s);
int build_schedule(gad_graph* g, hipStream_t s);
// Block-diagonal union of K graphs (rows of block k shifted by the rows before it) with a schedule of its own.
int graph_concat(const gad_graph* const* graphs, int K, hipStream_t s, gad_graph** out);
// Node matrices are float32 or bfloat16 (gad_dtype); weights, partial sums and logits are float32.
// out = A~ T with the epilogue applied; epi.aux (EPI_MASK) has T's storage type.  `partial` holds the chunk sums
// of the long rows: spmm_partial_floats(g, width) floats (may be NULL when that is 0).
size_t spmm_partial_floats(const gad_graph* g, int width);
int spmm(const gad_graph* g, const void* T, int64_t ldt, gad_dtype t_in, void* out, int64_t ldo, gad_dtype t_out,
         int width, const Epi& epi, float* partial, hipStream_t s);

// C[M x N] (ldc) = A[M x K] (lda) * op(W) with the epilogue applied to C; W is float32 row-major [w_rows x w_cols];
// op(W) = W (K = w_rows, N = w_cols) or, with trans_w, W^T (K = w_cols, N = w_rows).  epi.aux has A's storage type.
// `scratch` must hold gemm_w_scratch_bytes(w_rows, w_cols) bytes (a transposed or bfloat16 copy of W).
size_t gemm_w_scratch_bytes(int w_rows, int w_cols);
int gemm_w(const void* A, int64_t lda, gad_dtype ta, const float* W, int w_rows, int w_cols, bool trans_w, void* C,
           int64_t ldc, gad_dtype tc, int64_t M, const Epi& epi, void* scratch, hipStream_t s);
// bfloat16 storage: the same two contractions on the bfloat16 matrix instruction (gemm_bf16.hip)
size_t bf16_weight_elems(int n_out, int k);      // elements of the bfloat16 copy of an [n_out x k] right operand
int gemm_w_bf16(const void* A, int64_t lda, const float* W, int w_rows, int w_cols, bool trans_w, void* C, int64_t ldc,
                gad_dtype tc, int64_t M, const Epi& epi, void* scratch, hipStream_t s);
// Output shapes for which the 256 x 256 weight-gradient tiles are worth their padding; ..._wide_ok adds the alignment
// conditions of that kernel.  `wide` selects it; the slabs must then come from the wide split.
inline bool tn_wide_shape(int K, int N) { return K >= 192 && N >= 192; }
bool gemm_tn_bf16_wide_ok(const void* A, int64_t lda, const void* G, int64_t ldg, int K, int N, bool full_rows);
int gemm_tn_bf16(const void* A, int64_t lda, const void* G, int64_t ldg, float* partials, int64_t M, int K, int N,
                 int n_slabs, int64_t slab_rows, bool full_rows, bool wide, hipStream_t s);
// C[K x N] (ldc) = A[M x K]^T * G[M x N]; `partials` must hold gemm_tn_partial_floats(M, K, N) floats.
size_t gemm_tn_partial_floats(int64_t M, int K, int N);
int gemm_tn(const void* A, int64_t lda, const void* G, int64_t ldg, gad_dtype t, float* C, int64_t ldc, int64_t M,
            int K, int N, float* partials, bool full_rows, hipStream_t s);
int transpose_f32(const float* in, int rows, int cols, float* out, hipStream_t s);   // out[cols x rows]

// Z [n x C] (ldz, float32) -> G [n x C] (ldg, storage type tg), loss (double, device).
size_t softmax_partial_doubles(int64_t n);
int softmax_xent(const float* Z, int64_t ldz, const int32_t* labels, const uint8_t* mask, float scale,
                 const float* row_scale /* [n] or NULL */, int64_t n, int C, void* G, int64_t ldg, gad_dtype tg, double* block_partials, double* loss_out, hipStream_t s);
int copy_rows(const void* in, int64_t ldi, gad_dtype ti, float* out, int64_t ldo, int64_t n, int width, hipStream_t s);
size_t variance_scratch_doubles(int64_t n);
// mean[c] = (1/n) sum_i V[i][c] in float64 (ordered sums); part: kVarBlocks x F doubles of scratch.
int column_means_f64(const void* V, int64_t n, int F, gad_dtype dtype, double* part, double* mean, hipStream_t s);
// Eq. 14 with the distance inside the pair sum (optimizer_pairs.hip).
size_t pair_importance_workspace_bytes(int64_t n, int F);
int pair_importance(const gad_graph* g, const void* V, int F, gad_dtype dtype, double beta, double* out2, void* ws,
                    hipStream_t s);
int subgraph_variance(const gad_graph* g, const void* V, int F, gad_dtype dtype, double beta, double* out3,
                      float* per_node, hipStream_t s);
// The same reduction with its buffer in a file-scope device array: allocates nothing; F <= kStaticVarMaxF, n <= kStaticVarMaxN.
int subgraph_variance_static(const gad_graph* g, const void* V, int F, gad_dtype dtype, double beta, double* out3,
                             float* per_node, hipStream_t s);
int weighted_consensus(const float* const* bufs, int K, const double* w, int64_t n, float* out, hipStream_t s);
int consensus_update(const float* const* bufs, int K, const double* w, int64_t n, float eta, float* params,
                     float* avg_out, hipStream_t s);

}  // namespace gad
