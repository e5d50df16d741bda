// C ABI of libgad: argument validation, workspace planning and the order of kernels in the forward and
// backward passes of the per-processor GCN step (arXiv 2110.02987, Section 3.3, Eq. 7-10; Algorithm 2).
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>

#include <mutex>
#include <unordered_map>
#include <vector>

#include "gad_internal.h"

namespace gad {

static thread_local char g_error[512] = "";

int set_error(int status, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_error, sizeof(g_error), fmt, ap);
  va_end(ap);
  return status;
}

namespace {

constexpr size_t kAlign = 256;

inline int64_t pad_ld(int w) { return round_up(w, 16); }

// Where everything lives inside the caller's workspace (offsets in bytes).
struct Plan {
  int L = 0;
  int dims[kMaxLayers + 1];
  bool agg_first[kMaxLayers];      // layer l computes (A~ H) W  (true)  or  A~ (H W)  (false)
  size_t agg[kMaxLayers];          // M_l = A~ H_l, kept for dW_l     (agg_first layers)      [n x pad(dims[l])]
  size_t act[kMaxLayers + 1];      // H_l for 1 <= l < L (post-ReLU), act[L] = Z               [n x pad(dims[l])]
  size_t g_a = 0, g_b = 0, tmp = 0;  // [n x max_ld] each
  size_t wt = 0;                   // scratch copy of one weight matrix (transposed and / or bfloat16)
  size_t tn = 0;                   // slab partials of the weight-gradient GEMM
  size_t sm = 0;                   // softmax block partials (doubles)
  size_t sp = 0;                   // chunk sums of the long rows of the sparse product
  size_t total = 0;
  int64_t max_ld = 0;
};

int make_plan(const gad_graph* g, int L, const int32_t* dims, gad_dtype dtype, Plan* p) {
  if (!g || !dims) return set_error(GAD_ERR_NULL, "graph or dims is NULL");
  if (L < 1 || L > kMaxLayers) return set_error(GAD_ERR_SHAPE, "L = %d outside [1, %d]", L, kMaxLayers);
  for (int l = 0; l <= L; ++l)
    if (dims[l] < 1 || dims[l] > kMaxWidth)
      return set_error(GAD_ERR_SHAPE, "dims[%d] = %d outside [1, %d]", l, dims[l], kMaxWidth);
  if (dtype != GAD_F32 && dtype != GAD_BF16) return set_error(GAD_ERR_UNSUPPORTED, "unknown dtype %d", (int)dtype);
  const size_t esz = dtype == GAD_F32 ? sizeof(float) : sizeof(uint16_t);   // node matrices; logits stay float32
  p->L = L;
  const size_t n = (size_t)g->n;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    size_t o = off;
    off += (bytes + kAlign - 1) / kAlign * kAlign;
    return o;
  };
  p->max_ld = 0;
  size_t max_w = 0, max_tn = 0;
  for (int l = 0; l <= L; ++l) p->dims[l] = dims[l];
  for (int l = 1; l <= L; ++l)
    if (pad_ld(dims[l]) > p->max_ld) p->max_ld = pad_ld(dims[l]);
  for (int l = 0; l < L; ++l) {
    p->agg_first[l] = dims[l] <= dims[l + 1];
    p->agg[l] = p->agg_first[l] ? take(n * pad_ld(dims[l]) * esz) : 0;
    p->act[l + 1] = take(n * pad_ld(dims[l + 1]) * (l + 1 == L ? sizeof(float) : esz));
    if (p->agg_first[l] && pad_ld(dims[l]) > p->max_ld) p->max_ld = pad_ld(dims[l]);
    const size_t w = gemm_w_scratch_bytes(dims[l], dims[l + 1]);
    if (w > max_w) max_w = w;
    const size_t t = gemm_tn_partial_floats(g->n, dims[l], dims[l + 1]);
    if (t > max_tn) max_tn = t;
  }
  p->act[0] = 0;
  p->g_a = take(n * p->max_ld * esz);
  p->g_b = take(n * p->max_ld * esz);
  p->tmp = take(n * p->max_ld * esz);
  p->wt = take(max_w);
  p->tn = take(max_tn * sizeof(float));
  p->sm = take(softmax_partial_doubles(g->n) * sizeof(double));
  p->sp = take(spmm_partial_floats(g, (int)p->max_ld) * sizeof(float));
  p->total = off;
  return GAD_OK;
}

// Which forward a workspace currently holds (host-side bookkeeping; the workspace itself is device memory).
// An entry is erased when a forward starts on the workspace and written when its last launch has been enqueued, so
// a forward that fails half way leaves no entry behind.  A backward overwrites the seed gradient of the forward
// (and, for deeper models, the gradient buffers it swaps): it marks the entry, and a second backward is refused.
// The library cannot see a workspace being freed: gad_workspace_forget erases the entry, and the table holds at most
// kMaxSaved entries (the least recently written one is dropped beyond that).
struct Saved {
  const gad_graph* g;
  int L;
  std::vector<int32_t> dims;
  gad_dtype dtype;
  const void* X;
  float slope;
  bool grads_consumed;     // a backward has run on this forward
  uint64_t tick;           // order of insertion
};
constexpr size_t kMaxSaved = 1024;
std::mutex g_saved_mu;
std::unordered_map<const void*, Saved> g_saved;
uint64_t g_saved_tick = 0;

void forget_workspace(const void* ws) {
  std::lock_guard<std::mutex> lk(g_saved_mu);
  g_saved.erase(ws);
}

void remember_forward(const void* ws, const gad_graph* g, int L, const int32_t* dims, gad_dtype dtype, const void* X,
                      float slope) {
  std::lock_guard<std::mutex> lk(g_saved_mu);
  if (g_saved.size() >= kMaxSaved && g_saved.find(ws) == g_saved.end()) {
    auto oldest = g_saved.begin();
    for (auto it = g_saved.begin(); it != g_saved.end(); ++it)
      if (it->second.tick < oldest->second.tick) oldest = it;
    g_saved.erase(oldest);
  }
  g_saved[ws] = Saved{g, L, std::vector<int32_t>(dims, dims + L + 1), dtype, X, slope, false, ++g_saved_tick};
}

int check_common(const gad_graph* g, const void* X, int L, const int32_t* dims, const float* const* W, void* ws,
                 size_t ws_bytes, const Plan& p) {
  if (!X || !W || !ws) return set_error(GAD_ERR_NULL, "X, W or workspace is NULL");
  for (int l = 0; l < L; ++l)
    if (!W[l]) return set_error(GAD_ERR_NULL, "W[%d] is NULL", l);
  if ((reinterpret_cast<uintptr_t>(ws) & (kAlign - 1)) != 0)
    return set_error(GAD_ERR_WORKSPACE, "workspace is not %zu-byte aligned", kAlign);
  if (ws_bytes < p.total)
    return set_error(GAD_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", ws_bytes, p.total);
  (void)g;
  (void)dims;
  return GAD_OK;
}

// True iff `ws` holds a forward of exactly this problem (X = nullptr: any features).  for_backward: the forward's
// gradients must still be there; on success they are marked as consumed.
bool forward_saved(const gad_graph* g, const void* ws, int L, const int32_t* dims, gad_dtype dtype, const void* X,
                   const float* slope = nullptr, bool for_backward = false, bool* consumed = nullptr) {
  std::lock_guard<std::mutex> lk(g_saved_mu);
  auto it = g_saved.find(ws);
  bool ok = it != g_saved.end() && it->second.g == g && it->second.L == L && it->second.dtype == dtype &&
            (X == nullptr || it->second.X == X) && (slope == nullptr || it->second.slope == *slope);
  if (ok)
    for (int l = 0; l <= L; ++l) ok = ok && it->second.dims[l] == dims[l];
  if (ok && for_backward) {
    if (it->second.grads_consumed) {
      if (consumed) *consumed = true;
      return false;
    }
    it->second.grads_consumed = true;
  }
  return ok;
}

inline void* at(void* ws, size_t off) { return static_cast<char*>(ws) + off; }

// Measurement aid (gad_gcn_layer_events): events the forward and backward passes of this thread record at their
// layer boundaries.  Empty = off.
thread_local std::vector<hipEvent_t> g_layer_events;

inline bool layer_events_on(int L) { return (int)g_layer_events.size() >= 2 * L + 3; }

// The weight-gradient products of the backward pass are bound by the matrix cores, the sparse products next to them
// by memory, and neither needs the other's result: dW_l runs on a side stream while the main stream goes on with
// the gradient of the layer below.  One side stream (default priority) and two events per host thread and device,
// created at first use and kept until the process ends.  The fork / join pattern (event recorded on one stream,
// awaited on the other) is also valid while the caller's stream is being captured into a HIP graph.
constexpr double kForkFlops = 2e9;     // smallest weight-gradient product that is forked (about 20 us of matrix work)

struct Side {
  hipStream_t stream = nullptr;
  hipEvent_t fork = nullptr, done = nullptr;
};

int side_of_this_thread(Side** out) {
  thread_local std::unordered_map<int, Side> sides;
  int dev = 0;
  GAD_HIP(hipGetDevice(&dev));
  Side& sd = sides[dev];
  if (!sd.stream) {
    GAD_HIP(hipStreamCreateWithFlags(&sd.stream, hipStreamNonBlocking));
    GAD_HIP(hipEventCreateWithFlags(&sd.fork, hipEventDisableTiming));
    GAD_HIP(hipEventCreateWithFlags(&sd.done, hipEventDisableTiming));
  }
  *out = &sd;
  return GAD_OK;
}

// GAD_SERIAL_BACKWARD=1 in the environment keeps the whole backward pass on the caller's stream.
bool overlap_enabled() {
  static const bool on = [] {
    const char* v = getenv("GAD_SERIAL_BACKWARD");
    return !(v && v[0] == '1');
  }();
  return on;
}

}  // namespace
}  // namespace gad

using namespace gad;

// The launch checks of the library read the runtime's last-error slot, which keeps an error of ANY earlier HIP call
// on the thread until somebody reads it -- also one that the caller's framework handled itself (an allocator that
// ran out of memory, freed its cache and tried again).  Every entry point that launches work empties the slot first,
// so that what it reports is its own.
#define GAD_ENTER() (void)hipGetLastError()

extern "C" {

const char* gad_last_error(void) { return g_error; }

int gad_build_subgraph(const int64_t* src, const int64_t* dst, int64_t n_edges_in, int64_t n_global,
                       const int64_t* local_ids, int64_t n_local, const int64_t* halo_ids, int64_t n_halo,
                       void* hip_stream, gad_graph** out) {
  GAD_ENTER();
  if (!out) return set_error(GAD_ERR_NULL, "out is NULL");
  *out = nullptr;
  if (n_edges_in < 0 || n_local < 0 || n_halo < 0 || n_global < 1)
    return set_error(GAD_ERR_SHAPE, "negative size or n_global < 1");
  const int64_t n = n_local + n_halo;
  if (n < 1) return set_error(GAD_ERR_SHAPE, "the subgraph has no nodes");
  if (n > 2147483646ll) return set_error(GAD_ERR_SHAPE, "n = %lld exceeds 2^31 - 2", (long long)n);
  if (2 * n_edges_in + n >= 2147483648ll)
    return set_error(GAD_ERR_SHAPE, "2 * n_edges_in + n = %lld does not fit 31 bits", (long long)(2 * n_edges_in + n));
  if (n_global >= 2147483648ll) return set_error(GAD_ERR_SHAPE, "n_global does not fit 31 bits");
  if ((n_edges_in > 0 && (!src || !dst)) || (n_local > 0 && !local_ids) || (n_halo > 0 && !halo_ids))
    return set_error(GAD_ERR_NULL, "a required array is NULL");
  return build_subgraph(src, dst, n_edges_in, n_global, local_ids, n_local, halo_ids, n_halo,
                        static_cast<hipStream_t>(hip_stream), out);
}

int gad_graph_info(const gad_graph* g, int64_t* n, int64_t* n_local, int64_t* nnz, const int64_t** rowptr,
                   const int32_t** colidx, const int32_t** deg, const float** dinv) {
  if (!g) return set_error(GAD_ERR_NULL, "graph is NULL");
  if (n) *n = g->n;
  if (n_local) *n_local = g->n_local;
  if (nnz) *nnz = g->nnz;
  if (rowptr) *rowptr = g->rowptr;
  if (colidx) *colidx = g->colidx;
  if (deg) *deg = g->deg;
  if (dinv) *dinv = g->dinv;
  return GAD_OK;
}

int gad_graph_concat(const gad_graph* const* graphs, int K, void* hip_stream, gad_graph** out) {
  GAD_ENTER();
  if (!out) return set_error(GAD_ERR_NULL, "out is NULL");
  *out = nullptr;
  if (!graphs) return set_error(GAD_ERR_NULL, "graphs is NULL");
  if (K < 1 || K > 65536) return set_error(GAD_ERR_SHAPE, "K = %d outside [1, 65536]", K);
  for (int k = 0; k < K; ++k)
    if (!graphs[k]) return set_error(GAD_ERR_NULL, "graphs[%d] is NULL", k);
  return graph_concat(graphs, K, static_cast<hipStream_t>(hip_stream), out);
}

int gad_graph_destroy(gad_graph* g) {
  if (!g) return GAD_OK;
  void* ptrs[] = {g->rowptr,     g->colidx,    g->deg,       g->dinv,        g->ew,         g->row_order, g->long_row,
                  g->long_first, g->many_slot, g->chunk_row, g->chunk_begin, g->chunk_perm, g->red_scratch};
  int st = GAD_OK;
  for (void* p : ptrs)
    if (p && hipFree(p) != hipSuccess) st = set_error(GAD_ERR_HIP, "hipFree failed in gad_graph_destroy");
  {
    std::lock_guard<std::mutex> lk(g_saved_mu);
    for (auto it = g_saved.begin(); it != g_saved.end();)
      it = it->second.g == g ? g_saved.erase(it) : ++it;
  }
  delete g;
  return st;
}

int gad_augment_subgraph(const gad_graph* G, const int64_t* part_rows, int64_t n_part, int32_t walk_len, int64_t budget,
                         uint64_t seed, int64_t max_walks, int64_t* halo_rows_out, int64_t* n_halo_out,
                         int64_t* n_walks_out, void* hip_stream) {
  GAD_ENTER();
  if (!G || !n_halo_out) return set_error(GAD_ERR_NULL, "graph or n_halo_out is NULL");
  *n_halo_out = 0;
  if (n_part < 1 || n_part > G->n) return set_error(GAD_ERR_SHAPE, "n_part = %lld outside [1, n]", (long long)n_part);
  if (!part_rows) return set_error(GAD_ERR_NULL, "part_rows is NULL");
  if (walk_len < 1 || walk_len > 16) return set_error(GAD_ERR_SHAPE, "walk_len = %d outside [1, 16]", walk_len);
  if (budget < 0 || (budget > 0 && !halo_rows_out)) return set_error(GAD_ERR_NULL, "budget < 0, or halo_rows_out is NULL");
  if (max_walks < 1 || max_walks > (1ll << 26))
    return set_error(GAD_ERR_SHAPE, "max_walks = %lld outside [1, 2^26]", (long long)max_walks);
  return augment_subgraph(G, part_rows, n_part, walk_len, budget, seed, max_walks, halo_rows_out, n_halo_out, n_walks_out,
                          static_cast<hipStream_t>(hip_stream));
}

int gad_gcn_workspace_bytes(const gad_graph* g, int L, const int32_t* dims, gad_dtype dtype, size_t* bytes) {
  if (!bytes) return set_error(GAD_ERR_NULL, "bytes is NULL");
  Plan p;
  int st = make_plan(g, L, dims, dtype, &p);
  if (st != GAD_OK) return st;
  *bytes = p.total;
  return GAD_OK;
}

// reuse_first: the caller vouches that X is unchanged since the forward this workspace holds
static int forward_impl(const gad_graph* g, const void* X, gad_dtype dtype, int L, const int32_t* dims,
                        const float* const* W, const int32_t* labels, const uint8_t* mask, float loss_scale,
                        const float* row_scale, float negative_slope, void* workspace, size_t workspace_bytes,
                        float* logits_out, double* loss_out, void* hip_stream, bool reuse_first) {
  GAD_ENTER();
  Plan p;
  int st = make_plan(g, L, dims, dtype, &p);
  if (st != GAD_OK) return st;
  st = check_common(g, X, L, dims, W, workspace, workspace_bytes, p);
  if (st != GAD_OK) return st;
  if (!labels) return set_error(GAD_ERR_NULL, "labels is NULL");
  if (!isfinite(loss_scale)) return set_error(GAD_ERR_SHAPE, "loss_scale is not finite");
  if (!(negative_slope >= 0.f && negative_slope < 1.f))
    return set_error(GAD_ERR_SHAPE, "negative_slope must lie in [0, 1)");
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const int64_t n = g->n;
  // A~ X of the first layer is still in the workspace when the last forward on it had this graph, X and model
  const bool have_first = reuse_first && p.agg_first[0] && forward_saved(g, workspace, L, dims, dtype, X);
  forget_workspace(workspace);                           // from here on the workspace holds no complete forward
  const bool marks = layer_events_on(L);
  if (marks) GAD_HIP(hipEventRecord(g_layer_events[0], s));

  const void* h = X;
  int64_t ldh = dims[0];
  void* wsc = at(workspace, p.wt);
  float* psum = static_cast<float*>(at(workspace, p.sp));
  for (int l = 0; l < L; ++l) {
    const bool last = l == L - 1;
    Epi act;                                             // sigma of Eq. 7 on every layer but the last
    act.kind = last ? EPI_NONE : EPI_RELU;
    act.slope = negative_slope;
    act.full_rows = true;                                // its input is the aggregate in the workspace
    Epi none;
    none.full_rows = h != X;                             // workspace matrices are whole [n x ld] blocks; X is the caller's
    const gad_dtype t_dst = last ? GAD_F32 : dtype;      // the logits are kept in float32
    void* dst = at(workspace, p.act[l + 1]);
    const int64_t ldd = pad_ld(dims[l + 1]);
    if (p.agg_first[l]) {
      void* m = at(workspace, p.agg[l]);
      const int64_t ldm = pad_ld(dims[l]);
      const bool have = l == 0 && have_first;
      if (!have && (st = spmm(g, h, ldh, dtype, m, ldm, dtype, dims[l], none, psum, s)) != GAD_OK) return st;
      if ((st = gemm_w(m, ldm, dtype, W[l], dims[l], dims[l + 1], false, dst, ldd, t_dst, n, act, wsc, s)) != GAD_OK)
        return st;
    } else {
      void* t = at(workspace, p.tmp);
      if ((st = gemm_w(h, ldh, dtype, W[l], dims[l], dims[l + 1], false, t, ldd, dtype, n, none, wsc, s)) != GAD_OK)
        return st;
      if ((st = spmm(g, t, ldd, dtype, dst, ldd, t_dst, dims[l + 1], act, psum, s)) != GAD_OK) return st;
    }
    h = dst;
    ldh = ldd;
    if (marks) GAD_HIP(hipEventRecord(g_layer_events[l + 1], s));
  }
  const int C = dims[L];
  const int64_t ldz = pad_ld(C);
  const float* Z = static_cast<const float*>(h);
  st = softmax_xent(Z, ldz, labels, mask, loss_scale, row_scale, n, C, at(workspace, p.g_a), ldz, dtype,
                    static_cast<double*>(at(workspace, p.sm)), loss_out, s);
  if (st != GAD_OK) return st;
  if (logits_out && (st = copy_rows(Z, ldz, GAD_F32, logits_out, C, n, C, s)) != GAD_OK) return st;
  if (marks) GAD_HIP(hipEventRecord(g_layer_events[L + 1], s));
  remember_forward(workspace, g, L, dims, dtype, X, negative_slope);
  return GAD_OK;
}

int gad_gcn_layer_events(void* const* events, int count) {
  if (count < 0 || (count > 0 && !events)) return set_error(GAD_ERR_NULL, "count < 0, or events is NULL");
  for (int i = 0; i < count; ++i)
    if (!events[i]) return set_error(GAD_ERR_NULL, "events[%d] is NULL", i);
  g_layer_events.assign(reinterpret_cast<const hipEvent_t*>(events), reinterpret_cast<const hipEvent_t*>(events) + count);
  return GAD_OK;
}

int gad_workspace_forget(const void* workspace) {
  if (!workspace) return set_error(GAD_ERR_NULL, "workspace is NULL");
  forget_workspace(workspace);
  return GAD_OK;
}

int gad_gcn_forward(const gad_graph* g, const void* X, gad_dtype dtype, int L, const int32_t* dims,
                    const float* const* W, const int32_t* labels, const uint8_t* mask, float loss_scale,
                    const float* row_scale, float negative_slope, void* workspace, size_t workspace_bytes,
                    float* logits_out, double* loss_out, void* hip_stream) {
  return forward_impl(g, X, dtype, L, dims, W, labels, mask, loss_scale, row_scale, negative_slope, workspace,
                      workspace_bytes, logits_out, loss_out, hip_stream, false);
}

int gad_gcn_forward_cached(const gad_graph* g, const void* X, gad_dtype dtype, int L, const int32_t* dims,
                           const float* const* W, const int32_t* labels, const uint8_t* mask, float loss_scale,
                           const float* row_scale, float negative_slope, void* workspace, size_t workspace_bytes,
                           float* logits_out, double* loss_out, void* hip_stream) {
  return forward_impl(g, X, dtype, L, dims, W, labels, mask, loss_scale, row_scale, negative_slope, workspace,
                      workspace_bytes, logits_out, loss_out, hip_stream, true);
}

int gad_gcn_backward(const gad_graph* g, const void* X, gad_dtype dtype, int L, const int32_t* dims,
                     const float* const* W, float negative_slope, void* workspace, size_t workspace_bytes,
                     float* const* dW, float* const* G_out, void* hip_stream) {
  GAD_ENTER();
  Plan p;
  int st = make_plan(g, L, dims, dtype, &p);
  if (st != GAD_OK) return st;
  st = check_common(g, X, L, dims, W, workspace, workspace_bytes, p);
  if (st != GAD_OK) return st;
  if (!dW) return set_error(GAD_ERR_NULL, "dW is NULL");
  for (int l = 0; l < L; ++l)
    if (!dW[l]) return set_error(GAD_ERR_NULL, "dW[%d] is NULL", l);
  bool consumed = false;
  if (!forward_saved(g, workspace, L, dims, dtype, X, &negative_slope, true, &consumed))
    return set_error(GAD_ERR_STATE, consumed ? "a backward pass has already used this forward pass: run the forward again"
                                             : "workspace holds no forward pass matching this graph / model / X / slope");
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const int64_t n = g->n;
  void* gcur = at(workspace, p.g_a);
  void* gnext = at(workspace, p.g_b);
  void* tmp = at(workspace, p.tmp);
  void* wsc = at(workspace, p.wt);
  float* psum = static_cast<float*>(at(workspace, p.sp));
  float* tn = static_cast<float*>(at(workspace, p.tn));
  Side* side = nullptr;
  if (overlap_enabled() && (st = side_of_this_thread(&side)) != GAD_OK) return st;
  bool side_busy = false;                                // a weight gradient is in flight on the side stream
  // dW_l = A^T B on the side stream, after everything enqueued on the main stream so far
  auto weight_grad = [&](const void* A, int64_t lda, const void* B, int64_t ldb, int l) -> int {
    hipStream_t ws = s;
    // a product of a few microseconds gains nothing beside another kernel and would pay for the two events
    const bool fork = side && 2.0 * (double)n * dims[l] * dims[l + 1] >= kForkFlops;
    if (fork) {
      GAD_HIP(hipEventRecord(side->fork, s));
      GAD_HIP(hipStreamWaitEvent(side->stream, side->fork, 0));
      ws = side->stream;
    }
    int r = gemm_tn(A, lda, B, ldb, dtype, dW[l], dims[l + 1], n, dims[l], dims[l + 1], tn, A != X, ws);
    if (fork) {
      GAD_HIP(hipEventRecord(side->done, side->stream));
      side_busy = true;
    }
    return r;
  };
  // the main stream waits for the weight gradient in flight: before a buffer it reads is written again, and
  // before this call returns
  auto join = [&]() -> int {
    if (side_busy) GAD_HIP(hipStreamWaitEvent(s, side->done, 0));
    side_busy = false;
    return GAD_OK;
  };
  const bool marks = layer_events_on(L);
  if (marks) GAD_HIP(hipEventRecord(g_layer_events[L + 2], s));
  for (int l = L - 1; l >= 0; --l) {
    const int fin = dims[l], fout = dims[l + 1];
    const int64_t ldg = pad_ld(fout);        // G_l, S_l
    const int64_t ldi = pad_ld(fin);         // dM, G_{l-1}, H_l
    const void* hin = l == 0 ? X : at(workspace, p.act[l]);
    const int64_t ldhin = l == 0 ? dims[0] : ldi;
    Epi none;
    none.full_rows = true;                               // the dense products below read workspace matrices
    Epi dact;                                            // derivative of sigma, decided by the saved activation H_l
    dact.kind = EPI_MASK;
    dact.slope = negative_slope;
    dact.aux = hin;
    dact.ldaux = ldhin;
    dact.full_rows = true;
    if (G_out && G_out[l] && (st = copy_rows(gcur, ldg, dtype, G_out[l], fout, n, fout, s)) != GAD_OK) break;
    // the layer above may still be reading tmp and what is now gnext (its G); both are written below
    if ((st = join()) != GAD_OK) break;
    if (p.agg_first[l]) {
      // forked behind the dense product, so that the weight gradient (matrix cores) runs beside the sparse
      // product (memory) rather than beside another dense product
      if (l > 0 && (st = gemm_w(gcur, ldg, dtype, W[l], fin, fout, true, tmp, ldi, dtype, n, none, wsc, s)) != GAD_OK) break;
      if ((st = weight_grad(at(workspace, p.agg[l]), ldi, gcur, ldg, l)) != GAD_OK) break;
      dact.shares_gpu = side_busy;
      if (l > 0 && (st = spmm(g, tmp, ldi, dtype, gnext, ldi, dtype, fin, dact, psum, s)) != GAD_OK) break;
    } else {
      if ((st = spmm(g, gcur, ldg, dtype, tmp, ldg, dtype, fout, none, psum, s)) != GAD_OK) break;
      if ((st = weight_grad(hin, ldhin, tmp, ldg, l)) != GAD_OK) break;
      if (l > 0) {
        if ((st = gemm_w(tmp, ldg, dtype, W[l], fin, fout, true, gnext, ldi, dtype, n, dact, wsc, s)) != GAD_OK) break;
      }
    }
    void* t = gcur;
    gcur = gnext;
    gnext = t;
    if (marks) {                                         // a layer's time includes its weight gradient: join first
      if ((st = join()) != GAD_OK) break;
      if (hipEventRecord(g_layer_events[L + 3 + (L - 1 - l)], s) != hipSuccess) {
        st = set_error(GAD_ERR_HIP, "hipEventRecord failed on a layer event");
        break;
      }
    }
  }
  const int stj = join();                                // also on an error path: the side stream never outlives the call
  return st != GAD_OK ? st : stj;
}

int gad_gcn_activation(const gad_graph* g, const void* workspace, size_t workspace_bytes, int L,
                       const int32_t* dims, gad_dtype dtype, int layer, float* out, void* hip_stream) {
  GAD_ENTER();
  Plan p;
  int st = make_plan(g, L, dims, dtype, &p);
  if (st != GAD_OK) return st;
  if (!workspace || !out) return set_error(GAD_ERR_NULL, "workspace or out is NULL");
  if (workspace_bytes < p.total) return set_error(GAD_ERR_WORKSPACE, "workspace smaller than the plan");
  if (layer < 1 || layer > L) return set_error(GAD_ERR_SHAPE, "layer = %d outside [1, %d]", layer, L);
  if (!forward_saved(g, workspace, L, dims, dtype, nullptr))
    return set_error(GAD_ERR_STATE, "workspace holds no forward pass matching this graph / model");
  return copy_rows(at(const_cast<void*>(workspace), p.act[layer]), pad_ld(dims[layer]), layer == L ? GAD_F32 : dtype, out,
                   dims[layer], g->n, dims[layer], static_cast<hipStream_t>(hip_stream));
}

int gad_spmm_workspace_bytes(const gad_graph* g, int32_t width, size_t* bytes) {
  if (!g || !bytes) return set_error(GAD_ERR_NULL, "graph or bytes is NULL");
  if (width < 1 || width > kMaxWidth) return set_error(GAD_ERR_SHAPE, "width = %d outside [1, %d]", width, kMaxWidth);
  *bytes = spmm_partial_floats(g, width) * sizeof(float);
  return GAD_OK;
}

int gad_spmm(const gad_graph* g, const void* T, int64_t ldt, void* out, int64_t ldo, int32_t width, gad_dtype dtype,
             void* workspace, size_t workspace_bytes, void* hip_stream) {
  GAD_ENTER();
  if (!g || !T || !out) return set_error(GAD_ERR_NULL, "graph, T or out is NULL");
  if (width < 1 || width > kMaxWidth || ldt < width || ldo < width)
    return set_error(GAD_ERR_SHAPE, "width outside [1, %d] or a leading dimension < width", kMaxWidth);
  if (T == out) return set_error(GAD_ERR_SHAPE, "out must not alias T");
  if (dtype != GAD_F32 && dtype != GAD_BF16) return set_error(GAD_ERR_UNSUPPORTED, "unknown dtype %d", (int)dtype);
  const size_t need = spmm_partial_floats(g, width) * sizeof(float);
  if (need > 0 && (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 15u) != 0))
    return set_error(GAD_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed (16-byte aligned)", workspace_bytes, need);
  return spmm(g, T, ldt, dtype, out, ldo, dtype, width, Epi(), static_cast<float*>(workspace),
              static_cast<hipStream_t>(hip_stream));
}

static int gemm_args(int64_t M, int32_t K, int32_t N, gad_dtype dtype) {
  if (M < 0 || K < 1 || N < 1 || K > kMaxWidth || N > kMaxWidth)
    return set_error(GAD_ERR_SHAPE, "M < 0, or K / N outside [1, %d]", kMaxWidth);
  if (dtype != GAD_F32 && dtype != GAD_BF16) return set_error(GAD_ERR_UNSUPPORTED, "unknown dtype %d", (int)dtype);
  return GAD_OK;
}

int gad_gemm_workspace_bytes(int64_t M, int32_t K, int32_t N, size_t* bytes) {
  if (!bytes) return set_error(GAD_ERR_NULL, "bytes is NULL");
  int st = gemm_args(M, K, N, GAD_F32);
  if (st != GAD_OK) return st;
  const size_t w = (gemm_w_scratch_bytes(K, N) + kAlign - 1) / kAlign * kAlign;
  *bytes = w + gemm_tn_partial_floats(M, K, N) * sizeof(float);
  return GAD_OK;
}

int gad_gemm_w(const void* A, int64_t lda, const float* W, int32_t w_rows, int32_t w_cols, int transpose_w, void* C,
               int64_t ldc, int64_t M, gad_dtype dtype, void* workspace, size_t workspace_bytes, void* hip_stream) {
  GAD_ENTER();
  const int32_t K = transpose_w ? w_cols : w_rows, N = transpose_w ? w_rows : w_cols;
  int st = gemm_args(M, K, N, dtype);
  if (st != GAD_OK) return st;
  if (!A || !W || !C || !workspace) return set_error(GAD_ERR_NULL, "A, W, C or workspace is NULL");
  if (lda < K || ldc < N) return set_error(GAD_ERR_SHAPE, "a leading dimension is smaller than its row");
  if ((reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1)) != 0 || workspace_bytes < gemm_w_scratch_bytes(w_rows, w_cols))
    return set_error(GAD_ERR_WORKSPACE, "workspace too small or not %zu-byte aligned", kAlign);
  return gemm_w(A, lda, dtype, W, w_rows, w_cols, transpose_w != 0, C, ldc, dtype, M, Epi(), workspace,
                static_cast<hipStream_t>(hip_stream));
}

int gad_gemm_tn(const void* A, int64_t lda, const void* G, int64_t ldg, float* C, int64_t M, int32_t K, int32_t N,
                gad_dtype dtype, void* workspace, size_t workspace_bytes, void* hip_stream) {
  GAD_ENTER();
  int st = gemm_args(M, K, N, dtype);
  if (st != GAD_OK) return st;
  if (!A || !G || !C || !workspace) return set_error(GAD_ERR_NULL, "A, G, C or workspace is NULL");
  if (lda < K || ldg < N) return set_error(GAD_ERR_SHAPE, "a leading dimension is smaller than its row");
  if (M < 1) return set_error(GAD_ERR_SHAPE, "M must be positive");
  if ((reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1)) != 0 ||
      workspace_bytes < gemm_tn_partial_floats(M, K, N) * sizeof(float))
    return set_error(GAD_ERR_WORKSPACE, "workspace too small or not %zu-byte aligned", kAlign);
  return gemm_tn(A, lda, G, ldg, dtype, C, N, M, K, N, static_cast<float*>(workspace), false,
                 static_cast<hipStream_t>(hip_stream));
}

int gad_subgraph_variance(const gad_graph* g, const void* V, int32_t F, gad_dtype dtype, double beta, double* out3,
                          float* per_node_out, void* hip_stream) {
  GAD_ENTER();
  if (!g || !V || !out3) return set_error(GAD_ERR_NULL, "graph, V or out3 is NULL");
  if (F < 1 || F > kMaxWidth) return set_error(GAD_ERR_SHAPE, "F = %d outside [1, %d]", F, kMaxWidth);
  if (!(beta > 0.0) || !isfinite(beta)) return set_error(GAD_ERR_SHAPE, "beta must be positive and finite");
  if (dtype != GAD_F32 && dtype != GAD_BF16) return set_error(GAD_ERR_UNSUPPORTED, "unknown dtype");
  return subgraph_variance(g, V, F, dtype, beta, out3, per_node_out, static_cast<hipStream_t>(hip_stream));
}

int gad_subgraph_variance_static(const gad_graph* g, const void* V, int32_t F, gad_dtype dtype, double beta, double* out3,
                                 float* per_node_out, void* hip_stream) {
  GAD_ENTER();
  if (!g || !V || !out3) return set_error(GAD_ERR_NULL, "graph, V or out3 is NULL");
  if (F < 1) return set_error(GAD_ERR_SHAPE, "F = %d must be positive", F);
  if (!(beta > 0.0) || !isfinite(beta)) return set_error(GAD_ERR_SHAPE, "beta must be positive and finite");
  if (dtype != GAD_F32 && dtype != GAD_BF16) return set_error(GAD_ERR_UNSUPPORTED, "unknown dtype");
  return subgraph_variance_static(g, V, F, dtype, beta, out3, per_node_out, static_cast<hipStream_t>(hip_stream));
}

int gad_pair_importance_workspace_bytes(const gad_graph* g, int32_t F, size_t* bytes) {
  if (!g || !bytes) return set_error(GAD_ERR_NULL, "graph or bytes is NULL");
  if (F < 1 || F > kMaxWidth) return set_error(GAD_ERR_SHAPE, "F = %d outside [1, %d]", F, kMaxWidth);
  *bytes = pair_importance_workspace_bytes(g->n, F);
  return GAD_OK;
}

int gad_pair_importance(const gad_graph* g, const void* V, int32_t F, gad_dtype dtype, double beta, double* out2,
                        void* workspace, size_t workspace_bytes, void* hip_stream) {
  GAD_ENTER();
  if (!g || !V || !out2 || !workspace) return set_error(GAD_ERR_NULL, "graph, V, out2 or workspace is NULL");
  if (F < 1 || F > kMaxWidth) return set_error(GAD_ERR_SHAPE, "F = %d outside [1, %d]", F, kMaxWidth);
  if (!(beta > 0.0) || !isfinite(beta)) return set_error(GAD_ERR_SHAPE, "beta must be positive and finite");
  if (!((float)beta >= 1.17549435e-38f) || !isfinite((float)beta))      // the pair terms are formed in float32
    return set_error(GAD_ERR_SHAPE, "beta = %g is not a normal float32 number", beta);
  if (dtype != GAD_F32 && dtype != GAD_BF16) return set_error(GAD_ERR_UNSUPPORTED, "unknown dtype");
  if ((reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1)) != 0 ||
      workspace_bytes < pair_importance_workspace_bytes(g->n, F))
    return set_error(GAD_ERR_WORKSPACE, "workspace too small or not %zu-byte aligned", kAlign);
  return pair_importance(g, V, F, dtype, beta, out2, workspace, static_cast<hipStream_t>(hip_stream));
}

// Validates the importance weights and forms zeta_k / sum_j zeta_j in float64.
static int consensus_weights(const float* const* bufs, int K, const double* zeta, int64_t n_elems, double* w) {
  if (!bufs || !zeta) return set_error(GAD_ERR_NULL, "bufs or zeta is NULL");
  if (K < 1 || K > kMaxConsensus) return set_error(GAD_ERR_SHAPE, "K = %d outside [1, %d]", K, kMaxConsensus);
  if (n_elems < 0) return set_error(GAD_ERR_SHAPE, "n_elems is negative");
  double sum = 0.0;
  for (int k = 0; k < K; ++k) {
    if (!bufs[k]) return set_error(GAD_ERR_NULL, "bufs[%d] is NULL", k);
    if (!isfinite(zeta[k]) || zeta[k] < 0.0) return set_error(GAD_ERR_WEIGHTS, "zeta[%d] is negative or not finite", k);
    sum += zeta[k];
  }
  if (!(sum > 0.0) || !isfinite(sum)) return set_error(GAD_ERR_WEIGHTS, "the weights sum to zero (or overflow)");
  for (int k = 0; k < K; ++k) w[k] = zeta[k] / sum;
  return GAD_OK;
}

int gad_weighted_consensus(const float* const* bufs, int K, const double* zeta, int64_t n_elems, float* out,
                           void* hip_stream) {
  GAD_ENTER();
  if (!out) return set_error(GAD_ERR_NULL, "out is NULL");
  double w[kMaxConsensus];
  int st = consensus_weights(bufs, K, zeta, n_elems, w);
  if (st != GAD_OK) return st;
  return weighted_consensus(bufs, K, w, n_elems, out, static_cast<hipStream_t>(hip_stream));
}

int gad_consensus_update(const float* const* grads, int K, const double* zeta, int64_t n_elems, float eta,
                         float* params, float* avg_out, void* hip_stream) {
  GAD_ENTER();
  if (!params) return set_error(GAD_ERR_NULL, "params is NULL");
  if (!isfinite(eta)) return set_error(GAD_ERR_SHAPE, "eta is not finite");
  double w[kMaxConsensus];
  int st = consensus_weights(grads, K, zeta, n_elems, w);
  if (st != GAD_OK) return st;
  for (int k = 0; k < K; ++k)
    if (grads[k] == params) return set_error(GAD_ERR_SHAPE, "params must not alias a gradient buffer");
  return consensus_update(grads, K, w, n_elems, eta, params, avg_out, static_cast<hipStream_t>(hip_stream));
}

int gad_train_round(int K, const gad_graph* const* graphs, const void* const* X, gad_dtype dtype, int L,
                    const int32_t* dims, float* params, const int32_t* const* labels, const uint8_t* const* masks,
                    const float* loss_scales, float negative_slope, void* const* workspaces,
                    const size_t* workspace_bytes, float* grads, const double* zeta, float eta, double* losses,
                    int x_unchanged, void* hip_stream) {
  GAD_ENTER();
  if (K < 1 || K > kMaxConsensus) return set_error(GAD_ERR_SHAPE, "K = %d outside [1, %d]", K, kMaxConsensus);
  if (!graphs || !X || !dims || !params || !labels || !loss_scales || !workspaces || !workspace_bytes || !grads || !zeta)
    return set_error(GAD_ERR_NULL, "a required argument is NULL");
  if (L < 1 || L > kMaxLayers) return set_error(GAD_ERR_SHAPE, "L = %d outside [1, %d]", L, kMaxLayers);
  if (!isfinite(eta)) return set_error(GAD_ERR_SHAPE, "eta is not finite");
  int64_t off[kMaxLayers + 1];
  off[0] = 0;
  for (int l = 0; l < L; ++l) {
    if (dims[l] < 1 || dims[l + 1] < 1) return set_error(GAD_ERR_SHAPE, "dims must be positive");
    off[l + 1] = off[l] + (int64_t)dims[l] * dims[l + 1];
  }
  const int64_t P = off[L];
  const float* W[kMaxLayers];
  for (int l = 0; l < L; ++l) W[l] = params + off[l];
  const float* gptr[kMaxConsensus];
  double w[kMaxConsensus];
  for (int k = 0; k < K; ++k) gptr[k] = grads + (int64_t)k * P;
  int st = consensus_weights(gptr, K, zeta, P, w);           // reject bad weights before any launch
  if (st != GAD_OK) return st;
  for (int k = 0; k < K; ++k) {
    float* dW[kMaxLayers];
    for (int l = 0; l < L; ++l) dW[l] = grads + (int64_t)k * P + off[l];
    st = forward_impl(graphs[k], X[k], dtype, L, dims, W, labels[k], masks ? masks[k] : nullptr, loss_scales[k], nullptr,
                      negative_slope, workspaces[k], workspace_bytes[k], nullptr, losses ? losses + k : nullptr,
                      hip_stream, x_unchanged != 0);
    if (st != GAD_OK) return st;
    st = gad_gcn_backward(graphs[k], X[k], dtype, L, dims, W, negative_slope, workspaces[k], workspace_bytes[k], dW,
                          nullptr, hip_stream);
    if (st != GAD_OK) return st;
  }
  return consensus_update(gptr, K, w, P, eta, params, nullptr, static_cast<hipStream_t>(hip_stream));
}

int gad_train_round_batched(const gad_graph* g, const void* X, gad_dtype dtype, int L, const int32_t* dims, float* params,
                            const int32_t* labels, const uint8_t* mask, const float* row_scale, float negative_slope,
                            void* workspace, size_t workspace_bytes, float* grad, float eta, double* loss,
                            int x_unchanged, void* hip_stream) {
  GAD_ENTER();
  if (!dims || !params || !grad) return set_error(GAD_ERR_NULL, "dims, params or grad is NULL");
  if (L < 1 || L > kMaxLayers) return set_error(GAD_ERR_SHAPE, "L = %d outside [1, %d]", L, kMaxLayers);
  if (!isfinite(eta)) return set_error(GAD_ERR_SHAPE, "eta is not finite");
  int64_t off[kMaxLayers + 1];
  off[0] = 0;
  for (int l = 0; l < L; ++l) {
    if (dims[l] < 1 || dims[l + 1] < 1) return set_error(GAD_ERR_SHAPE, "dims must be positive");
    off[l + 1] = off[l] + (int64_t)dims[l] * dims[l + 1];
  }
  const float* W[kMaxLayers];
  float* dW[kMaxLayers];
  for (int l = 0; l < L; ++l) {
    W[l] = params + off[l];
    dW[l] = grad + off[l];
  }
  int st = forward_impl(g, X, dtype, L, dims, W, labels, mask, 1.f, row_scale, negative_slope, workspace, workspace_bytes,
                        nullptr, loss, hip_stream, x_unchanged != 0);
  if (st != GAD_OK) return st;
  st = gad_gcn_backward(g, X, dtype, L, dims, W, negative_slope, workspace, workspace_bytes, dW, nullptr, hip_stream);
  if (st != GAD_OK) return st;
  const float* gp[1] = {grad};
  const double one[1] = {1.0};
  return consensus_update(gp, 1, one, off[L], eta, params, nullptr, static_cast<hipStream_t>(hip_stream));
}

}  // extern "C"
