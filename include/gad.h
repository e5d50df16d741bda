/* libgad -- C ABI of the MI355X (gfx950) hot path of GAD's per-processor GCN training step.
 *
 * Paper: "Distributed Optimization of Graph Convolutional Network using Subgraph Variance"
 * (arXiv 2110.02987).  One processor holds one augmented subgraph g' = (v + v', e + e')
 * (Algorithm 1, last step; Algorithm 2, Require) and runs, per iteration, the forward
 * propagation of Eq. 7/8, the loss and gradient of Eq. 9/10 (Algorithm 2, the two steps inside
 * the per-processor loop), and then takes part in the weighted global consensus of Eq. 15 with
 * the variance-based importance zeta of Eq. 14.
 *
 * Conventions
 *  - Every pointer is a DEVICE pointer unless its comment says "host".
 *  - Matrices are row-major.  "ld" is the leading dimension in elements.
 *  - The caller owns every buffer it passes in, including the workspaces.  The library owns only
 *    gad_graph objects (create / destroy pair) and scratch memory that lives inside one call.
 *    The calls that allocate or free device memory (gad_build_subgraph, gad_graph_concat, gad_augment_subgraph,
 *    gad_graph_destroy) must not run while a stream of the process is being captured into a HIP graph.
 *    Everything else only enqueues kernels and may be captured, after ONE un-captured call of the same kind and
 *    shapes on the device: the first use of a kernel sets its attributes and the first backward creates the
 *    library's side stream and events, which does not belong inside a capture.
 *    A graph is read-only to every call except gad_subgraph_variance, which uses a reduction buffer inside
 *    the graph: variance calls on ONE graph from different streams must not overlap.
 *  - All calls enqueue work on `hip_stream` (a hipStream_t, NULL = default stream) and return
 *    without synchronising, except gad_build_subgraph, gad_graph_concat and gad_augment_subgraph, which
 *    synchronise the stream.  gad_gcn_backward (and the training rounds built on it) runs its weight-gradient
 *    products on a stream of the library's own that forks from `hip_stream` and joins it again before the
 *    call returns: everything the call enqueues is ordered before later work on `hip_stream`, also while that
 *    stream is being captured into a HIP graph.  GAD_SERIAL_BACKWARD=1 in the environment keeps all of it on
 *    `hip_stream`.
 *  - Every function returns a gad_status.  Arguments are validated on the host before any kernel
 *    is launched; nothing is launched when the status is an argument error.  gad_last_error()
 *    returns a thread-local, statically stored message for the last failure on this thread.
 *  - Node order is part of the contract: row k < n_local is local_ids[k]; row n_local + j is
 *    halo_ids[j].  No internal reordering is visible through the interface.
 */
#ifndef GAD_H_
#define GAD_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct gad_graph gad_graph; /* opaque: device CSR of A + I, degrees, d~^-1/2, SpMM schedule */

typedef enum {
  GAD_F32 = 0, /* float32 storage, float32 accumulation */
  GAD_BF16 = 1 /* bfloat16 storage of features / activations, float32 accumulation, float32 weights */
} gad_dtype;

typedef enum {
  GAD_OK = 0,
  GAD_ERR_NULL = -1,        /* a required pointer is NULL */
  GAD_ERR_SHAPE = -2,       /* negative / zero / inconsistent sizes */
  GAD_ERR_ID_RANGE = -3,    /* a local or halo id lies outside [0, n_global) */
  GAD_ERR_ID_DUP = -4,      /* an id occurs twice within or across local_ids and halo_ids */
  GAD_ERR_WORKSPACE = -5,   /* workspace too small or misaligned (needs 256-byte alignment) */
  GAD_ERR_WEIGHTS = -6,     /* consensus weights: negative, non-finite, or summing to zero */
  GAD_ERR_HIP = -7,         /* a HIP runtime call failed (message in gad_last_error) */
  GAD_ERR_UNSUPPORTED = -8, /* valid request outside what this build implements */
  GAD_ERR_STATE = -9        /* backward called on a workspace that holds no matching forward */
} gad_status;

const char* gad_last_error(void);

/* ---------------------------------------------------------------------------------------------
 * 1. Augmented-subgraph CSR and normalisation.
 *
 * Builds g' = (v + v', e + e') (Algorithm 1, last step; Algorithm 2, Require) as the CSR of A + I,
 * where A is the adjacency of the induced simple undirected graph on local ++ halo nodes, and the
 * normalisation of A~ in Eq. 7, read as A~ = D~^-1/2 (A + I) D~^-1/2 with D~ = diag(1 + deg), the
 * degrees being those inside g'.
 *
 *   src, dst      [n_edges_in] int64, global ids of the endpoint pairs.  A pair is kept iff both
 *                 ends are in local ++ halo and differ; direction and multiplicity are ignored.
 *                 Pairs with an end outside [0, n_global) are dropped like any pair leaving g'.
 *   local_ids     [n_local] int64, halo_ids [n_halo] int64: distinct ids in [0, n_global).
 *   out           host pointer; receives the new graph.  Destroy with gad_graph_destroy.
 *
 * Result (bit-exact, deterministic): rowptr int64[n+1], colidx int32[nnz] with strictly ascending
 * columns per row and exactly one self loop per row; deg int32[n] (self loop not counted);
 * dinv float32[n] = (1 + deg)^-1/2 evaluated in float64 and rounded once.
 * Device memory of a graph: a little over 8 bytes per non-zero (the column index, the factor dinv[column] again
 * beside it for the sparse product, scheduling data of the rows above 128 non-zeros) and about 24 bytes per row.
 * Errors: NULL pointers (src/dst may be NULL iff n_edges_in = 0, halo_ids iff n_halo = 0),
 * n_local + n_halo = 0 or > 2^31 - 2, 2 * n_edges_in + n >= 2^31, ids out of range, duplicate ids.
 * Synchronises hip_stream (sizes must be read back to allocate the CSR). */
int gad_build_subgraph(const int64_t* src, const int64_t* dst, int64_t n_edges_in, int64_t n_global,
                       const int64_t* local_ids, int64_t n_local, const int64_t* halo_ids, int64_t n_halo,
                       void* hip_stream, gad_graph** out);

/* Sizes and borrowed device pointers of a graph; any output pointer may be NULL. */
int gad_graph_info(const gad_graph* g, int64_t* n, int64_t* n_local, int64_t* nnz, const int64_t** rowptr,
                   const int32_t** colidx, const int32_t** deg, const float** dinv);

int gad_graph_destroy(gad_graph* g);

/* Block-diagonal union of K graphs: the subgraphs one processor holds (Algorithm 2: "each batch g_k in p_i") as
 * ONE graph, so that a forward / backward pass over all of them is one set of launches.  Row i of graphs[k]
 * becomes row (n_0 + .. + n_{k-1}) + i; no edge joins two blocks; degrees and normalisation are the blocks' own.
 * The inputs stay valid and independent.  graphs: host array of K handles, 1 <= K <= 65536.  Synchronises hip_stream. */
int gad_graph_concat(const gad_graph* const* graphs, int K, void* hip_stream, gad_graph** out);

/* Importance-based augmentation of one partition (Section 3.2.2; Algorithm 1): which nodes of the original graph
 * to replicate into the partition.  This is the step that produces the halo_ids of gad_build_subgraph.
 *
 *   G           the ORIGINAL graph as a gad_graph (e.g. gad_build_subgraph with all its nodes as local_ids); the
 *               walks run on it, nodes are its rows.
 *   part_rows   [n_part] int64, distinct rows of G: the partition v_i.
 *   walk_len    l, the number of GCN layers (Property 1: walks of that length reach exactly the candidates of
 *               Definition 2); 1 <= l <= 16.
 *   budget      n(g_i) of Eq. 6, the number of replication nodes wanted (the caller evaluates Eq. 5 / Eq. 6).
 *   seed        walk j is a pure function of (seed, j): start = uniformly drawn boundary node, l uniform steps.
 *   max_walks   cap on the number of walks (<= 2^26).
 *   halo_rows_out  device int64[budget]: the chosen rows of G in selection order;  n_halo_out (host): how many
 *               (fewer than budget when the walks met fewer candidates);  n_walks_out (host, may be NULL).
 * Steps: boundary nodes B (a neighbour outside the partition); a first batch of sum_{v in B} deg(v) walks
 * (Algorithm 1: average boundary degree times |B|); visit counts c_v of the nodes outside the partition, once
 * per walk (Eq. 3, I(v) = c_v / n); total number of walks n = ceil((1.96 / 0.05)^2 (m S2 - S1^2) / S1^2) from
 * Eq. 4 with the mean and population variance of I(v) over the m visited candidates (S1 = sum c, S2 = sum c^2),
 * at least the first batch; walks scored by the sum of I(v) over their steps, taken in descending score (ties:
 * walk number), their nodes added in step order until the budget is met (depth-first selection: no dangling node).
 * Integer arithmetic throughout: the result is exact and reproducible.  Synchronises hip_stream.
 * Errors: rows out of range (GAD_ERR_ID_RANGE) or listed twice (GAD_ERR_ID_DUP), sizes out of range. */
int gad_augment_subgraph(const gad_graph* G, const int64_t* part_rows, int64_t n_part, int32_t walk_len, int64_t budget,
                         uint64_t seed, int64_t max_walks, int64_t* halo_rows_out, int64_t* n_halo_out,
                         int64_t* n_walks_out, void* hip_stream);

/* ---------------------------------------------------------------------------------------------
 * 2./3. Forward and backward propagation (Section 3.3; Algorithm 2, forward and backward steps).
 *
 * Model: H_0 = X;  P_l = A~ H_{l-1} W_l (Eq. 7);  H_l = sigma(P_l) for l < L;  Z = P_L (Eq. 8: no bias,
 * no activation after the last layer);  sigma(p) = p for p > 0, negative_slope * p otherwise: ReLU for
 * negative_slope = 0, LeakyReLU for 0 < negative_slope < 1 (the two activations Eq. 7 names);  y^ = softmax(Z).  Loss (Eq. 9 read as softmax cross-entropy):
 *   loss = loss_scale * sum_{i : mask_i != 0} ( log sum_c exp Z_ic - Z_{i, labels_i} ).
 * Backward (Eq. 10 through the softmax):  G_L = loss_scale * mask_i * (y^ - onehot(labels)),
 *   dW_l = (A~ H_{l-1})^T G_l,   G_{l-1} = (A~ G_l W_l^T) * sigma'(P_{l-1}),  sigma'(p) = 1 for p > 0, negative_slope
 *   otherwise (so ReLU'(0) = 0).
 * Per layer the library evaluates A~ (H W) or (A~ H) W, whichever has the narrower sparse product.
 *
 *   X          [n x dims[0]] features, leading dimension dims[0]; float32, or bfloat16 for GAD_BF16.
 *   dims       host, int32[L+1]: F_0 .. F_L (F_L = number of classes); 1 <= L <= 16, 1 <= F <= 4096.
 *   W          host array of L device pointers; W[l] is float32 [dims[l] x dims[l+1]], ld dims[l+1].
 *   labels     int32[n] in [0, F_L); mask uint8[n] (NULL = all ones).
 *   row_scale  float32[n] or NULL: per-node weight of the loss; node i then carries loss_scale * row_scale[i].
 *              With the blocks of a gad_graph_concat union weighted by c_k * zeta_k / sum_j zeta_j, the gradient
 *              of the pass IS the weighted consensus of Eq. 15 (gradients are linear in these weights).
 *   workspace  device, 256-byte aligned, at least gad_gcn_workspace_bytes(); keeps the activations
 *              between forward and backward.  Its contents are private to the library.
 *   logits_out float32 [n x F_L] (ld F_L) or NULL;  loss_out device double[1] or NULL.
 *   dW         host array of L device pointers; dW[l] is float32 [dims[l] x dims[l+1]], overwritten.
 *   G_out      NULL, or a host array of L device pointers, each NULL or float32 [n x dims[l+1]] (ld dims[l+1])
 *              that receives the per-node gradient G_{l+1} = dLoss/dP_{l+1} (e.g. as node vectors for
 *              gad_subgraph_variance).
 *
 * gad_gcn_backward must follow a gad_gcn_forward on the same graph, workspace, L, dims, dtype and negative_slope
 * (else GAD_ERR_STATE); X and W must still hold the values the forward saw.  One backward per forward: the backward
 * overwrites the forward's seed gradient, so a second backward on the same forward returns GAD_ERR_STATE (the saved
 * activations stay readable through gad_gcn_activation, and the first layer's aggregate stays reusable by
 * gad_gcn_forward_cached).  Rows whose label is outside [0, F_L) contribute nothing (treated as masked).
 *
 * Which forward a workspace holds is kept on the host, keyed by the workspace address; the record is dropped when a
 * forward starts on that address (a forward that fails leaves none), when its graph is destroyed, and by
 * gad_workspace_forget.  The library cannot see a workspace being freed: before the memory of a workspace is freed
 * or used for anything else, call gad_workspace_forget on it -- otherwise a later buffer at the same address would be
 * taken to hold that forward (gad_gcn_backward and gad_gcn_activation would accept it, gad_gcn_forward_cached would
 * reuse an aggregate that is not there).  At most 1024 workspaces are remembered; the oldest record is dropped
 * beyond that. */
int gad_gcn_workspace_bytes(const gad_graph* g, int L, const int32_t* dims, gad_dtype dtype, size_t* bytes);

/* Drops what the library remembers about the forward held by `workspace` (host call, nothing is launched).
 * GAD_OK whether or not anything was remembered. */
int gad_workspace_forget(const void* workspace);

int gad_gcn_forward(const gad_graph* g, const void* X, gad_dtype dtype, int L, const int32_t* dims,
                    const float* const* W, const int32_t* labels, const uint8_t* mask, float loss_scale,
                    const float* row_scale, float negative_slope, void* workspace, size_t workspace_bytes,
                    float* logits_out, double* loss_out, void* hip_stream);

/* gad_gcn_forward for a caller that guarantees that X holds what it held at the last forward on this workspace:
 * the first layer's aggregate A~ X (Eq. 7 applied to H_0 = X) does not depend on the weights, so it is the same
 * in every iteration of Algorithm 2 and is then taken from the workspace instead of being computed again.  Runs
 * the full forward when the workspace holds no forward of this (g, X, L, dims, dtype), or when the first layer
 * transforms before it aggregates (dims[0] > dims[1]).  Same arguments, results and errors as gad_gcn_forward. */
int gad_gcn_forward_cached(const gad_graph* g, const void* X, gad_dtype dtype, int L, const int32_t* dims,
                           const float* const* W, const int32_t* labels, const uint8_t* mask, float loss_scale,
                           const float* row_scale, float negative_slope, void* workspace, size_t workspace_bytes,
                           float* logits_out, double* loss_out, void* hip_stream);

int gad_gcn_backward(const gad_graph* g, const void* X, gad_dtype dtype, int L, const int32_t* dims,
                     const float* const* W, float negative_slope, void* workspace, size_t workspace_bytes,
                     float* const* dW, float* const* G_out, void* hip_stream);

/* Measurement aid: per-layer timing of the two passes (the per-layer edge rate of a layer is nnz over its forward
 * plus its backward time).  events: host array of `count` hipEvent_t created by the caller with timing enabled;
 * the setting belongs to the calling host thread; count = 0 switches it off.  While count >= 2 L + 3, a forward or
 * backward pass of an L-layer model on this thread records, on its stream,
 *   events[0] before its first kernel, events[l] after the last kernel of layer l (1 <= l <= L), events[L + 1] after
 *   the loss and seed gradient (forward);
 *   events[L + 2] before the first kernel of the backward, events[L + 3 + k] after layer L - k is done (0 <= k < L;
 *   the weight-gradient product that otherwise runs beside the next layer's kernels is waited for first, so the
 *   instrumented backward can take a little longer than the plain one).
 * Do not use while the stream is being captured into a HIP graph. */
int gad_gcn_layer_events(void* const* events, int count);

/* Copies a saved activation of the last forward on `workspace` into out (float32 [n x dims[layer]], ld
 * dims[layer]):  layer in [1, L-1] gives H_layer = sigma(P_layer), layer = L gives the logits Z.
 * GAD_ERR_STATE if the workspace holds no forward matching (g, L, dims, dtype). */
int gad_gcn_activation(const gad_graph* g, const void* workspace, size_t workspace_bytes, int L,
                       const int32_t* dims, gad_dtype dtype, int layer, float* out, void* hip_stream);

/* The normalised sparse product on its own (the A~ H of Eq. 7):  out = A~ T.
 *   T, out     [n x width] row-major with leading dimensions ldt, ldo (>= width); float32 or bfloat16.
 *   workspace  device, 16-byte aligned, gad_spmm_workspace_bytes(g, width) bytes (may be NULL when that is 0): the
 *              partial sums of the rows that are split over several waves.
 * out must not alias T.  Exposed so that the dominant kernel can be tested and timed directly. */
int gad_spmm_workspace_bytes(const gad_graph* g, int32_t width, size_t* bytes);
int gad_spmm(const gad_graph* g, const void* T, int64_t ldt, void* out, int64_t ldo, int32_t width,
             gad_dtype dtype, void* workspace, size_t workspace_bytes, void* hip_stream);

/* The dense contractions of Eq. 7 and of its backward step on their own (the H W of the forward pass, the S W^T
 * of the input gradient, and the weight gradient A^T G reduced over the nodes), exposed so that the matrix-core
 * kernels can be tested and timed directly.  Node matrices (A, G, C of gad_gemm_w) are float32, or bfloat16 for
 * GAD_BF16 (then W is rounded to bfloat16 for the product; accumulation is float32 in both cases).
 *   gad_gemm_w:  C[M x N] (ldc) = A[M x K] (lda) op(W);  W float32 row-major [w_rows x w_cols];  op(W) = W
 *                (K = w_rows, N = w_cols), or W^T when transpose_w != 0 (K = w_cols, N = w_rows).
 *   gad_gemm_tn: C[K x N] (ld N, float32) = A[M x K]^T (lda) G[M x N] (ldg), summed over M in a fixed order.
 *   workspace:   device, 256-byte aligned, gad_gemm_workspace_bytes(M, K, N) bytes (serves either call).
 * Errors: K, N outside [1, 4096], M < 0 (M < 1 for gad_gemm_tn), leading dimension below the row length. */
int gad_gemm_workspace_bytes(int64_t M, int32_t K, int32_t N, size_t* bytes);
int gad_gemm_w(const void* A, int64_t lda, const float* W, int32_t w_rows, int32_t w_cols, int transpose_w, void* C,
               int64_t ldc, int64_t M, gad_dtype dtype, void* workspace, size_t workspace_bytes, void* hip_stream);
int gad_gemm_tn(const void* A, int64_t lda, const void* G, int64_t ldg, float* C, int64_t M, int32_t K, int32_t N,
                gad_dtype dtype, void* workspace, size_t workspace_bytes, void* hip_stream);

/* ---------------------------------------------------------------------------------------------
 * 4. Variance-based subgraph importance (Section 3.4.1, Eq. 14 and its worked example).
 *
 *   zeta = S_pp / (D + beta),  S_pp = sum_{i<j} p_i p_j,  p_i = deg_i / sum_k deg_k (deg without the
 *   self loop, all unordered pairs: fixed by the worked example),  D = sqrt(2 var),
 *   var = (1/n) sum_i ||v_i - mean(v)||^2 (squared deviations summed over the F dimensions), i.e. D is
 *   the root-mean-square Euclidean distance over all node pairs.  sum deg and sum deg^2 are exact
 *   64-bit integers.  An edgeless subgraph has S_pp = zeta = 0.
 *
 *   V            [n x F] node vectors (features, an activation, or per-node gradients), ld = F.
 *   out3         device double[3]: zeta, S_pp, var.
 *   per_node_out float32[n] = ||v_i - mean(v)||^2, or NULL.
 * Errors: beta <= 0 or non-finite, F < 1. */
int gad_subgraph_variance(const gad_graph* g, const void* V, int32_t F, gad_dtype dtype, double beta,
                          double* out3, float* per_node_out, void* hip_stream);

/* gad_subgraph_variance for callers that cannot allocate device memory or tolerate a library that does (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same kernels and the same results,
 * but the reduction buffer is a fixed array inside the library (4.8 MB of device memory on every GPU the library
 * runs on, held until the process ends) instead of memory owned by the graph.  The call allocates and frees
 * nothing.  Limits: F <= 1024 and n <= 8,388,608 (GAD_ERR_SHAPE beyond them, nothing launched).  The current device
 * must be the graph's (GAD_ERR_STATE).  All calls on one GPU share the one array: calls that overlap on a GPU
 * (different streams or threads) race; calls on one stream are ordered.  Nothing in the array has to start at
 * zero: every word a kernel reads is written earlier in the same call.  The first call on a device looks up the
 * array's device address; make that call outside a stream capture. */
int gad_subgraph_variance_static(const gad_graph* g, const void* V, int32_t F, gad_dtype dtype, double beta,
                                 double* out3, float* per_node_out, void* hip_stream);

/* Eq. 14 read with the distance inside the sum (the formula as printed sums only its numerator and leaves i, j
 * free in the denominator; with identical node vectors, as in the paper's worked example, both readings agree):
 *
 *   zeta_pair = sum_{i<j} p_i p_j / (||v_i - v_j||_2 + beta),   p_i as above.
 *
 * All n (n - 1) / 2 pairs are visited: the cost is O(n^2 F).
 *   V          [n x F] node vectors, ld = F; float32 or bfloat16.
 *   out2       device double[2]: zeta_pair, S_pp.
 *   workspace  device, 256-byte aligned, gad_pair_importance_workspace_bytes(g, F) bytes.
 * The pair terms are formed in float32 (distances below 1e-19 count as 0) and summed in float64.
 * Errors: as gad_subgraph_variance; beta outside the normal float32 range; n above about 47 million (more pair
 * tiles than one launch holds). */
int gad_pair_importance_workspace_bytes(const gad_graph* g, int32_t F, size_t* bytes);
int gad_pair_importance(const gad_graph* g, const void* V, int32_t F, gad_dtype dtype, double beta, double* out2,
                        void* workspace, size_t workspace_bytes, void* hip_stream);

/* ---------------------------------------------------------------------------------------------
 * 5. Weighted global consensus (Section 3.4.2, Eq. 15; Eq. 11 is the case of equal zeta).
 *
 *   out[e] = sum_k (zeta_k / sum_j zeta_j) * bufs[k][e],  weights formed in float64.
 *
 *   bufs   host array of K device pointers to float32[n_elems];  zeta host double[K];  1 <= K <= 128.
 *   out    float32[n_elems]; may alias any bufs[k].
 * Errors: K out of range, any zeta_k negative or non-finite, sum zeta = 0 (GAD_ERR_WEIGHTS). */
int gad_weighted_consensus(const float* const* bufs, int K, const double* zeta, int64_t n_elems, float* out,
                           void* hip_stream);

/* ---------------------------------------------------------------------------------------------
 * 6. Consensus with parameter update, and one synchronous training round (Algorithm 2, the steps after the
 *    per-processor loop; Eq. 15 followed by Eq. 16, read as plain SGD:  W <- W - eta * grad_hat).
 *
 * gad_consensus_update:  params[e] <- params[e] - eta * sum_k (zeta_k / sum_j zeta_j) * grads[k][e];
 *   the averaged gradient is also written to avg_out when avg_out != NULL.  grads: host array of K device
 *   pointers to float32[n_elems]; params must not alias any of them.  Errors as gad_weighted_consensus.
 *
 * gad_train_round: the K subgraphs play the K processors of Algorithm 2 on one device.  All of them see the same
 *   parameters (one flat float32 buffer `params` holding W_1 .. W_L back to back, W_l row-major
 *   [dims[l-1] x dims[l]]); for k = 0..K-1 a forward and a backward on graphs[k] fill gradient copy k
 *   (grads + k * n_params, same layout), then gad_consensus_update is applied with zeta (host, K doubles) and eta.
 *   X, labels, masks, workspaces: host arrays of K device pointers (masks or masks[k] may be NULL);
 *   loss_scales, workspace_bytes: host arrays of K values; losses: device double[K] or NULL.
 *   x_unchanged != 0: the caller vouches that every X[k] holds what it held at the last round on workspaces[k];
 *   the forward passes then run as gad_gcn_forward_cached (the features of Algorithm 2 do not change between
 *   rounds, so every round after the first can say so).
 *   Nothing is launched if the weights are invalid. */
int gad_consensus_update(const float* const* grads, int K, const double* zeta, int64_t n_elems, float eta,
                         float* params, float* avg_out, void* hip_stream);

/* One synchronous round of Algorithm 2 over the blocks of a gad_graph_concat union in one pass: forward with
 * row_scale[i] = c_k * zeta_k / sum_j zeta_j on the rows of block k (c_k = the block's own loss scale), backward
 * into `grad` (float32[n_params], the layout of `params`) -- which is the weighted consensus gradient of Eq. 15 --
 * then params <- params - eta * grad (Eq. 16).  loss (device double[1] or NULL) receives the weighted loss
 * sum_k (zeta_k / sum zeta) loss_k.  Other arguments (x_unchanged included) as gad_gcn_forward / gad_train_round. */
int gad_train_round_batched(const gad_graph* g, const void* X, gad_dtype dtype, int L, const int32_t* dims, float* params,
                            const int32_t* labels, const uint8_t* mask, const float* row_scale, float negative_slope,
                            void* workspace, size_t workspace_bytes, float* grad, float eta, double* loss,
                            int x_unchanged, void* hip_stream);

int gad_train_round(int K, const gad_graph* const* graphs, const void* const* X, gad_dtype dtype, int L,
                    const int32_t* dims, float* params, const int32_t* const* labels, const uint8_t* const* masks,
                    const float* loss_scales, float negative_slope, void* const* workspaces,
                    const size_t* workspace_bytes, float* grads, const double* zeta, float eta, double* losses,
                    int x_unchanged, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* GAD_H_ */
