/* CSR-level CPU oracle (tier T1) for GAD's per-processor GCN step.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain C + OpenMP, float64 arithmetic, no blocking or fusion: every function is the
 * definition written out over a CSR.  It shares no code with the HIP path and is
 * called only by tests, the smoke check and the benchmark's CPU-baseline leg
 * (through oracle/gad_csr.py).  It is validated against the dense definition-level
 * oracle (oracle/gad_dense.py) on small graphs and scales to the large workloads.
 *
 * Paper: arXiv 2110.02987.  g' = (v + v', e + e'): Algorithm 1 (last step) / Algorithm 2
 * (Require); A~ of Eq. 7 read as D~^-1/2 (A+I) D~^-1/2 with degrees inside g';
 * Eq. 14 (variance-based importance) under the aggregate-distance reading.
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC oracle/csr_oracle.c -o oracle/libgad_oracle.so -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define T1_OK 0
#define T1_ERR_ID_RANGE (-3)
#define T1_ERR_ID_DUP (-4)
#define T1_ERR_NOMEM (-9)

int t1_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

static int cmp_i32(const void* a, const void* b) {
  int32_t x = *(const int32_t*)a, y = *(const int32_t*)b;
  return (x > y) - (x < y);
}

/* Induced simple undirected graph on local ++ halo, plus one self loop per row, as CSR.
 * Row k < n_local is local_ids[k]; row n_local + j is halo_ids[j].  Columns ascending.
 * rowptr_out must hold n+1 int64.  *colidx_out is malloc'ed (free with t1_free). */
int t1_build(const int64_t* src, const int64_t* dst, int64_t n_edges, int64_t n_global,
             const int64_t* local_ids, int64_t n_local, const int64_t* halo_ids, int64_t n_halo,
             int64_t* rowptr_out, int32_t** colidx_out, int64_t* nnz_out) {
  int64_t n = n_local + n_halo;
  int64_t* lut = (int64_t*)malloc(sizeof(int64_t) * (size_t)(n_global > 0 ? n_global : 1));
  if (!lut) return T1_ERR_NOMEM;
  for (int64_t g = 0; g < n_global; ++g) lut[g] = -1;
  for (int64_t k = 0; k < n; ++k) {
    int64_t id = k < n_local ? local_ids[k] : halo_ids[k - n_local];
    if (id < 0 || id >= n_global) { free(lut); return T1_ERR_ID_RANGE; }
    if (lut[id] != -1) { free(lut); return T1_ERR_ID_DUP; }
    lut[id] = k;
  }
  /* pass 1: count both directions of every kept pair, plus the self loop */
  int64_t* cnt = (int64_t*)calloc((size_t)n + 1, sizeof(int64_t));
  if (!cnt) { free(lut); return T1_ERR_NOMEM; }
  for (int64_t k = 0; k < n; ++k) cnt[k + 1] = 1;
  for (int64_t e = 0; e < n_edges; ++e) {
    if (src[e] < 0 || src[e] >= n_global || dst[e] < 0 || dst[e] >= n_global) continue;
    int64_t r = lut[src[e]], c = lut[dst[e]];
    if (r < 0 || c < 0 || r == c) continue;
    cnt[r + 1]++; cnt[c + 1]++;
  }
  for (int64_t k = 0; k < n; ++k) cnt[k + 1] += cnt[k];
  int64_t total = cnt[n];
  int32_t* raw = (int32_t*)malloc(sizeof(int32_t) * (size_t)(total > 0 ? total : 1));
  int64_t* cur = (int64_t*)malloc(sizeof(int64_t) * (size_t)(n > 0 ? n : 1));
  if (!raw || !cur) { free(lut); free(cnt); free(raw); free(cur); return T1_ERR_NOMEM; }
  for (int64_t k = 0; k < n; ++k) { cur[k] = cnt[k]; raw[cur[k]++] = (int32_t)k; }
  for (int64_t e = 0; e < n_edges; ++e) {
    if (src[e] < 0 || src[e] >= n_global || dst[e] < 0 || dst[e] >= n_global) continue;
    int64_t r = lut[src[e]], c = lut[dst[e]];
    if (r < 0 || c < 0 || r == c) continue;
    raw[cur[r]++] = (int32_t)c;
    raw[cur[c]++] = (int32_t)r;
  }
  free(lut); free(cur);
  /* per row: sort, drop repeats */
  int64_t* uniq = (int64_t*)malloc(sizeof(int64_t) * (size_t)(n > 0 ? n : 1));
  if (!uniq) { free(cnt); free(raw); return T1_ERR_NOMEM; }
#pragma omp parallel for schedule(dynamic, 256)
  for (int64_t k = 0; k < n; ++k) {
    int32_t* seg = raw + cnt[k];
    int64_t len = cnt[k + 1] - cnt[k];
    qsort(seg, (size_t)len, sizeof(int32_t), cmp_i32);
    int64_t u = 0;
    for (int64_t j = 0; j < len; ++j)
      if (j == 0 || seg[j] != seg[j - 1]) seg[u++] = seg[j];
    uniq[k] = u;
  }
  rowptr_out[0] = 0;
  for (int64_t k = 0; k < n; ++k) rowptr_out[k + 1] = rowptr_out[k] + uniq[k];
  int64_t nnz = rowptr_out[n];
  int32_t* col = (int32_t*)malloc(sizeof(int32_t) * (size_t)(nnz > 0 ? nnz : 1));
  if (!col) { free(cnt); free(raw); free(uniq); return T1_ERR_NOMEM; }
#pragma omp parallel for schedule(static)
  for (int64_t k = 0; k < n; ++k)
    memcpy(col + rowptr_out[k], raw + cnt[k], sizeof(int32_t) * (size_t)uniq[k]);
  free(cnt); free(raw); free(uniq);
  *colidx_out = col;
  *nnz_out = nnz;
  return T1_OK;
}

void t1_copy_colidx(const int32_t* col, int64_t nnz, int32_t* dst) {
  memcpy(dst, col, sizeof(int32_t) * (size_t)nnz);
}

void t1_free(void* p) { free(p); }

/* deg_i = (row length) - 1  (the self loop is not a neighbour);  dinv_i = (1 + deg_i)^-1/2,
 * computed in float64 and rounded once to float32. */
void t1_degree(const int64_t* rowptr, int64_t n, int32_t* deg, float* dinv) {
  for (int64_t i = 0; i < n; ++i) {
    int64_t d = rowptr[i + 1] - rowptr[i] - 1;
    deg[i] = (int32_t)d;
    dinv[i] = (float)(1.0 / sqrt((double)(d + 1)));
  }
}

/* out = A~ T,  A~_ij = 1 / sqrt(d~_i d~_j) on the pattern of A + I,  d~_i = row length.  T, out: [n x w] float64. */
void t1_spmm(const int64_t* rowptr, const int32_t* colidx, int64_t n, int64_t w, const double* T, double* out) {
#pragma omp parallel for schedule(dynamic, 64)
  for (int64_t i = 0; i < n; ++i) {
    double* o = out + i * w;
    for (int64_t f = 0; f < w; ++f) o[f] = 0.0;
    double di = (double)(rowptr[i + 1] - rowptr[i]);
    for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
      int64_t j = colidx[p];
      double dj = (double)(rowptr[j + 1] - rowptr[j]);
      double a = 1.0 / sqrt(di * dj);
      const double* t = T + j * w;
      for (int64_t f = 0; f < w; ++f) o[f] += a * t[f];
    }
  }
}

/* Selected rows of A~ T with T stored as float32 (used to check sampled outputs of large workloads). */
void t1_spmm_rows_f32(const int64_t* rowptr, const int32_t* colidx, int64_t w, int64_t ld, const float* T,
                      const int64_t* rows, int64_t n_rows, double* out) {
#pragma omp parallel for schedule(dynamic, 8)
  for (int64_t k = 0; k < n_rows; ++k) {
    int64_t i = rows[k];
    double* o = out + k * w;
    for (int64_t f = 0; f < w; ++f) o[f] = 0.0;
    double di = (double)(rowptr[i + 1] - rowptr[i]);
    for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
      int64_t j = colidx[p];
      double dj = (double)(rowptr[j + 1] - rowptr[j]);
      double a = 1.0 / sqrt(di * dj);
      const float* t = T + j * ld;
      for (int64_t f = 0; f < w; ++f) o[f] += a * (double)t[f];
    }
  }
}

/* Eq. 14 pieces.  s[0] = sum deg, s[1] = sum deg^2 (exact integers). */
void t1_degree_sums(const int32_t* deg, int64_t n, int64_t* s) {
  int64_t s1 = 0, s2 = 0;
  for (int64_t i = 0; i < n; ++i) { s1 += deg[i]; s2 += (int64_t)deg[i] * deg[i]; }
  s[0] = s1; s[1] = s2;
}

/* r_i = ||v_i - vbar||^2 summed over the F dimensions; returns var = mean_i r_i.  V: [n x F] float64. */
double t1_deviation(const double* V, int64_t n, int64_t F, double* r /* [n] */) {
  double* mean = (double*)calloc((size_t)F, sizeof(double));
  for (int64_t i = 0; i < n; ++i)
    for (int64_t f = 0; f < F; ++f) mean[f] += V[i * F + f];
  for (int64_t f = 0; f < F; ++f) mean[f] /= (double)n;
  double tot = 0.0;
  for (int64_t i = 0; i < n; ++i) {
    double s = 0.0;
    for (int64_t f = 0; f < F; ++f) { double d = V[i * F + f] - mean[f]; s += d * d; }
    r[i] = s;
    tot += s;
  }
  free(mean);
  return n > 0 ? tot / (double)n : 0.0;
}

/* Eq. 14 with the distance inside the sum: sum_{i<j} deg_i deg_j / (||v_i - v_j||_2 + beta), to be divided by
 * (sum deg)^2 by the caller.  Plain double loop over the pairs (rows of the pair matrix shared among threads);
 * V: [n x F] float64. */
double t1_pair_sum(const int32_t* deg, const double* V, int64_t n, int64_t F, double beta) {
  double tot = 0.0;
#pragma omp parallel for schedule(dynamic, 16) reduction(+ : tot)
  for (int64_t i = 0; i < n; ++i) {
    const double* vi = V + i * F;
    double row = 0.0;
    for (int64_t j = i + 1; j < n; ++j) {
      const double* vj = V + j * F;
      double d2 = 0.0;
      for (int64_t f = 0; f < F; ++f) { double d = vi[f] - vj[f]; d2 += d * d; }
      row += (double)deg[j] / (sqrt(d2) + beta);
    }
    tot += (double)deg[i] * row;
  }
  return tot;
}

