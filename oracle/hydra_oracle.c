/*
 * fp64 CPU oracle for packed variable-length attention.  TEST INFRASTRUCTURE ONLY:
 * nothing on the product path may call into this file.  It shares no code, header,
 * table or helper with the HIP kernels.
 *
 * What is computed (textbook scaled-dot-product attention, the operation whose cost
 * the paper models as "multiply the query with the key, then multiply the value",
 * Appendix "Computation and Memory Access in MLLMs", attention equations, and
 * Table 2 rows Attention/encode and Attention/prefill):
 *
 *   for every sequence b with packed token range [cu[b], cu[b+1]) of length L,
 *   every query head h (KV head hk = h / (Hq/Hkv)), every local query index i:
 *     visible keys J(i) = {0..L-1} (bidirectional)  or  {0..i} (causal)
 *     z_j = scale * <Q[s+i,h,:], K[s+j,hk,:]>              j in J(i)
 *     p_j = exp(z_j - max_J z) / sum_{j' in J} exp(z_j' - max_J z)
 *     O[s+i,h,:] = sum_{j in J(i)} p_j * V[s+j,hk,:]
 *
 * All arithmetic is IEEE double.  The mask is an explicit L x L byte matrix per
 * sequence, applied as -infinity before the softmax.  No tiling, no running
 * (online) softmax, no reordering: one row at a time, three plain passes.
 * Sequences are independent (Section 2.1: each request's tokens form its own
 * input X of length s = n + m; stage-level batching only packs them together).
 *
 * Layouts: q [N, Hq, d], k and v [N, Hkv, d], out [N, Hq, d], row-major doubles.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Explicit visibility mask for one sequence: m[i*L + j] = 1 iff key j is visible to query i. */
static unsigned char* build_mask(int L, int causal) {
  unsigned char* m = (unsigned char*)malloc((size_t)L * (size_t)L + 1);
  if (!m) return NULL;
  for (int i = 0; i < L; i++)
    for (int j = 0; j < L; j++) m[(size_t)i * L + j] = causal ? (j <= i) : 1;
  return m;
}

/* One output row.  z is scratch of length L; if probs != NULL the normalised
 * probabilities (0 for masked keys) are written there.  Returns the number of visible keys. */
static int attend_row(const double* qrow, const double* kbase, const double* vbase, int L, int kv_stride, int d,
                      const unsigned char* mask_row, double scale, double* z, double* probs, double* orow) {
  int visible = 0;
  double zmax = -INFINITY;
  for (int j = 0; j < L; j++) {
    if (mask_row[j]) {
      double acc = 0.0;
      const double* kr = kbase + (size_t)j * kv_stride;
      for (int c = 0; c < d; c++) acc += qrow[c] * kr[c];
      z[j] = scale * acc;
      visible++;
    } else {
      z[j] = -INFINITY;
    }
    if (z[j] > zmax) zmax = z[j];
  }
  double denom = 0.0;
  for (int j = 0; j < L; j++) {
    z[j] = mask_row[j] ? exp(z[j] - zmax) : 0.0;
    denom += z[j];
  }
  for (int c = 0; c < d; c++) orow[c] = 0.0;
  for (int j = 0; j < L; j++) {
    double p = z[j] / denom;
    if (probs) probs[j] = p;
    if (p != 0.0) {
      const double* vr = vbase + (size_t)j * kv_stride;
      for (int c = 0; c < d; c++) orow[c] += p * vr[c];
    }
  }
  return visible;
}

/* Full packed batch.  Returns 0, or a negative code on bad arguments / allocation failure.
 * nthreads <= 0 means "all cores OpenMP reports".  *threads_used receives the team size. */
int hydra_oracle_attn_varlen(const double* q, const double* k, const double* v, double* out, const int32_t* cu,
                             int batch, int n_q_heads, int n_kv_heads, int head_dim, int causal, double scale,
                             int nthreads, int* threads_used) {
  if (batch < 0 || n_q_heads <= 0 || n_kv_heads <= 0 || head_dim <= 0 || n_q_heads % n_kv_heads) return -1;
  const int g = n_q_heads / n_kv_heads;
  int status = 0, used = 1;
#ifdef _OPENMP
  if (nthreads <= 0) nthreads = omp_get_max_threads();
#else
  nthreads = 1;
#endif
  for (int b = 0; b < batch; b++) {
    const int s = cu[b], L = cu[b + 1] - cu[b];
    if (L < 0) return -2;
    if (L == 0) continue;
    unsigned char* mask = build_mask(L, causal);
    if (!mask) return -3;
    const int units = n_q_heads * L;
#pragma omp parallel num_threads(nthreads)
    {
#ifdef _OPENMP
#pragma omp single
      used = omp_get_num_threads(); /* one thread writes; the construct ends with a barrier */
#endif
      double* z = (double*)malloc(sizeof(double) * (size_t)L);
#pragma omp for schedule(dynamic, 16)
      for (int u = 0; u < units; u++) {
        const int h = u / L, i = u % L, hk = h / g;
        if (!z) {
#pragma omp atomic write
          status = -3;
          continue;
        }
        int vis = attend_row(q + ((size_t)(s + i) * n_q_heads + h) * head_dim, k + ((size_t)s * n_kv_heads + hk) * head_dim,
                             v + ((size_t)s * n_kv_heads + hk) * head_dim, L, n_kv_heads * head_dim, head_dim,
                             mask + (size_t)i * L, scale, z, NULL, out + ((size_t)(s + i) * n_q_heads + h) * head_dim);
        if (vis == 0) { /* a row with no visible key cannot occur for L >= 1 */
#pragma omp atomic write
          status = -4;
        }
      }
      free(z);
    }
    free(mask);
    if (status) return status;
  }
  if (threads_used) *threads_used = used;
  return 0;
}

/* Selected rows only: rows[2*r] = packed token index, rows[2*r+1] = query head.
 * out_rows [n_rows, d].  If probs != NULL it is [n_rows, max_len] and receives each row's
 * probabilities over its own sequence (zero padded).  Same row routine as the full call. */
int hydra_oracle_attn_rows(const double* q, const double* k, const double* v, const int32_t* cu, int batch,
                           int n_q_heads, int n_kv_heads, int head_dim, int causal, double scale, const int32_t* rows,
                           int n_rows, double* out_rows, double* probs, int max_len) {
  if (batch < 0 || n_q_heads <= 0 || n_kv_heads <= 0 || head_dim <= 0 || n_q_heads % n_kv_heads) return -1;
  const int g = n_q_heads / n_kv_heads;
  int status = 0;
#pragma omp parallel for schedule(dynamic, 1)
  for (int r = 0; r < n_rows; r++) {
    const int t = rows[2 * r], h = rows[2 * r + 1];
    int b = -1;
    for (int bb = 0; bb < batch; bb++)
      if (t >= cu[bb] && t < cu[bb + 1]) b = bb;
    if (b < 0 || h < 0 || h >= n_q_heads) {
#pragma omp atomic write
      status = -5;
      continue;
    }
    const int s = cu[b], L = cu[b + 1] - cu[b], i = t - s, hk = h / g;
    if (probs && L > max_len) {
#pragma omp atomic write
      status = -6;
      continue;
    }
    /* the explicit mask row for query i of this sequence */
    unsigned char* mrow = (unsigned char*)malloc((size_t)L);
    double* z = (double*)malloc(sizeof(double) * (size_t)L);
    if (!mrow || !z) {
#pragma omp atomic write
      status = -3;
      free(mrow);
      free(z);
      continue;
    }
    for (int j = 0; j < L; j++) mrow[j] = causal ? (j <= i) : 1;
    double* pr = probs ? probs + (size_t)r * max_len : NULL;
    if (pr) memset(pr, 0, sizeof(double) * (size_t)max_len);
    attend_row(q + ((size_t)t * n_q_heads + h) * head_dim, k + ((size_t)s * n_kv_heads + hk) * head_dim,
               v + ((size_t)s * n_kv_heads + hk) * head_dim, L, n_kv_heads * head_dim, head_dim, mrow, scale, z, pr,
               out_rows + (size_t)r * head_dim);
    free(mrow);
    free(z);
  }
  return status;
}

/* Number of (query, key) pairs the explicit masks leave visible, summed over sequences
 * (per head).  Bidirectional: sum L^2, the T^2 of the paper's attention FLOP formula. */
long long hydra_oracle_unmasked_pairs(const int32_t* cu, int batch, int causal) {
  long long total = 0;
  for (int b = 0; b < batch; b++) {
    const int L = cu[b + 1] - cu[b];
    if (L <= 0) continue;
    unsigned char* mask = build_mask(L, causal);
    if (!mask) return -1;
    for (size_t e = 0; e < (size_t)L * L; e++) total += mask[e];
    free(mask);
  }
  return total;
}
