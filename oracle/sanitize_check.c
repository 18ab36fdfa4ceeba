/* Host-side sanitizer leg for the C oracle (test infrastructure, CPU only).
 *
 * Linked with hydra_oracle.c under -fsanitize=address,undefined by tests/test_host_sanitizers.py.
 * Runs the oracle's entry points over ragged packed batches (zero-length and one-token sequences,
 * lengths around the kernels' tile sizes, grouped heads, both masks, several OpenMP threads) so that
 * an out-of-bounds access, a leak, a misaligned or overflowing operation in the oracle is reported,
 * and checks every output row against a scalar evaluation of the definition written out here:
 *   z_j = scale * <q_i, k_j> over the visible keys (all keys, or j <= i with the causal mask),
 *   p = softmax(z), out_i = sum_j p_j v_j, query head h reading KV head h / (Hq / Hkv)
 * (scaled-dot-product attention as in the paper's Table 2, rows Attention/encode and /prefill).
 * Exit status 0: clean and equal; 1: mismatch or error code.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int hydra_oracle_attn_varlen(const double* q, const double* k, const double* v, double* out, const int32_t* cu, int batch, int n_q_heads,
                             int n_kv_heads, int head_dim, int causal, double scale, int nthreads, int* threads_used);
int hydra_oracle_attn_rows(const double* q, const double* k, const double* v, const int32_t* cu, int batch, int n_q_heads, int n_kv_heads,
                           int head_dim, int causal, double scale, const int32_t* rows, int n_rows, double* out_rows, double* probs,
                           int max_len);
long long hydra_oracle_unmasked_pairs(const int32_t* cu, int batch, int causal);

static uint64_t rng_state = 0x9e3779b97f4a7c15ull;
static double next_value(void) { /* uniform in [-1, 1), from a 64-bit LCG */
  rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull;
  return (double)(int64_t)(rng_state >> 11) / (double)(1ll << 52) - 1.0;
}

static double* filled(size_t n) {
  double* p = (double*)malloc(sizeof(double) * (n ? n : 1));
  if (!p) exit(1);
  for (size_t i = 0; i < n; i++) p[i] = next_value();
  return p;
}

static int run_case(const int* lengths, int batch, int hq, int hkv, int d, int causal) {
  int32_t* cu = (int32_t*)malloc(sizeof(int32_t) * (size_t)(batch + 1));
  if (!cu) exit(1);
  cu[0] = 0;
  int max_len = 1;
  for (int b = 0; b < batch; b++) {
    cu[b + 1] = cu[b] + lengths[b];
    if (lengths[b] > max_len) max_len = lengths[b];
  }
  const int n = cu[batch], g = hq / hkv;
  const double scale = 1.0 / sqrt((double)d);
  double *q = filled((size_t)n * hq * d), *k = filled((size_t)n * hkv * d), *v = filled((size_t)n * hkv * d);
  double* out = (double*)calloc((size_t)n * hq * d + 1, sizeof(double));
  int used = 0, bad = 0;
  if (!out) exit(1);
  if (hydra_oracle_attn_varlen(q, k, v, out, cu, batch, hq, hkv, d, causal, scale, 4, &used) != 0) bad = 1;

  /* closed-form pair count against the oracle's explicit masks */
  long long pairs = 0;
  for (int b = 0; b < batch; b++) pairs += causal ? (long long)lengths[b] * (lengths[b] + 1) / 2 : (long long)lengths[b] * lengths[b];
  if (hydra_oracle_unmasked_pairs(cu, batch, causal) != pairs) bad = 1;

  /* every row again through the row-wise entry point (with probabilities), and by the scalar definition */
  int32_t* rows = (int32_t*)malloc(sizeof(int32_t) * 2 * (size_t)(n * hq + 1));
  double* out_rows = (double*)malloc(sizeof(double) * ((size_t)n * hq * d + 1));
  double* probs = (double*)malloc(sizeof(double) * ((size_t)n * hq * max_len + 1));
  double* z = (double*)malloc(sizeof(double) * (size_t)max_len);
  if (!rows || !out_rows || !probs || !z) exit(1);
  for (int t = 0; t < n; t++)
    for (int h = 0; h < hq; h++) {
      rows[2 * (t * hq + h)] = t;
      rows[2 * (t * hq + h) + 1] = h;
    }
  if (hydra_oracle_attn_rows(q, k, v, cu, batch, hq, hkv, d, causal, scale, rows, n * hq, out_rows, probs, max_len) != 0) bad = 1;
  for (int b = 0; b < batch && !bad; b++) {
    const int s = cu[b], L = lengths[b];
    for (int i = 0; i < L; i++)
      for (int h = 0; h < hq; h++) {
        const int hk = h / g, last = causal ? i : L - 1;
        double zmax = -INFINITY, denom = 0.0, psum = 0.0;
        for (int j = 0; j <= last; j++) {
          double acc = 0.0;
          for (int c = 0; c < d; c++) acc += q[((size_t)(s + i) * hq + h) * d + c] * k[((size_t)(s + j) * hkv + hk) * d + c];
          z[j] = scale * acc;
          if (z[j] > zmax) zmax = z[j];
        }
        for (int j = 0; j <= last; j++) denom += exp(z[j] - zmax);
        const size_t r = (size_t)(s + i) * hq + h;
        for (int j = 0; j < max_len; j++) psum += probs[r * max_len + j];
        if (fabs(psum - 1.0) > 1e-12) bad = 1;
        for (int c = 0; c < d; c++) {
          double want = 0.0;
          for (int j = 0; j <= last; j++) want += exp(z[j] - zmax) / denom * v[((size_t)(s + j) * hkv + hk) * d + c];
          if (fabs(out[r * d + c] - want) > 1e-12 || fabs(out_rows[r * d + c] - want) > 1e-12) bad = 1;
        }
      }
  }
  printf("lengths[%d] hq %d hkv %d d %d causal %d threads %d: %s\n", batch, hq, hkv, d, causal, used, bad ? "MISMATCH" : "ok");
  free(cu); free(q); free(k); free(v); free(out); free(rows); free(out_rows); free(probs); free(z);
  return bad;
}

int main(void) {
  static const int ragged[] = {17, 0, 64, 1, 100, 65, 0, 33};
  static const int small[] = {1, 2, 3};
  static const int one[] = {129};
  int bad = 0;
  for (int causal = 0; causal < 2; causal++) {
    bad |= run_case(ragged, 8, 4, 2, 16, causal);
    bad |= run_case(small, 3, 3, 1, 8, causal);
    bad |= run_case(one, 1, 2, 2, 24, causal);
    bad |= run_case(ragged, 0, 2, 2, 8, causal); /* empty batch */
  }
  /* argument errors return codes, touching nothing */
  int32_t cu_bad[2] = {0, -1};
  if (hydra_oracle_attn_varlen(NULL, NULL, NULL, NULL, cu_bad, 1, 2, 2, 8, 0, 1.0, 1, NULL) != -2) bad = 1;
  if (hydra_oracle_attn_varlen(NULL, NULL, NULL, NULL, cu_bad, 1, 3, 2, 8, 0, 1.0, 1, NULL) != -1) bad = 1;
  return bad;
}
