/*
 * CPU oracle for context-parallel ring attention: TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, fp64 statement of what the per-rank hot path computes. It is
 * used by the tests, by the smoke check and by the benchmark's CPU baseline
 * leg, and by nothing else. It shares no code with the HIP library: no
 * headers, helpers, tables or constants.
 *
 * Every function follows the defining formula directly, with no blocking,
 * fusion or re-ordering:
 *
 *   oracle_attn   - scaled dot-product attention and its log-sum-exp
 *                   (Appendix B "Merge Attention": O = softmax(QK^T/sqrt(d))V,
 *                   LSE = log sum_i exp(Q.K_i/sqrt(d))), restricted to the
 *                   keys a query may see under causal attention ("each token
 *                   attends to all tokens before it in the same sequence",
 *                   Section 3.5.1), with the GQA head grouping of Section 3.4
 *                   (shape(Q) = [T, N_H, D_H], shape(K) = [T+P, N_KV, D_H]).
 *   oracle_merge  - Appendix B, Equation 4 (merge of partial outputs).
 *
 * Readings of points the paper leaves open (all listed in the design notes):
 *   - the diagonal is visible: key j is seen by query i iff kv_pos[j] <= q_pos[i];
 *   - a query with no visible key yields O = 0 and LSE = -inf;
 *   - a merge whose partials all have LSE = -inf yields O = 0, LSE = -inf;
 *   - the merged LSE is LSE_max + log sum_s exp(LSE_s - LSE_max), which is the
 *     LSE definition of Appendix B applied to the union of the key sets;
 *   - query head h reads KV head h / (N_H / N_KV).
 *
 * Parity pins: see tests/test_oracle_*.py (closed forms, a library attention
 * routine on the unsharded special case, brute force written independently in
 * NumPy, the sharded == unsharded invariant, permutation invariance).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void oracle_set_num_threads(int n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

/*
 * q   [total_q,  n_q_heads,  d]   fp64 (exact upcast of the values the GPU sees)
 * k,v [total_kv, n_kv_heads, d]
 * q_pos [total_q], kv_pos [total_kv]: absolute token positions
 * cu_q, cu_kv [batch+1]: packed sequence boundaries, or NULL when batch == 1
 * out [total_q, n_q_heads, d], lse [total_q, n_q_heads]
 * Returns the number of visible (query, key) pairs summed over rows
 * (counted once per query token, not per head).
 */
int64_t oracle_attn(const double *q, const double *k, const double *v,
                    const int32_t *q_pos, const int32_t *kv_pos,
                    const int32_t *cu_q, const int32_t *cu_kv, int32_t batch,
                    int64_t total_q, int64_t total_kv, int32_t n_q_heads,
                    int32_t n_kv_heads, int32_t d, double scale, double *out,
                    double *lse) {
  const int group = n_q_heads / n_kv_heads;
  int64_t pairs = 0;
  for (int32_t b = 0; b < batch; ++b) {
    const int64_t q0 = cu_q ? cu_q[b] : 0, q1 = cu_q ? cu_q[b + 1] : total_q;
    const int64_t k0 = cu_kv ? cu_kv[b] : 0, k1 = cu_kv ? cu_kv[b + 1] : total_kv;
#pragma omp parallel for schedule(dynamic, 1) reduction(+ : pairs)
    for (int64_t i = q0; i < q1; ++i) {
      double *s = (double *)malloc(sizeof(double) * (size_t)(k1 - k0 + 1));
      for (int32_t h = 0; h < n_q_heads; ++h) {
        const int32_t g = h / group;
        const double *qi = q + (i * n_q_heads + h) * d;
        double *oi = out + (i * n_q_heads + h) * d;
        /* scores of the visible keys and their maximum */
        double m = -INFINITY;
        int64_t n_vis = 0;
        for (int64_t j = k0; j < k1; ++j) {
          if (kv_pos[j] > q_pos[i]) continue;
          const double *kj = k + (j * n_kv_heads + g) * d;
          double dot = 0.0;
          for (int32_t c = 0; c < d; ++c) dot += qi[c] * kj[c];
          s[j - k0] = dot * scale;
          if (s[j - k0] > m) m = s[j - k0];
          ++n_vis;
        }
        if (h == 0) pairs += n_vis;
        for (int32_t c = 0; c < d; ++c) oi[c] = 0.0;
        if (n_vis == 0) {
          lse[i * n_q_heads + h] = -INFINITY;
          continue;
        }
        /* denominator, then the weighted sum of values */
        double l = 0.0;
        for (int64_t j = k0; j < k1; ++j) {
          if (kv_pos[j] > q_pos[i]) continue;
          l += exp(s[j - k0] - m);
        }
        for (int64_t j = k0; j < k1; ++j) {
          if (kv_pos[j] > q_pos[i]) continue;
          const double w = exp(s[j - k0] - m) / l;
          const double *vj = v + (j * n_kv_heads + g) * d;
          for (int32_t c = 0; c < d; ++c) oi[c] += w * vj[c];
        }
        lse[i * n_q_heads + h] = m + log(l);
      }
      free(s);
    }
  }
  return pairs;
}

/*
 * Equation 4. outs[s] is [rows, d], lses[s] is [rows]; "rows" counts
 * (token, head) pairs. out [rows, d]; lse_out [rows] may be NULL.
 */
void oracle_merge(const double *const *outs, const double *const *lses,
                  int32_t n_parts, int64_t rows, int32_t d, double *out,
                  double *lse_out) {
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < rows; ++r) {
    double lmax = -INFINITY;
    for (int32_t s = 0; s < n_parts; ++s)
      if (lses[s][r] > lmax) lmax = lses[s][r];
    double *o = out + r * d;
    for (int32_t c = 0; c < d; ++c) o[c] = 0.0;
    if (lmax == -INFINITY) {
      if (lse_out) lse_out[r] = -INFINITY;
      continue;
    }
    double den = 0.0;
    for (int32_t s = 0; s < n_parts; ++s) den += exp(lses[s][r] - lmax);
    for (int32_t s = 0; s < n_parts; ++s) {
      const double w = exp(lses[s][r] - lmax);
      if (w == 0.0) continue; /* a partial with LSE = -inf carries no keys */
      const double *os = outs[s] + r * d;
      for (int32_t c = 0; c < d; ++c) o[c] += os[c] * w;
    }
    for (int32_t c = 0; c < d; ++c) o[c] /= den;
    if (lse_out) lse_out[r] = lmax + log(den);
  }
}
