/* fp64 CPU oracle for prefix-shared GRPO prefill attention, plain C.
 * TEST INFRASTRUCTURE ONLY: used by tests, the smoke check and the benchmark's
 * cpu_baseline leg.  The product path never links or calls it, and it shares no
 * code with the HIP kernels.
 *
 * Definition followed (paper Sec. 5.1: video embeddings are gathered once and
 * reused by all rollouts; Sec. 5.2: each rollout is prefilled over the whole
 * sequence; Sec. 4.2: G responses per question): for rollout g, q-head h
 * (kv head c = h / (Hq/Hkv)), suffix row i, the visible keys are the P prefix
 * tokens and the rollout's own suffix tokens 0..i.
 *     s_j = scale * <q, k_j>,  m = max s_j,  Z = sum exp(s_j - m),
 *     LSE = m + ln Z,          O = sum (exp(s_j - m) / Z) v_j.
 * Two-pass softmax in double, one query row at a time, no tiling, no online
 * rescaling, no merging of partial results.
 *
 * Inputs are float arrays whose values both sides consume unchanged (bf16-rounded
 * or fp32 values, widened exactly to double here).
 *
 * Pinned in tests/test_oracle_pins.py against the numpy definition, a loop-only
 * brute-force full-sequence attention, torch's SDPA and closed forms.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double dot_fd(const float* a, const float* b, int D) {
  double acc = 0.0;
#pragma omp simd reduction(+ : acc)
  for (int d = 0; d < D; ++d) acc += (double)a[d] * (double)b[d];
  return acc;
}

/* rows == NULL: every packed token row 0..T-1 is computed (n_rows must be T).
 * out [n_rows, Hq, D] double; lse [Hq, n_rows] double.
 * Returns the number of threads used, or a negative value on a bad argument. */
int ref_prefix_shared_attention(const float* q, const float* k_prefix, const float* v_prefix,
                                const float* k_suffix, const float* v_suffix,
                                const int32_t* suffix_lens, int G, int64_t P, int Hq, int Hkv, int D,
                                double scale, const int64_t* rows, int64_t n_rows, double* out,
                                double* lse, int num_threads) {
  if (!q || !k_suffix || !v_suffix || !suffix_lens || !out || !lse) return -1;
  if (P > 0 && (!k_prefix || !v_prefix)) return -1;
  if (G < 1 || Hq < 1 || Hkv < 1 || Hq % Hkv != 0 || D < 1 || P < 0) return -2;
  int64_t* off = (int64_t*)malloc(sizeof(int64_t) * (size_t)(G + 1));
  if (!off) return -3;
  off[0] = 0;
  for (int g = 0; g < G; ++g) {
    if (suffix_lens[g] < 1) { free(off); return -2; }
    off[g + 1] = off[g] + suffix_lens[g];
  }
  const int64_t T = off[G];
  if (!rows && n_rows != T) { free(off); return -2; }
  const int r = Hq / Hkv;
  int used = 1;
#ifdef _OPENMP
  if (num_threads > 0) omp_set_num_threads(num_threads);
  used = omp_get_max_threads();
#endif
  int bad = 0;
#pragma omp parallel
  {
    double* s = (double*)malloc(sizeof(double) * (size_t)(P + T));
    if (!s) {
#pragma omp atomic write
      bad = 1;
    }
#pragma omp for schedule(dynamic, 1) collapse(2)
    for (int64_t n = 0; n < n_rows; ++n) {
      for (int h = 0; h < Hq; ++h) {
        if (!s) continue;
        const int64_t t = rows ? rows[n] : n;
        if (t < 0 || t >= T) {
#pragma omp atomic write
          bad = 1;
          continue;
        }
        int g = 0;
        while (off[g + 1] <= t) ++g;
        const int64_t i = t - off[g];
        const int c = h / r;
        const float* qv = q + ((size_t)t * Hq + h) * D;
        /* pass 1: scores over the visible keys and their maximum */
        double m = -INFINITY;
        for (int64_t j = 0; j < P; ++j) {
          const double x = scale * dot_fd(qv, k_prefix + ((size_t)j * Hkv + c) * D, D);
          s[j] = x;
          if (x > m) m = x;
        }
        for (int64_t j = 0; j <= i; ++j) {
          const double x = scale * dot_fd(qv, k_suffix + ((size_t)(off[g] + j) * Hkv + c) * D, D);
          s[P + j] = x;
          if (x > m) m = x;
        }
        /* pass 2: normaliser */
        const int64_t nk = P + i + 1;
        double Z = 0.0;
        for (int64_t j = 0; j < nk; ++j) {
          s[j] = exp(s[j] - m);
          Z += s[j];
        }
        double* o = out + ((size_t)n * Hq + h) * D;
        for (int d = 0; d < D; ++d) o[d] = 0.0;
        for (int64_t j = 0; j < nk; ++j) {
          const double w = s[j] / Z;
          const float* vv = (j < P) ? v_prefix + ((size_t)j * Hkv + c) * D
                                    : v_suffix + ((size_t)(off[g] + j - P) * Hkv + c) * D;
          for (int d = 0; d < D; ++d) o[d] += w * (double)vv[d];
        }
        lse[(size_t)h * n_rows + n] = m + log(Z);
      }
    }
    free(s);
  }
  free(off);
  return bad ? -4 : used;
}

/* ---------------------------------------------------------------------------------------------
 * Backward: gradients of L = sum(d_out * out) with respect to q, k, v (the policy model is
 * trained through the attention, paper Eq. 1 / Sec. 5.2).  Chain rule on the definition above,
 * with W = softmax weights of a row:
 *     dV_j = sum_rows W_j dO,   dW_j = <dO, v_j>,   delta = sum_j W_j dW_j,
 *     dS_j = W_j (dW_j - delta),   dQ = scale sum_j dS_j k_j,   dK_j = scale sum_rows dS_j q.
 * A kv head sums over the q heads of its group; a prefix key/value also sums over all
 * rollouts, since every rollout attends to the same cached prefix (Sec. 5.1).
 *
 * Phase 1 visits every query row (two-pass softmax as above), writes dQ and keeps the row's
 * LSE and delta.  Phase 2 visits every key and sums over the rows that see it, with
 * W_j = exp(s_j - LSE).  rows != NULL: only dQ of those packed token rows is produced
 * (dq [n_rows,Hq,D]) and phase 2 is skipped (the four key/value gradients may be NULL).
 * Returns the number of threads used, or a negative value on a bad argument.
 */
int ref_prefix_shared_attention_backward(const float* q, const float* k_prefix, const float* v_prefix,
                                         const float* k_suffix, const float* v_suffix, const float* d_out,
                                         const int32_t* suffix_lens, int G, int64_t P, int Hq, int Hkv,
                                         int D, double scale, const int64_t* rows, int64_t n_rows,
                                         double* dq, double* dk_prefix, double* dv_prefix,
                                         double* dk_suffix, double* dv_suffix, int num_threads) {
  if (!q || !k_suffix || !v_suffix || !d_out || !suffix_lens || !dq) return -1;
  if (P > 0 && (!k_prefix || !v_prefix)) return -1;
  if (!rows && (!dk_suffix || !dv_suffix || (P > 0 && (!dk_prefix || !dv_prefix)))) return -1;
  if (G < 1 || Hq < 1 || Hkv < 1 || Hq % Hkv != 0 || D < 1 || P < 0) return -2;
  int64_t* off = (int64_t*)malloc(sizeof(int64_t) * (size_t)(G + 1));
  if (!off) return -3;
  off[0] = 0;
  for (int g = 0; g < G; ++g) {
    if (suffix_lens[g] < 1) { free(off); return -2; }
    off[g + 1] = off[g] + suffix_lens[g];
  }
  const int64_t T = off[G];
  if (!rows && n_rows != T) { free(off); return -2; }
  const int r = Hq / Hkv;
  int used = 1;
#ifdef _OPENMP
  if (num_threads > 0) omp_set_num_threads(num_threads);
  used = omp_get_max_threads();
#endif
  double* lse = NULL;
  double* delta = NULL;
  if (!rows) {
    lse = (double*)malloc(sizeof(double) * (size_t)T * Hq);
    delta = (double*)malloc(sizeof(double) * (size_t)T * Hq);
    if (!lse || !delta) { free(lse); free(delta); free(off); return -3; }
  }
  int bad = 0;
#pragma omp parallel
  {
    double* s = (double*)malloc(sizeof(double) * (size_t)(P + T));
    double* dw = (double*)malloc(sizeof(double) * (size_t)(P + T));
    if (!s || !dw) {
#pragma omp atomic write
      bad = 1;
    }
#pragma omp for schedule(dynamic, 1) collapse(2)
    for (int64_t n = 0; n < n_rows; ++n) {
      for (int h = 0; h < Hq; ++h) {
        if (!s || !dw) continue;
        const int64_t t = rows ? rows[n] : n;
        if (t < 0 || t >= T) {
#pragma omp atomic write
          bad = 1;
          continue;
        }
        int g = 0;
        while (off[g + 1] <= t) ++g;
        const int64_t i = t - off[g];
        const int c = h / r;
        const float* qv = q + ((size_t)t * Hq + h) * D;
        const float* dov = d_out + ((size_t)t * Hq + h) * D;
        const int64_t nk = P + i + 1;
        double m = -INFINITY;
        for (int64_t j = 0; j < nk; ++j) {
          const float* kv = (j < P) ? k_prefix + ((size_t)j * Hkv + c) * D
                                    : k_suffix + ((size_t)(off[g] + j - P) * Hkv + c) * D;
          const float* vv = (j < P) ? v_prefix + ((size_t)j * Hkv + c) * D
                                    : v_suffix + ((size_t)(off[g] + j - P) * Hkv + c) * D;
          s[j] = scale * dot_fd(qv, kv, D);
          dw[j] = dot_fd(dov, vv, D);
          if (s[j] > m) m = s[j];
        }
        double Z = 0.0;
        for (int64_t j = 0; j < nk; ++j) {
          s[j] = exp(s[j] - m);
          Z += s[j];
        }
        double dl = 0.0;
        for (int64_t j = 0; j < nk; ++j) {
          s[j] /= Z;               /* W_j */
          dl += s[j] * dw[j];
        }
        double* o = dq + ((size_t)n * Hq + h) * D;
        for (int d = 0; d < D; ++d) o[d] = 0.0;
        for (int64_t j = 0; j < nk; ++j) {
          const double ds = s[j] * (dw[j] - dl);
          const float* kv = (j < P) ? k_prefix + ((size_t)j * Hkv + c) * D
                                    : k_suffix + ((size_t)(off[g] + j - P) * Hkv + c) * D;
          for (int d = 0; d < D; ++d) o[d] += scale * ds * (double)kv[d];
        }
        if (!rows) {
          lse[(size_t)t * Hq + h] = m + log(Z);
          delta[(size_t)t * Hq + h] = dl;
        }
      }
    }
    free(s);
    free(dw);

    if (!rows && !bad) {
      /* phase 2: one key (jj < P: prefix token jj, else packed suffix token jj - P) and kv head at a time */
#pragma omp for schedule(dynamic, 1) collapse(2)
      for (int64_t jj = 0; jj < P + T; ++jj) {
        for (int c = 0; c < Hkv; ++c) {
          const int is_prefix = jj < P;
          const int64_t tj = jj - P;  /* packed row of a suffix key */
          const float* kv = is_prefix ? k_prefix + ((size_t)jj * Hkv + c) * D : k_suffix + ((size_t)tj * Hkv + c) * D;
          const float* vv = is_prefix ? v_prefix + ((size_t)jj * Hkv + c) * D : v_suffix + ((size_t)tj * Hkv + c) * D;
          double* dk = is_prefix ? dk_prefix + ((size_t)jj * Hkv + c) * D : dk_suffix + ((size_t)tj * Hkv + c) * D;
          double* dv = is_prefix ? dv_prefix + ((size_t)jj * Hkv + c) * D : dv_suffix + ((size_t)tj * Hkv + c) * D;
          for (int d = 0; d < D; ++d) { dk[d] = 0.0; dv[d] = 0.0; }
          /* rows that see this key: every packed row for a prefix key; for a suffix key the rows of
           * its own rollout from the key's position on */
          int64_t t0 = 0, t1 = T;
          if (!is_prefix) {
            int g = 0;
            while (off[g + 1] <= tj) ++g;
            t0 = tj;
            t1 = off[g + 1];
          }
          for (int64_t t = t0; t < t1; ++t) {
            for (int h = c * r; h < (c + 1) * r; ++h) {
              const float* qv = q + ((size_t)t * Hq + h) * D;
              const float* dov = d_out + ((size_t)t * Hq + h) * D;
              const double w = exp(scale * dot_fd(qv, kv, D) - lse[(size_t)t * Hq + h]);
              const double ds = w * (dot_fd(dov, vv, D) - delta[(size_t)t * Hq + h]);
              for (int d = 0; d < D; ++d) {
                dk[d] += scale * ds * (double)qv[d];
                dv[d] += w * (double)dov[d];
              }
            }
          }
        }
      }
    }
  }
  free(lse);
  free(delta);
  free(off);
  return bad ? -4 : used;
}
