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
 * One query row (token, q head) at a time, exactly as the formulas read: its scores and weights
 * (two-pass softmax as above), dW, delta and dS over its visible keys; dQ of the row is written,
 * and the row's terms W_j dO and scale dS_j q are added to dV_j and dK_j of every key it sees.
 * Nothing is saved between rows and nothing is recomputed per key.  (Threads work on different
 * rows and add into accumulators of their own, which are summed at the end.)
 * rows != NULL: only dQ of those packed token rows is produced (dq [n_rows,Hq,D]); the four
 * key/value gradients are not touched and may be NULL.
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
  /* per thread: dK and dV of every key ([P + T][Hkv][D] each; prefix keys first, then the packed suffix keys) */
  const size_t n_kv = (size_t)(P + T) * Hkv * D;
  double* acc = NULL;
  if (!rows) {
    acc = (double*)calloc((size_t)used * 2 * n_kv, sizeof(double));
    if (!acc) { free(off); return -3; }
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
        if (!rows) { /* this row's share of dK and dV of the keys it sees */
          int tid = 0;
#ifdef _OPENMP
          tid = omp_get_thread_num();
#endif
          double* acc_k = acc + (size_t)tid * 2 * n_kv;
          double* acc_v = acc_k + n_kv;
          for (int64_t j = 0; j < nk; ++j) {
            const double ds = s[j] * (dw[j] - dl);
            const size_t key = (j < P) ? (size_t)j : (size_t)(P + off[g] + (j - P));
            double* dk = acc_k + (key * Hkv + c) * D;
            double* dv = acc_v + (key * Hkv + c) * D;
            for (int d = 0; d < D; ++d) {
              dk[d] += scale * ds * (double)qv[d];
              dv[d] += s[j] * (double)dov[d];
            }
          }
        }
      }
    }
    free(s);
    free(dw);

    if (!rows && !bad) { /* sum the threads' accumulators in thread order */
#pragma omp for schedule(static)
      for (int64_t e = 0; e < (int64_t)n_kv; ++e) {
        double sk = 0.0, sv = 0.0;
        for (int th = 0; th < used; ++th) {
          sk += acc[(size_t)th * 2 * n_kv + (size_t)e];
          sv += acc[(size_t)th * 2 * n_kv + n_kv + (size_t)e];
        }
        const size_t n_pre = (size_t)P * Hkv * D;
        if ((size_t)e < n_pre) {
          dk_prefix[e] = sk;
          dv_prefix[e] = sv;
        } else {
          dk_suffix[(size_t)e - n_pre] = sk;
          dv_suffix[(size_t)e - n_pre] = sv;
        }
      }
    }
  }
  free(acc);
  free(off);
  return bad ? -4 : used;
}
