/*
 * CPU oracle for causal linear attention with per-head exponential decay
 * (Lightning Attention-2).  TEST INFRASTRUCTURE ONLY: tests, the smoke check and
 * the benchmark's cpu_baseline leg call this; the GPU library never does and
 * shares no code with it.
 *
 * Everything is fp64, plain loops, no blocking, no fusion.  Tensors are dense
 * row-major [batch, heads, n, d]; lambda is [heads]; states are [batch, heads, d, d]
 * with the key feature as the row index and the value feature as the column index.
 *
 * Two independent forms are provided:
 *   *_direct     the definition: o_t = q_t * sum_{s<=t} lambda^(t-s) k_s^T v_s
 *                (Sec. 3.2.1, first equation of "Forward Pass") and the gradients
 *                that follow from it (Sec. 3.2.2, first equation of "Backward Pass",
 *                with kv_t and dkv_t written out as their sums), O(n^2 d) per head;
 *   *_recurrent  the token-by-token recursion kv_t = lambda kv_{t-1} + k_t^T v_t,
 *                o_t = q_t kv_t (Sec. 3.2.1, recursive form) and the reverse recursion
 *                dkv_{t-1} = lambda dkv_t + q_{t-1}^T do_{t-1} (Sec. 3.2.2), O(n d^2).
 * The recurrent form also runs SEGMENTS of a sequence (start state in, final state out, and the
 * matching gradients); the tests pin those against the direct form of the whole sequence.
 * The tests pin each against closed forms, finite differences and each other.
 *
 * The weight of the diagonal term (s == t) is exactly 1 for every lambda in (0, 1].
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int la2_oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* table pw[m] = lambda^m, m = 0..n-1, by the library pow (pw[0] is exactly 1) */
static double *power_table(double lambda, int64_t n) {
  double *pw = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
  for (int64_t m = 0; m < n; m++) pw[m] = (m == 0) ? 1.0 : pow(lambda, (double)m);
  return pw;
}

static double dot(const double *a, const double *b, int d) {
  double s = 0.0;
  for (int i = 0; i < d; i++) s += a[i] * b[i];
  return s;
}

/* ---- one head, selected rows, direct form --------------------------------------------- */

/* o_t = sum_{s<=t} lambda^(t-s) (q_t . k_s) v_s   for t in rows[] */
void la2_oracle_fwd_rows(int64_t n, int d, const double *q, const double *k, const double *v,
                         double lambda, int64_t nrows, const int64_t *rows, double *o_rows) {
  double *pw = power_table(lambda, n);
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t i = 0; i < nrows; i++) {
    int64_t t = rows[i];
    double *o = o_rows + i * d;
    for (int j = 0; j < d; j++) o[j] = 0.0;
    for (int64_t s = 0; s <= t; s++) {
      double w = pw[t - s] * dot(q + t * d, k + s * d, d);
      for (int j = 0; j < d; j++) o[j] += w * v[s * d + j];
    }
  }
  free(pw);
}

/*
 * dq_t = sum_{s<=t} lambda^(t-s) (do_t . v_s) k_s
 * dk_s = sum_{t>=s} lambda^(t-s) (do_t . v_s) q_t
 * dv_s = sum_{t>=s} lambda^(t-s) (q_t . k_s) do_t        for the positions in rows[]
 */
void la2_oracle_bwd_rows(int64_t n, int d, const double *q, const double *k, const double *v,
                         const double *d_o, double lambda, int64_t nrows, const int64_t *rows,
                         double *dq_rows, double *dk_rows, double *dv_rows) {
  double *pw = power_table(lambda, n);
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t i = 0; i < nrows; i++) {
    int64_t p = rows[i];
    double *dq = dq_rows + i * d, *dk = dk_rows + i * d, *dv = dv_rows + i * d;
    for (int j = 0; j < d; j++) dq[j] = dk[j] = dv[j] = 0.0;
    for (int64_t s = 0; s <= p; s++) {
      double w = pw[p - s] * dot(d_o + p * d, v + s * d, d);
      for (int j = 0; j < d; j++) dq[j] += w * k[s * d + j];
    }
    for (int64_t t = p; t < n; t++) {
      double wk = pw[t - p] * dot(d_o + t * d, v + p * d, d);
      double wv = pw[t - p] * dot(q + t * d, k + p * d, d);
      for (int j = 0; j < d; j++) {
        dk[j] += wk * q[t * d + j];
        dv[j] += wv * d_o[t * d + j];
      }
    }
  }
  free(pw);
}

/* ---- whole tensors, direct form ---------------------------------------------------------- */

void la2_oracle_fwd_direct(int b, int H, int64_t n, int d, const double *q, const double *k,
                           const double *v, const double *lambda, double *o) {
  for (int64_t c = 0; c < (int64_t)b * H; c++) {
    int64_t off = c * n * d;
    double *pw = power_table(lambda[c % H], n);
#pragma omp parallel for schedule(dynamic, 8)
    for (int64_t t = 0; t < n; t++) {
      double *ot = o + off + t * d;
      for (int j = 0; j < d; j++) ot[j] = 0.0;
      for (int64_t s = 0; s <= t; s++) {
        double w = pw[t - s] * dot(q + off + t * d, k + off + s * d, d);
        for (int j = 0; j < d; j++) ot[j] += w * v[off + s * d + j];
      }
    }
    free(pw);
  }
}

void la2_oracle_bwd_direct(int b, int H, int64_t n, int d, const double *q, const double *k,
                           const double *v, const double *d_o, const double *lambda, double *dq,
                           double *dk, double *dv) {
  for (int64_t c = 0; c < (int64_t)b * H; c++) {
    int64_t off = c * n * d;
    double *pw = power_table(lambda[c % H], n);
#pragma omp parallel for schedule(dynamic, 8)
    for (int64_t p = 0; p < n; p++) {
      double *dqp = dq + off + p * d, *dkp = dk + off + p * d, *dvp = dv + off + p * d;
      for (int j = 0; j < d; j++) dqp[j] = dkp[j] = dvp[j] = 0.0;
      for (int64_t s = 0; s <= p; s++) {
        double w = pw[p - s] * dot(d_o + off + p * d, v + off + s * d, d);
        for (int j = 0; j < d; j++) dqp[j] += w * k[off + s * d + j];
      }
      for (int64_t t = p; t < n; t++) {
        double wk = pw[t - p] * dot(d_o + off + t * d, v + off + p * d, d);
        double wv = pw[t - p] * dot(q + off + t * d, k + off + p * d, d);
        for (int j = 0; j < d; j++) {
          dkp[j] += wk * q[off + t * d + j];
          dvp[j] += wv * d_o[off + t * d + j];
        }
      }
    }
    free(pw);
  }
}

/* ---- whole tensors, recurrent form (independent of the direct form) ------------------------ */

/* kv_0 = kv_init (or 0); kv_t = lambda kv_{t-1} + k_t^T v_t; o_t = q_t kv_t.
 * kv_init / kv_final may be NULL; both are [b, H, d, d]. */
void la2_oracle_fwd_recurrent(int b, int H, int64_t n, int d, const double *q, const double *k,
                              const double *v, const double *lambda, const double *kv_init,
                              double *o, double *kv_final) {
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t c = 0; c < (int64_t)b * H; c++) {
    int64_t off = c * n * d;
    double lam = lambda[c % H];
    double *kv = (double *)calloc((size_t)d * d, sizeof(double));
    if (kv_init) memcpy(kv, kv_init + c * d * d, sizeof(double) * (size_t)d * d);
    for (int64_t t = 0; t < n; t++) {
      const double *qt = q + off + t * d, *kt = k + off + t * d, *vt = v + off + t * d;
      for (int i = 0; i < d; i++)
        for (int j = 0; j < d; j++) kv[i * d + j] = lam * kv[i * d + j] + kt[i] * vt[j];
      for (int j = 0; j < d; j++) {
        double s = 0.0;
        for (int i = 0; i < d; i++) s += qt[i] * kv[i * d + j];
        o[off + t * d + j] = s;
      }
    }
    if (kv_final) memcpy(kv_final + c * d * d, kv, sizeof(double) * (size_t)d * d);
    free(kv);
  }
}

/* forward sweep: dq_t = do_t kv_t^T;  reverse sweep: dkv_t = lambda dkv_{t+1} + q_t^T do_t,
 * dk_t = v_t dkv_t^T, dv_t = k_t dkv_t. */
void la2_oracle_bwd_recurrent(int b, int H, int64_t n, int d, const double *q, const double *k,
                              const double *v, const double *d_o, const double *lambda,
                              double *dq, double *dk, double *dv) {
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t c = 0; c < (int64_t)b * H; c++) {
    int64_t off = c * n * d;
    double lam = lambda[c % H];
    double *kv = (double *)calloc((size_t)d * d, sizeof(double));
    double *dkv = (double *)calloc((size_t)d * d, sizeof(double));
    for (int64_t t = 0; t < n; t++) {
      const double *kt = k + off + t * d, *vt = v + off + t * d, *dot_ = d_o + off + t * d;
      for (int i = 0; i < d; i++)
        for (int j = 0; j < d; j++) kv[i * d + j] = lam * kv[i * d + j] + kt[i] * vt[j];
      for (int i = 0; i < d; i++) {
        double s = 0.0;
        for (int j = 0; j < d; j++) s += dot_[j] * kv[i * d + j];
        dq[off + t * d + i] = s;
      }
    }
    for (int64_t t = n - 1; t >= 0; t--) {
      const double *qt = q + off + t * d, *kt = k + off + t * d, *vt = v + off + t * d,
                   *dot_ = d_o + off + t * d;
      for (int i = 0; i < d; i++)
        for (int j = 0; j < d; j++) dkv[i * d + j] = lam * dkv[i * d + j] + qt[i] * dot_[j];
      for (int i = 0; i < d; i++) {
        double s = 0.0;
        for (int j = 0; j < d; j++) s += vt[j] * dkv[i * d + j];
        dk[off + t * d + i] = s;
      }
      for (int j = 0; j < d; j++) {
        double s = 0.0;
        for (int i = 0; i < d; i++) s += kt[i] * dkv[i * d + j];
        dv[off + t * d + j] = s;
      }
    }
    free(kv);
    free(dkv);
  }
}

/* The same two sweeps for a segment of a longer sequence (Sec. 3.2.1 recursion started from a
 * non-zero kv_0 = kv_init; chain rule through the recursion when the loss also depends on the
 * segment's final state kv_n, whose gradient d_kv_final is handed in):
 *   forward sweep   kv_t = lambda kv_{t-1} + k_t^T v_t (kv_0 = kv_init),   dq_t = do_t kv_t^T
 *   reverse sweep   g_n = q_n^T do_n + d_kv_final,  g_t = lambda g_{t+1} + q_t^T do_t   (total gradient
 *                   with respect to kv_t),  dk_t = v_t g_t^T,  dv_t = k_t g_t
 *   d_kv_init = lambda g_1   (kv_0 enters kv_1 with the factor lambda)
 * kv_init, d_kv_final may be NULL (zero); d_kv_init may be NULL (not wanted).  n == 0: d_kv_init = d_kv_final. */
void la2_oracle_bwd_recurrent_state(int b, int H, int64_t n, int d, const double *q, const double *k,
                                    const double *v, const double *d_o, const double *lambda,
                                    const double *kv_init, const double *d_kv_final, double *dq,
                                    double *dk, double *dv, double *d_kv_init) {
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t c = 0; c < (int64_t)b * H; c++) {
    int64_t off = c * n * d;
    double lam = lambda[c % H];
    double *kv = (double *)calloc((size_t)d * d, sizeof(double));
    double *g = (double *)calloc((size_t)d * d, sizeof(double));
    if (kv_init) memcpy(kv, kv_init + c * d * d, sizeof(double) * (size_t)d * d);
    for (int64_t t = 0; t < n; t++) {
      const double *kt = k + off + t * d, *vt = v + off + t * d, *dot_ = d_o + off + t * d;
      for (int i = 0; i < d; i++)
        for (int j = 0; j < d; j++) kv[i * d + j] = lam * kv[i * d + j] + kt[i] * vt[j];
      for (int i = 0; i < d; i++) {
        double s = 0.0;
        for (int j = 0; j < d; j++) s += dot_[j] * kv[i * d + j];
        dq[off + t * d + i] = s;
      }
    }
    for (int64_t t = n - 1; t >= 0; t--) {
      const double *qt = q + off + t * d, *kt = k + off + t * d, *vt = v + off + t * d,
                   *dot_ = d_o + off + t * d;
      for (int i = 0; i < d; i++)
        for (int j = 0; j < d; j++) {
          double carried = (t == n - 1) ? (d_kv_final ? d_kv_final[c * d * d + i * d + j] : 0.0)
                                        : lam * g[i * d + j];
          g[i * d + j] = carried + qt[i] * dot_[j];
        }
      for (int i = 0; i < d; i++) {
        double s = 0.0;
        for (int j = 0; j < d; j++) s += vt[j] * g[i * d + j];
        dk[off + t * d + i] = s;
      }
      for (int j = 0; j < d; j++) {
        double s = 0.0;
        for (int i = 0; i < d; i++) s += kt[i] * g[i * d + j];
        dv[off + t * d + j] = s;
      }
    }
    if (d_kv_init) {
      for (int i = 0; i < d * d; i++)
        d_kv_init[c * d * d + i] = (n > 0) ? lam * g[i] : (d_kv_final ? d_kv_final[c * d * d + i] : 0.0);
    }
    free(kv);
    free(g);
  }
}

/* ---- decode step: kv <- lambda_h kv + k^T v (in place), then o = q kv ------------------------ */
void la2_oracle_decode_step(int b, int H, int d, const double *q, const double *k, const double *v,
                            const double *lambda, double *kv, double *o) {
#pragma omp parallel for schedule(static)
  for (int64_t c = 0; c < (int64_t)b * H; c++) {
    double lam = lambda[c % H];
    double *s = kv + c * d * d;
    const double *qc = q + c * d, *kc = k + c * d, *vc = v + c * d;
    for (int i = 0; i < d; i++)
      for (int j = 0; j < d; j++) s[i * d + j] = lam * s[i * d + j] + kc[i] * vc[j];
    for (int j = 0; j < d; j++) {
      double acc = 0.0;
      for (int i = 0; i < d; i++) acc += qc[i] * s[i * d + j];
      o[c * d + j] = acc;
    }
  }
}
