/*
 * CPU fp64 oracle for document-masked causal attention on a packed microbatch,
 * forward and backward.  TEST INFRASTRUCTURE ONLY: nothing in the product path may
 * call this; it shares no code with the HIP kernels.
 *
 * What is computed (Section 5.2, "Micro-Batch Time Prediction": documents of lengths
 * l_1..l_k with sum N are concatenated and a block-diagonal mask keeps attention inside
 * each document; the models are decoder-only, hence causal inside the block):
 *
 *   token t lives in document b  (cu[b] <= t < cu[b+1]);  q-head h reads kv-head
 *   kappa = h / (Hq/Hkv);  allowed keys J(t) = { j : cu[b] <= j <= t }.
 *
 *   S_tj   = scale * sum_c Q[t,h,c] K[j,kappa,c]
 *   LSE_th = m + ln sum_{j in J} exp(S_tj - m),   m = max_{j in J} S_tj
 *   P_tj   = exp(S_tj - LSE_th)
 *   O[t,h] = sum_{j in J} P_tj V[j,kappa]
 *   D_th   = sum_c dO[t,h,c] O[t,h,c]
 *   dP_tj  = sum_c dO[t,h,c] V[j,kappa,c]
 *   dS_tj  = P_tj (dP_tj - D_th)
 *   dQ[t,h]     = scale * sum_{j in J(t)} dS_tj K[j,kappa]
 *   dK[j,kappa] = scale * sum_{h in group(kappa)} sum_{t : j in J(t)} dS_tj Q[t,h]
 *   dV[j,kappa] =         sum_{h in group(kappa)} sum_{t : j in J(t)} P_tj  dO[t,h]
 *
 * i.e. the gradients of L = sum O * dO.  Every output element is evaluated from its
 * own formula (row-wise for O, LSE, dQ; column-wise for dK, dV): no tiling, no online
 * softmax, no fusion.  Layouts: Q, O, dO, dQ are [N, Hq, d]; K, V, dK, dV are
 * [N, Hkv, d]; LSE and D are [Hq, N]; all double, row-major.
 *
 * Row-subset entry points evaluate the same formulas for a list of token indices only,
 * so that single outputs of a very large problem can be checked one by one.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
  int32_t N, B, Hq, Hkv, d;
  double scale;
  const double *q, *k, *v;
  const int32_t *cu;
} vao_problem;

static int doc_of_token(const int32_t *cu, int B, int t) {
  /* the unique b with cu[b] <= t < cu[b+1] (empty documents never match) */
  for (int b = 0; b < B; ++b)
    if (cu[b] <= t && t < cu[b + 1]) return b;
  return -1;
}

static double dot(const double *a, const double *b, int d) {
  double s = 0.0;
#pragma omp simd reduction(+ : s)
  for (int c = 0; c < d; ++c) s += a[c] * b[c];
  return s;
}

int vao_set_threads(int n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
  return omp_get_max_threads();
#else
  (void)n;
  return 1;
#endif
}

int vao_validate_cu(const int32_t *cu, int B, int N) {
  if (B < 1 || cu[0] != 0 || cu[B] != N) return 0;
  for (int b = 0; b < B; ++b)
    if (cu[b + 1] < cu[b]) return 0;
  return 1;
}

/* scores of one (t, h) row over its allowed keys; returns LSE; p[0..n) = P_tj */
static double softmax_row(const vao_problem *P, int t, int h, int start, double *p) {
  const int g = P->Hq / P->Hkv, kap = h / g, d = P->d;
  const double *qt = P->q + ((size_t)t * P->Hq + h) * d;
  const int n = t - start + 1;
  double m = -INFINITY;
  for (int i = 0; i < n; ++i) {
    const double *kj = P->k + ((size_t)(start + i) * P->Hkv + kap) * d;
    p[i] = P->scale * dot(qt, kj, d);
    if (p[i] > m) m = p[i];
  }
  double l = 0.0;
  for (int i = 0; i < n; ++i) l += exp(p[i] - m);
  const double lse = m + log(l);
  for (int i = 0; i < n; ++i) p[i] = exp(p[i] - lse);
  return lse;
}

/*
 * Forward for a list of tokens (rows == NULL: all tokens 0..N-1, n_rows = N).
 * o_out:   [n_rows, Hq, d]      lse_out: [Hq, n_rows]
 */
int vao_fwd_rows(int32_t N, int32_t B, int32_t Hq, int32_t Hkv, int32_t d, double scale,
                 const double *q, const double *k, const double *v, const int32_t *cu,
                 const int32_t *rows, int32_t n_rows, double *o_out, double *lse_out) {
  if (!vao_validate_cu(cu, B, N) || Hq % Hkv) return -1;
  vao_problem P = {N, B, Hq, Hkv, d, scale, q, k, v, cu};
  const int g = Hq / Hkv;
  int err = 0;
#pragma omp parallel
  {
    double *p = (double *)malloc(sizeof(double) * (size_t)(N > 0 ? N : 1));
#pragma omp for collapse(2) schedule(dynamic, 4)
    for (int r = 0; r < n_rows; ++r)
      for (int h = 0; h < Hq; ++h) {
        const int t = rows ? rows[r] : r;
        const int b = doc_of_token(cu, B, t);
        if (b < 0) { err = 1; continue; }
        const int start = cu[b], n = t - start + 1, kap = h / g;
        const double lse = softmax_row(&P, t, h, start, p);
        double *o = o_out + ((size_t)r * Hq + h) * d;
        for (int c = 0; c < d; ++c) o[c] = 0.0;
        for (int i = 0; i < n; ++i) {
          const double *vj = v + ((size_t)(start + i) * Hkv + kap) * d;
          const double pij = p[i];
          for (int c = 0; c < d; ++c) o[c] += pij * vj[c];
        }
        lse_out[(size_t)h * n_rows + r] = lse;
      }
    free(p);
  }
  return err ? -2 : 0;
}

/*
 * dQ (and D) for a list of tokens.  dq_out: [n_rows, Hq, d];  d_out: [Hq, n_rows] (may be NULL)
 */
int vao_dq_rows(int32_t N, int32_t B, int32_t Hq, int32_t Hkv, int32_t d, double scale,
                const double *q, const double *k, const double *v, const double *d_o,
                const int32_t *cu, const int32_t *rows, int32_t n_rows, double *dq_out,
                double *d_out) {
  if (!vao_validate_cu(cu, B, N) || Hq % Hkv) return -1;
  vao_problem P = {N, B, Hq, Hkv, d, scale, q, k, v, cu};
  const int g = Hq / Hkv;
  int err = 0;
#pragma omp parallel
  {
    double *p = (double *)malloc(sizeof(double) * (size_t)(N > 0 ? N : 1));
    double *o = (double *)malloc(sizeof(double) * (size_t)d);
#pragma omp for collapse(2) schedule(dynamic, 4)
    for (int r = 0; r < n_rows; ++r)
      for (int h = 0; h < Hq; ++h) {
        const int t = rows ? rows[r] : r;
        const int b = doc_of_token(cu, B, t);
        if (b < 0) { err = 1; continue; }
        const int start = cu[b], n = t - start + 1, kap = h / g;
        softmax_row(&P, t, h, start, p);
        for (int c = 0; c < d; ++c) o[c] = 0.0;
        for (int i = 0; i < n; ++i) {
          const double *vj = v + ((size_t)(start + i) * Hkv + kap) * d;
          for (int c = 0; c < d; ++c) o[c] += p[i] * vj[c];
        }
        const double *dot_ = d_o + ((size_t)t * Hq + h) * d;
        const double D = dot(dot_, o, d);
        double *dq = dq_out + ((size_t)r * Hq + h) * d;
        for (int c = 0; c < d; ++c) dq[c] = 0.0;
        for (int i = 0; i < n; ++i) {
          const double *vj = v + ((size_t)(start + i) * Hkv + kap) * d;
          const double *kj = k + ((size_t)(start + i) * Hkv + kap) * d;
          const double ds = p[i] * (dot(dot_, vj, d) - D);
          for (int c = 0; c < d; ++c) dq[c] += ds * kj[c];
        }
        for (int c = 0; c < d; ++c) dq[c] *= scale;
        if (d_out) d_out[(size_t)h * n_rows + r] = D;
      }
    free(p);
    free(o);
  }
  return err ? -2 : 0;
}

/*
 * dK, dV for a list of key tokens j, given the full LSE [Hq, N] and D [Hq, N].
 * dk_out, dv_out: [n_rows, Hkv, d]
 */
int vao_dkv_rows(int32_t N, int32_t B, int32_t Hq, int32_t Hkv, int32_t d, double scale,
                 const double *q, const double *k, const double *v, const double *d_o,
                 const double *lse, const double *D, const int32_t *cu, const int32_t *rows,
                 int32_t n_rows, double *dk_out, double *dv_out) {
  if (!vao_validate_cu(cu, B, N) || Hq % Hkv) return -1;
  const int g = Hq / Hkv;
  int err = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 4)
  for (int r = 0; r < n_rows; ++r)
    for (int kap = 0; kap < Hkv; ++kap) {
      const int j = rows ? rows[r] : r;
      const int b = doc_of_token(cu, B, j);
      if (b < 0) { err = 1; continue; }
      const int end = cu[b + 1];
      const double *kj = k + ((size_t)j * Hkv + kap) * d;
      const double *vj = v + ((size_t)j * Hkv + kap) * d;
      double *dk = dk_out + ((size_t)r * Hkv + kap) * d;
      double *dv = dv_out + ((size_t)r * Hkv + kap) * d;
      for (int c = 0; c < d; ++c) dk[c] = dv[c] = 0.0;
      for (int h = kap * g; h < (kap + 1) * g; ++h)
        for (int t = j; t < end; ++t) {
          const double *qt = q + ((size_t)t * Hq + h) * d;
          const double *dot_ = d_o + ((size_t)t * Hq + h) * d;
          const double p = exp(scale * dot(qt, kj, d) - lse[(size_t)h * N + t]);
          const double ds = p * (dot(dot_, vj, d) - D[(size_t)h * N + t]);
          for (int c = 0; c < d; ++c) dk[c] += ds * qt[c];
          for (int c = 0; c < d; ++c) dv[c] += p * dot_[c];
        }
      for (int c = 0; c < d; ++c) dk[c] *= scale;
    }
  return err ? -2 : 0;
}

/* Full forward: o [N,Hq,d], lse [Hq,N]. */
int vao_fwd(int32_t N, int32_t B, int32_t Hq, int32_t Hkv, int32_t d, double scale,
            const double *q, const double *k, const double *v, const int32_t *cu, double *o,
            double *lse) {
  return vao_fwd_rows(N, B, Hq, Hkv, d, scale, q, k, v, cu, NULL, N, o, lse);
}

/* Full backward: dq [N,Hq,d], dk, dv [N,Hkv,d].  Recomputes the forward itself. */
int vao_bwd(int32_t N, int32_t B, int32_t Hq, int32_t Hkv, int32_t d, double scale,
            const double *q, const double *k, const double *v, const double *d_o,
            const int32_t *cu, double *dq, double *dk, double *dv) {
  double *lse = (double *)malloc(sizeof(double) * (size_t)Hq * N);
  double *D = (double *)malloc(sizeof(double) * (size_t)Hq * N);
  double *o = (double *)malloc(sizeof(double) * (size_t)N * Hq * d);
  if (!lse || !D || !o) { free(lse); free(D); free(o); return -3; }
  int rc = vao_fwd_rows(N, B, Hq, Hkv, d, scale, q, k, v, cu, NULL, N, o, lse);
  if (rc == 0) rc = vao_dq_rows(N, B, Hq, Hkv, d, scale, q, k, v, d_o, cu, NULL, N, dq, D);
  if (rc == 0)
    rc = vao_dkv_rows(N, B, Hq, Hkv, d, scale, q, k, v, d_o, lse, D, cu, NULL, N, dk, dv);
  free(lse); free(D); free(o);
  return rc;
}
