/*
 * M2RNN recurrence oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, float64 CPU statement of what the recurrent scan computes,
 * one time step after the other, exactly as the paper defines it.  It exists
 * so that the GPU library can be checked against something that can be read
 * next to the paper by eye.  It shares no code, header, table or helper with
 * the GPU path and must never be reached from it: only the tests, the smoke
 * check and the benchmark's cpu_baseline leg may build, load or call it.
 *
 * Forward  : the recurrence equations of the paper's "M2RNN layer" section
 *            (Z_t = tanh(H_{t-1} W + k_t v_t^T); H_t = f_t H_{t-1} + (1-f_t) Z_t;
 *            y_t = H_t^T q_t), in the loop order of the forward algorithm
 *            (Algorithm 1).  The residual term w_r (.) v_t of the y equation
 *            (w_r: one weight per head and value channel) is added when w_r is
 *            given; Algorithm 1 leaves it out, and so does a NULL w_r.
 * Backward : back-propagation through time as in the backward algorithm
 *            (Algorithm 2), with three readings of the printed listing:
 *              (1) the gradient of H_t is  q_t dy_t^T PLUS the gradient carried
 *                  from step t+1 (the listing drops the carried term);
 *              (2) the gradient passed to step t-1 is  f_t * G + dX W^T
 *                  (the listing's elementwise product there is a misprint);
 *              (3) dF is real valued.
 *            These readings are what the chain rule gives for the forward
 *            equations; the tests pin them with finite differences and with
 *            reverse-mode differentiation of an unrolled forward.
 *            Per-step clipping of the state gradient (the paper's "Gradient
 *            Clipping" paragraph names it without a rule): with clip > 0 every
 *            element of the gradient handed from step t to step t-1 is clamped
 *            to [-clip, clip] as soon as it is formed, i.e. before q dy^T of
 *            step t-1 is added; dH0 is the clamped value; dHT is taken as
 *            given.  clip <= 0 switches it off (exact gradients).
 *
 * Pins (tests/test_oracle_*.py): T=1 closed form, unrolled brute force,
 * finite differences, the Elman-RNN reduction of Theorem 1, the W=0 closed
 * form, the f=1 / f=0 gate limits, segment chaining, row independence and
 * permutation symmetries, the |H|<=1 bound, linearity of the backward.
 *
 * Forget gate (the paper's "Forget Gate" section): with gate parameters alpha, beta
 * (one each per head) the argument f holds the gate's input x, and the gate value is
 * f = psi(x) = (1 + e^(x + beta))^(-alpha); the backward then returns the gradient with
 * respect to x in df, and dalpha, dbeta summed over b and t.  Without them f is the gate
 * value itself.
 *
 * Layouts (dense, row-major, host memory, all double):
 *   q, k  [B,T,Nqk,K]   v, y, dy, dv [B,T,N,V]   f, df [B,T,N]
 *   W, dW [N,V,V]       H0, HT, dHT, dH0 [B,N,K,V]     w_r, dw_r [N,V]
 * Head n reads q/k head  n / (N/Nqk)  (Nqk = N: one q/k per head; Nqk = 1: the
 * paper's multi-value form where all heads share q and k).
 * K and V are NOT restricted to multiples of 16 here, so that tiny brute-force
 * cases (K = V = 2) can be run.
 *
 * OpenMP spreads independent (b, n) recurrences over threads; nothing inside
 * a recurrence is blocked, fused or reordered.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define IDX_QK(b, t, g, i) ((((size_t)(b) * T + (t)) * Nqk + (g)) * K + (i))
#define IDX_V(b, t, n, j) ((((size_t)(b) * T + (t)) * N + (n)) * V + (j))
#define IDX_F(b, t, n) (((size_t)(b) * T + (t)) * N + (n))
#define IDX_H(b, n) (((size_t)(b) * N + (n)) * K * V)

int m2rnn_oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* psi(x) = (1 + e^(x + beta))^(-alpha), through log1p for large |x + beta| */
static double softplus(double u) {
  return (u > 0.0 ? u : 0.0) + log1p(exp(-fabs(u)));
}
static double gate_value(const double *alpha, const double *beta, int n, double x) {
  if (!alpha) return x;
  return exp(-alpha[n] * softplus(x + beta[n]));
}

/* One step of the recurrence for one (b, n): H (K x V) is updated in place.
 * Z, if not NULL, receives tanh(H_prev W + k v^T).  S is K*V scratch. */
static void step_forward(int K, int V, const double *W, const double *kt,
                         const double *vt, double ft, double *H, double *S,
                         double *Z) {
  for (int i = 0; i < K; ++i)
    for (int j = 0; j < V; ++j) {
      double s = 0.0;
      for (int c = 0; c < V; ++c) s += H[i * V + c] * W[c * V + j];
      S[i * V + j] = s + kt[i] * vt[j];
    }
  for (int e = 0; e < K * V; ++e) {
    double z = tanh(S[e]);
    if (Z) Z[e] = z;
    H[e] = ft * H[e] + (1.0 - ft) * z;
  }
}

/* Forward recurrence.  H0 may be NULL (zero state); HT may be NULL. */
int m2rnn_oracle_fwd(int B, int T, int N, int Nqk, int K, int V,
                     const double *q, const double *k, const double *v,
                     const double *f, const double *W, const double *H0,
                     const double *w_r, const double *alpha, const double *beta,
                     double *y, double *HT) {
  if (B < 0 || T < 0 || N <= 0 || Nqk <= 0 || K <= 0 || V <= 0) return 1;
  if (N % Nqk != 0) return 1;
  const int heads_per_group = N / Nqk;
  int fail = 0;
#pragma omp parallel for collapse(2) schedule(dynamic)
  for (int b = 0; b < B; ++b)
    for (int n = 0; n < N; ++n) {
      const int g = n / heads_per_group;
      const double *Wn = W + (size_t)n * V * V;
      double *H = (double *)malloc(sizeof(double) * K * V);
      double *S = (double *)malloc(sizeof(double) * K * V);
      if (!H || !S) {
        fail = 1;
        free(H);
        free(S);
        continue;
      }
      if (H0)
        memcpy(H, H0 + IDX_H(b, n), sizeof(double) * K * V);
      else
        memset(H, 0, sizeof(double) * K * V);
      for (int t = 0; t < T; ++t) {
        step_forward(K, V, Wn, k + IDX_QK(b, t, g, 0), v + IDX_V(b, t, n, 0),
                     gate_value(alpha, beta, n, f[IDX_F(b, t, n)]), H, S, NULL);
        const double *qt = q + IDX_QK(b, t, g, 0);
        for (int j = 0; j < V; ++j) {
          double acc = 0.0;
          for (int i = 0; i < K; ++i) acc += H[i * V + j] * qt[i];
          if (w_r) acc += w_r[(size_t)n * V + j] * v[IDX_V(b, t, n, j)];
          y[IDX_V(b, t, n, j)] = acc;
        }
      }
      if (HT) memcpy(HT + IDX_H(b, n), H, sizeof(double) * K * V);
      free(H);
      free(S);
    }
  return fail;
}

/* Backward (BPTT).  Every state of the forward run is kept in memory for the
 * unit being processed (T+1 matrices of K x V).  H0, dHT, dH0 may be NULL.
 * dq, dk are sums over the heads that share a q/k head, added in increasing
 * head order; dW is the sum over the batch, added in increasing b.
 * w_r (with dw_r) may be NULL: no residual.  clip <= 0: no clipping. */
int m2rnn_oracle_bwd(int B, int T, int N, int Nqk, int K, int V,
                     const double *q, const double *k, const double *v,
                     const double *f, const double *W, const double *H0,
                     const double *w_r, double clip, const double *alpha,
                     const double *beta, const double *dy, const double *dHT,
                     double *dq, double *dk, double *dv, double *df, double *dW,
                     double *dH0, double *dw_r, double *dalpha, double *dbeta) {
  if (B < 0 || T < 0 || N <= 0 || Nqk <= 0 || K <= 0 || V <= 0) return 1;
  if (N % Nqk != 0) return 1;
  const int heads_per_group = N / Nqk;
  const size_t KV = (size_t)K * V;
  /* per-unit results that are summed afterwards in a fixed order */
  double *dq_unit = (double *)calloc((size_t)B * T * N * K + 1, sizeof(double));
  double *dk_unit = (double *)calloc((size_t)B * T * N * K + 1, sizeof(double));
  double *dW_unit = (double *)calloc((size_t)B * N * V * V + 1, sizeof(double));
  if (!dq_unit || !dk_unit || !dW_unit) {
    free(dq_unit);
    free(dk_unit);
    free(dW_unit);
    return 2;
  }
  int fail = 0;
#pragma omp parallel for collapse(2) schedule(dynamic)
  for (int b = 0; b < B; ++b)
    for (int n = 0; n < N; ++n) {
      const int g = n / heads_per_group;
      const double *Wn = W + (size_t)n * V * V;
      double *Hall = (double *)malloc(sizeof(double) * KV * ((size_t)T + 1));
      double *S = (double *)malloc(sizeof(double) * KV);
      double *Z = (double *)malloc(sizeof(double) * KV);
      double *G = (double *)malloc(sizeof(double) * KV);
      double *dS = (double *)malloc(sizeof(double) * KV);
      double *C = (double *)malloc(sizeof(double) * KV);
      double *Hp = (double *)malloc(sizeof(double) * KV);
      if (!Hall || !S || !Z || !G || !dS || !C || !Hp) {
        fail = 1;
        free(Hall); free(S); free(Z); free(G); free(dS); free(C); free(Hp);
        continue;
      }
      /* forward sweep, keeping H_0 .. H_T (state before step t is Hall[t]) */
      if (H0)
        memcpy(Hall, H0 + IDX_H(b, n), sizeof(double) * KV);
      else
        memset(Hall, 0, sizeof(double) * KV);
      for (int t = 0; t < T; ++t) {
        memcpy(Hall + (size_t)(t + 1) * KV, Hall + (size_t)t * KV,
               sizeof(double) * KV);
        step_forward(K, V, Wn, k + IDX_QK(b, t, g, 0), v + IDX_V(b, t, n, 0),
                     gate_value(alpha, beta, n, f[IDX_F(b, t, n)]),
                     Hall + (size_t)(t + 1) * KV, S, NULL);
      }
      /* gradient carried into the last state */
      if (dHT)
        memcpy(C, dHT + IDX_H(b, n), sizeof(double) * KV);
      else
        memset(C, 0, sizeof(double) * KV);
      double *dWu = dW_unit + ((size_t)b * N + n) * V * V;

      for (int t = T - 1; t >= 0; --t) {
        const double *Hprev = Hall + (size_t)t * KV;
        const double *Hnext = Hall + (size_t)(t + 1) * KV;
        const double *qt = q + IDX_QK(b, t, g, 0);
        const double *kt = k + IDX_QK(b, t, g, 0);
        const double *vt = v + IDX_V(b, t, n, 0);
        const double *dyt = dy + IDX_V(b, t, n, 0);
        const double ft = gate_value(alpha, beta, n, f[IDX_F(b, t, n)]);
        /* recompute Z_t from the state before the step */
        memcpy(Hp, Hprev, sizeof(double) * KV);
        step_forward(K, V, Wn, kt, vt, ft, Hp, S, Z);
        /* dq_t = H_t dy_t */
        double *dqt = dq_unit + (((size_t)b * T + t) * N + n) * K;
        for (int i = 0; i < K; ++i) {
          double acc = 0.0;
          for (int j = 0; j < V; ++j) acc += Hnext[i * V + j] * dyt[j];
          dqt[i] = acc;
        }
        /* G = q_t dy_t^T + carried gradient : total dL/dH_t */
        for (int i = 0; i < K; ++i)
          for (int j = 0; j < V; ++j) G[i * V + j] = qt[i] * dyt[j] + C[i * V + j];
        /* df_t = sum G (.) (H_{t-1} - Z_t) */
        double dft = 0.0;
        for (size_t e = 0; e < KV; ++e) dft += G[e] * (Hprev[e] - Z[e]);
        df[IDX_F(b, t, n)] = dft;
        /* through the gate's non-linear branch and through tanh */
        for (size_t e = 0; e < KV; ++e)
          dS[e] = (1.0 - ft) * G[e] * (1.0 - Z[e] * Z[e]);
        /* gradient of the state before the step: f_t G + dS W^T */
        for (int i = 0; i < K; ++i)
          for (int c = 0; c < V; ++c) {
            double acc = 0.0;
            for (int j = 0; j < V; ++j) acc += dS[i * V + j] * Wn[c * V + j];
            C[i * V + c] = ft * G[i * V + c] + acc;
          }
        if (clip > 0.0)
          for (size_t e = 0; e < KV; ++e)
            C[e] = C[e] > clip ? clip : (C[e] < -clip ? -clip : C[e]);
        /* dW += H_{t-1}^T dS */
        for (int c = 0; c < V; ++c)
          for (int j = 0; j < V; ++j) {
            double acc = 0.0;
            for (int i = 0; i < K; ++i) acc += Hprev[i * V + c] * dS[i * V + j];
            dWu[c * V + j] += acc;
          }
        /* dk_t = dS v_t ;  dv_t = dS^T k_t */
        double *dkt = dk_unit + (((size_t)b * T + t) * N + n) * K;
        for (int i = 0; i < K; ++i) {
          double acc = 0.0;
          for (int j = 0; j < V; ++j) acc += dS[i * V + j] * vt[j];
          dkt[i] = acc;
        }
        for (int j = 0; j < V; ++j) {
          double acc = 0.0;
          for (int i = 0; i < K; ++i) acc += dS[i * V + j] * kt[i];
          /* y_t also holds w_r (.) v_t */
          if (w_r) acc += w_r[(size_t)n * V + j] * dyt[j];
          dv[IDX_V(b, t, n, j)] = acc;
        }
      }
      if (dH0) memcpy(dH0 + IDX_H(b, n), C, sizeof(double) * KV);
      free(Hall); free(S); free(Z); free(G); free(dS); free(C); free(Hp);
    }
  /* ordered sums: heads of a q/k group, then the batch for dW */
  for (int b = 0; b < B; ++b)
    for (int t = 0; t < T; ++t)
      for (int g = 0; g < Nqk; ++g)
        for (int i = 0; i < K; ++i) {
          double sq = 0.0, sk = 0.0;
          for (int h = 0; h < heads_per_group; ++h) {
            const int n = g * heads_per_group + h;
            sq += dq_unit[(((size_t)b * T + t) * N + n) * K + i];
            sk += dk_unit[(((size_t)b * T + t) * N + n) * K + i];
          }
          dq[IDX_QK(b, t, g, i)] = sq;
          dk[IDX_QK(b, t, g, i)] = sk;
        }
  for (int n = 0; n < N; ++n)
    for (int e = 0; e < V * V; ++e) {
      double s = 0.0;
      for (int b = 0; b < B; ++b) s += dW_unit[((size_t)b * N + n) * V * V + e];
      dW[(size_t)n * V * V + e] = s;
    }
  /* through the gate function: df holds dL/d(gate value) so far.
   * d psi/dx = d psi/dbeta = -alpha psi sigmoid(x + beta);  d psi/dalpha = -psi softplus(x + beta) */
  if (alpha) {
    for (int n = 0; n < N; ++n) {
      double sa = 0.0, sb = 0.0;
      for (int b = 0; b < B; ++b)
        for (int t = 0; t < T; ++t) {
          const double u = f[IDX_F(b, t, n)] + beta[n];
          const double sp = softplus(u);
          const double psi = exp(-alpha[n] * sp);
          const double g = df[IDX_F(b, t, n)];
          const double dx = -g * alpha[n] * psi / (1.0 + exp(-u));
          sa += -g * psi * sp;
          sb += dx;
          df[IDX_F(b, t, n)] = dx;
        }
      dalpha[n] = sa;
      dbeta[n] = sb;
    }
  }
  /* dw_r[n][j] = sum over b and t of dy (.) v */
  if (w_r && dw_r)
    for (int n = 0; n < N; ++n)
      for (int j = 0; j < V; ++j) {
        double s = 0.0;
        for (int b = 0; b < B; ++b)
          for (int t = 0; t < T; ++t)
            s += dy[IDX_V(b, t, n, j)] * v[IDX_V(b, t, n, j)];
        dw_r[(size_t)n * V + j] = s;
      }
  free(dq_unit);
  free(dk_unit);
  free(dW_unit);
  return fail;
}
