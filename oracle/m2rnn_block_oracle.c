/*
 * Oracle for the two neighbours of the scan in the M2RNN block -- TEST INFRASTRUCTURE, NOT
 * PRODUCT CODE.  Plain float64 loops, one output element after the other, written from the
 * paper's "M2RNN Block" layer equations and its "RMSNormTP Module" appendix.  Shares nothing
 * with the GPU library; only tests, the smoke check and the benchmark's cpu_baseline leg
 * may build, load or call it.
 *
 * (1) Prologue of q, k, v:  out = SiLU(conv1d(x)),  a depthwise causal convolution of kernel
 *     size 4 along time followed by SiLU (layer equations for q_t, k_t, v_t; x is the
 *     projected input W x_t + b of the equation).  Readings: "causal" = the output at step t
 *     sees steps t-3 .. t and the sequence is padded with zeros on the left; tap j of the
 *     kernel multiplies step t-3+j (so tap 3 meets the current step), the cross-correlation
 *     convention of deep-learning libraries; the convolution's own bias is optional (the
 *     paper prints none).  x, out [B,T,C]; w [C,4]; bias [C] or NULL.
 * (2) Epilogue of y:  y_g = RMSNorm(y (.) g),  g = SiLU(a)  (layer equations for g_t and
 *     y_gt; RMSNorm forward and backward as printed in the appendix:
 *         s = 1 / sqrt(mean_j x_j^2),  out_i = w_i x_i s
 *         p_i = w_i dout_i,  r = sum_j p_j x_j,  dx_i = s p_i - r s^3 x_i / d,
 *         dw_i = dout_i x_i s  summed over tokens).
 *     Readings: the normalised axis is ALL d = N V features of a token (the appendix shards
 *     the features over tensor-parallel ranks that hold different heads and needs an
 *     all-reduce for s, so the norm spans the heads); eps is added to the mean square
 *     under the root (the paper prints none; eps = 0 gives the printed formula); the gate
 *     enters as its pre-activation a = W_g x_t and the SiLU is part of this function.
 *     y, a, out [B,T,D]; w [D]; s [B,T] (the cached inverse norm of the appendix).
 */
#include <math.h>
#include <stddef.h>

static double sigmoid(double u) { return 1.0 / (1.0 + exp(-u)); }
/* d/du of SiLU(u) = u sigmoid(u) */
static double silu_grad(double u) {
  const double sg = sigmoid(u);
  return sg * (1.0 + u * (1.0 - sg));
}

#define CONV_TAPS 4

/* pre-activation of the convolution at (b, t, c) */
static double conv_pre(int T, int C, const double *x, const double *w, const double *bias,
                       int b, int t, int c) {
  double a = bias ? bias[c] : 0.0;
  for (int j = 0; j < CONV_TAPS; ++j) {
    const int ts = t - (CONV_TAPS - 1) + j;
    if (ts >= 0) a += w[(size_t)c * CONV_TAPS + j] * x[((size_t)b * T + ts) * C + c];
  }
  return a;
}

int m2rnn_oracle_conv_silu_fwd(int B, int T, int C, const double *x, const double *w,
                               const double *bias, double *out) {
  if (B < 0 || T < 0 || C <= 0) return 1;
  for (int b = 0; b < B; ++b)
    for (int t = 0; t < T; ++t)
      for (int c = 0; c < C; ++c) {
        const double a = conv_pre(T, C, x, w, bias, b, t, c);
        out[((size_t)b * T + t) * C + c] = a * sigmoid(a);
      }
  return 0;
}

/* dx [B,T,C], dw [C,4], dbias [C] (may be NULL) from dout [B,T,C]; all overwritten */
int m2rnn_oracle_conv_silu_bwd(int B, int T, int C, const double *x, const double *w,
                               const double *bias, const double *dout, double *dx, double *dw,
                               double *dbias) {
  if (B < 0 || T < 0 || C <= 0) return 1;
  for (size_t e = 0; e < (size_t)B * T * C; ++e) dx[e] = 0.0;
  for (size_t e = 0; e < (size_t)C * CONV_TAPS; ++e) dw[e] = 0.0;
  if (dbias)
    for (int c = 0; c < C; ++c) dbias[c] = 0.0;
  for (int b = 0; b < B; ++b)
    for (int t = 0; t < T; ++t)
      for (int c = 0; c < C; ++c) {
        const double a = conv_pre(T, C, x, w, bias, b, t, c);
        const double da = dout[((size_t)b * T + t) * C + c] * silu_grad(a);
        if (dbias) dbias[c] += da;
        for (int j = 0; j < CONV_TAPS; ++j) {
          const int ts = t - (CONV_TAPS - 1) + j;
          if (ts < 0) continue;
          dx[((size_t)b * T + ts) * C + c] += w[(size_t)c * CONV_TAPS + j] * da;
          dw[(size_t)c * CONV_TAPS + j] += da * x[((size_t)b * T + ts) * C + c];
        }
      }
  return 0;
}

int m2rnn_oracle_gated_rmsnorm_fwd(int B, int T, int D, const double *y, const double *a,
                                   const double *w, double eps, double *out, double *s_out) {
  if (B < 0 || T < 0 || D <= 0) return 1;
  for (size_t tok = 0; tok < (size_t)B * T; ++tok) {
    const double *yt = y + tok * D, *at = a + tok * D;
    double ss = 0.0;
    for (int j = 0; j < D; ++j) {
      const double xj = yt[j] * (at[j] * sigmoid(at[j]));
      ss += xj * xj;
    }
    const double s = 1.0 / sqrt(ss / D + eps);
    if (s_out) s_out[tok] = s;
    for (int i = 0; i < D; ++i) {
      const double xi = yt[i] * (at[i] * sigmoid(at[i]));
      out[tok * D + i] = w[i] * xi * s;
    }
  }
  return 0;
}

/* dy, da [B,T,D], dw [D] from dout; s is recomputed (the cache is an optimisation) */
int m2rnn_oracle_gated_rmsnorm_bwd(int B, int T, int D, const double *y, const double *a,
                                   const double *w, double eps, const double *dout, double *dy,
                                   double *da, double *dw) {
  if (B < 0 || T < 0 || D <= 0) return 1;
  for (int i = 0; i < D; ++i) dw[i] = 0.0;
  for (size_t tok = 0; tok < (size_t)B * T; ++tok) {
    const double *yt = y + tok * D, *at = a + tok * D, *dot = dout + tok * D;
    double ss = 0.0, r = 0.0;
    for (int j = 0; j < D; ++j) {
      const double xj = yt[j] * (at[j] * sigmoid(at[j]));
      ss += xj * xj;
      r += (w[j] * dot[j]) * xj;
    }
    const double s = 1.0 / sqrt(ss / D + eps);
    for (int i = 0; i < D; ++i) {
      const double g = at[i] * sigmoid(at[i]);
      const double xi = yt[i] * g;
      const double p = w[i] * dot[i];
      const double dxi = s * p - r * s * s * s * xi / D;
      dw[i] += dot[i] * xi * s;
      dy[tok * D + i] = dxi * g;
      da[tok * D + i] = dxi * yt[i] * silu_grad(at[i]);
    }
  }
  return 0;
}
