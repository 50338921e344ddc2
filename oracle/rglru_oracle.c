/*
 * Float64 CPU oracle for the recurrent block's temporal Conv1D -> RG-LRU path
 * (Griffin/Hawk, arxiv 2402.19427).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is the plain definition of what the path
 * computes, written as sequential loops in double precision: no blocking, no
 * fusion, no reordering, no code shared with the HIP library.  Only the test
 * suite, the smoke check and the benchmark's cpu_baseline leg may call it.
 *
 * What it follows:
 *   - Conv1D: Section 2.3 "Recurrent block" (separable temporal filter of
 *     width 4, 4*D_RNN parameters) and Appendix F "Cache sizes" (the decode
 *     state keeps the 3 previous inputs).
 *   - RG-LRU: Section 2.4, eqs. (1)-(4), a = sigmoid(Lambda), c = 8,
 *     y_t = h_t; Appendix A for evaluating a_t in log space.
 *   - Block-diagonal gate weights: Section 4.1 "Recurrent Block".
 *   - Eq. (4) alone as a linear scan over given a_t (or log a_t) and gated
 *     inputs: Section 4.2 "A custom linear scan", Appendix A.3 "Scan runtimes".
 *   - The block's merge, out = y * GeLU(other branch): Section 2.3 "Recurrent
 *     block".
 *   - Backward: not printed in the paper; it is the adjoint of the forward
 *     equations, derived by hand (see oracle_backward below) and pinned by
 *     finite differences in the test suite.
 *
 * Readings taken where the paper is silent or inconsistent:
 *   - Appendix A prints log a_t = -c*softplus(Lambda)*r_t, which contradicts
 *     a = sigmoid(Lambda) from Section 2.4 (log sigmoid(L) = -softplus(-L)).
 *     The main text is followed: log a_t = -c*softplus(-Lambda)*r_t.
 *   - The convolution is causal, taps are indexed by lag (w[k] multiplies
 *     u_{t-k}), inputs before the start of the sequence come from a carried
 *     state when one is given and are zero otherwise; bias is optional.
 *   - x_t in eqs. (1)-(4) is the convolution output.
 *   - GeLU is the exact z*Phi(z) of the cited reference unless the caller
 *     selects that reference's tanh form; the paper does not say which.
 *   - h_{-1} = h0 if given, else 0; the sqrt(1-a^2) factor applies at t = 0
 *     like at any other step.
 *   - Documents packed into one sequence (the paper trains on packed
 *     sequences but gives no convention): an optional mask reset[b][t] != 0
 *     says that a new document starts at step t. Nothing crosses that
 *     boundary: the state entering step t is zero (h_{t-1} := 0) and the
 *     Conv1D sees zeros in place of every input before t - exactly as if the
 *     document were a sequence of its own with no carried states. A NULL
 *     mask means no boundaries.
 *
 * Layouts (all double, row-major, last index fastest):
 *   u, x, y, dy, du : [B][T][D]
 *   W_a, W_x        : [nb][bs][bs]   W[g][j][k]: output j, input k of block g,
 *                     block g covers channels g*bs .. (g+1)*bs-1, bs = D/nb
 *   b_a, b_x, Lambda: [D]
 *   conv_w          : [K][D]  (K = conv width), conv_b : [D] or NULL
 *   h0, hT, dh0, dhT: [B][D]
 *   conv state      : [B][K-1][D], CHRONOLOGICAL: row 0 is the oldest input
 *                     (u_{-(K-1)}), row K-2 is u_{-1}.
 *
 * Parity status: every function here is pinned by tests (closed forms,
 * library special cases, brute force, finite differences, high-precision
 * spot values); none is "parity unpinned".
 */
#include <math.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

static const double PI = 3.14159265358979323846;

static double sigmoid(double z) { return 1.0 / (1.0 + exp(-z)); }

/* log(1 + e^z) without overflow */
static double softplus(double z) {
  return z > 0.0 ? z + log1p(exp(-z)) : log1p(exp(z));
}

/* 1 if a document boundary lies at one of the steps lo+1 .. hi of sequence b
   (steps below 0 are before the call and carry no boundary) */
static int boundary_between(const unsigned char *reset, int T, int b, int lo,
                            int hi) {
  if (!reset) return 0;
  for (int j = (lo + 1 > 0 ? lo + 1 : 0); j <= hi; ++j)
    if (reset[(size_t)b * T + j]) return 1;
  return 0;
}

int oracle_max_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* number of threads the (batch, gate-block) loop of oracle_rglru may use;
 * the canonical parity order is one thread */
void oracle_set_threads(int n) {
#ifdef _OPENMP
  omp_set_num_threads(n > 0 ? n : 1);
#else
  (void)n;
#endif
}

/* ------------------------------------------------------------------------ */
/* Conv1D (Section 2.3): x[b,t,d] = sum_k w[k,d] * u[b,t-k,d] (+ bias[d]).   */
/* u[b,t-k,d] for t-k < 0 is state_in[b][(K-1)+(t-k)][d], or 0 without state. */
/* state_out = the last K-1 inputs seen (carried-in ones included if T<K-1). */
/* ------------------------------------------------------------------------ */
void oracle_conv1d(int B, int T, int D, int K, const double *u,
                   const double *w, const double *bias,
                   const double *state_in, double *x, double *state_out,
                   const unsigned char *reset) {
  const int S = K - 1;
  for (int b = 0; b < B; ++b) {
    for (int t = 0; t < T; ++t) {
      for (int d = 0; d < D; ++d) {
        double acc = bias ? bias[d] : 0.0;
        for (int k = 0; k < K; ++k) {
          int s = t - k;
          double v;
          if (boundary_between(reset, T, b, s, t))
            v = 0.0; /* the input at s belongs to an earlier document */
          else if (s >= 0)
            v = u[((size_t)b * T + s) * D + d];
          else if (state_in)
            v = state_in[((size_t)b * S + (S + s)) * D + d];
          else
            v = 0.0;
          acc += w[(size_t)k * D + d] * v;
        }
        x[((size_t)b * T + t) * D + d] = acc;
      }
    }
    if (state_out) {
      /* position p = T-S+r (r = 0..S-1) in the stream "state_in ++ u" */
      for (int r = 0; r < S; ++r) {
        int s = T - S + r;
        for (int d = 0; d < D; ++d) {
          double v;
          if (boundary_between(reset, T, b, s, T - 1))
            v = 0.0; /* before the last document: not part of its history */
          else if (s >= 0)
            v = u[((size_t)b * T + s) * D + d];
          else if (state_in)
            v = state_in[((size_t)b * S + (S + s)) * D + d];
          else
            v = 0.0;
          state_out[((size_t)b * S + r) * D + d] = v;
        }
      }
    }
  }
}

/* ------------------------------------------------------------------------ */
/* RG-LRU (Section 2.4 eqs. 1-4) on an already convolved input x.            */
/* Optional outputs r_out, i_out, a_out, m_out ([B][T][D]) expose the gates, */
/* the decay a_t and the input scale sqrt(1-a_t^2) for tests.                */
/* ------------------------------------------------------------------------ */
void oracle_rglru(int B, int T, int D, int nb, double c, const double *x,
                  const double *W_a, const double *W_x, const double *b_a,
                  const double *b_x, const double *Lambda, const double *h0,
                  double *y, double *hT, double *r_out, double *i_out,
                  double *a_out, double *m_out, const unsigned char *reset) {
  const int bs = D / nb;
#pragma omp parallel for collapse(2) schedule(dynamic)
  for (int b = 0; b < B; ++b) {
    for (int g = 0; g < nb; ++g) {
      for (int j = 0; j < bs; ++j) {
        const int d = g * bs + j;
        const double *wa = W_a + ((size_t)g * bs + j) * bs;
        const double *wx = W_x + ((size_t)g * bs + j) * bs;
        /* log a = log sigmoid(Lambda) = -softplus(-Lambda)  (Section 2.4) */
        const double log_a = -softplus(-Lambda[d]);
        double h = h0 ? h0[(size_t)b * D + d] : 0.0;
        for (int t = 0; t < T; ++t) {
          const double *xt = x + ((size_t)b * T + t) * D;
          double p = b_a[d], q = b_x[d];
          for (int k = 0; k < bs; ++k) {
            p += wa[k] * xt[g * bs + k];
            q += wx[k] * xt[g * bs + k];
          }
          const double r = sigmoid(p);            /* eq. (1) */
          const double i = sigmoid(q);            /* eq. (2) */
          const double la = c * r * log_a;        /* eq. (3), log space */
          const double a = exp(la);
          const double m = sqrt(-expm1(2.0 * la)); /* sqrt(1 - a^2) */
          if (reset && reset[(size_t)b * T + t]) h = 0.0; /* new document */
          h = a * h + m * (i * xt[d]);            /* eq. (4) */
          const size_t o = ((size_t)b * T + t) * D + d;
          y[o] = h;
          if (r_out) r_out[o] = r;
          if (i_out) i_out[o] = i;
          if (a_out) a_out[o] = a;
          if (m_out) m_out[o] = m;
        }
        if (hT) hT[(size_t)b * D + d] = h;
      }
    }
  }
}

/* ------------------------------------------------------------------------ */
/* Eq. (4) alone, as a linear scan over given sequences (Section 4.2, "A     */
/* custom linear scan"; the operation timed in Appendix A.3, "Scan           */
/* runtimes"): per element the decay a_t - or log a_t, the form Appendix A   */
/* evaluates it in - and the gated input g_t = i_t x_t.                      */
/*   h_t = a_t h_{t-1} + m_t g_t,  m_t = sqrt(1 - a_t^2) (normalize != 0)    */
/*                                 m_t = 1               (normalize == 0)    */
/* a, g, h: [B][T][D]; h0, hT: [B][D] (h0 NULL = zeros, hT NULL = skipped).  */
/* ------------------------------------------------------------------------ */
void oracle_scan(int B, int T, int D, int a_is_log, int normalize,
                 const double *a, const double *g, const double *h0,
                 double *h, double *hT) {
  for (int b = 0; b < B; ++b) {
    for (int d = 0; d < D; ++d) {
      double s = h0 ? h0[(size_t)b * D + d] : 0.0;
      for (int t = 0; t < T; ++t) {
        const size_t o = ((size_t)b * T + t) * D + d;
        const double av = a_is_log ? exp(a[o]) : a[o];
        double m = 1.0;
        if (normalize)
          m = a_is_log ? sqrt(-expm1(2.0 * a[o])) : sqrt(1.0 - av * av);
        s = av * s + m * g[o];
        h[o] = s;
      }
      if (hT) hT[(size_t)b * D + d] = s;
    }
  }
}

/* ------------------------------------------------------------------------ */
/* The adjoint of that scan with respect to its inputs (not printed in the   */
/* paper; it is what training through eq. (4) needs): for                    */
/*   h_t = a_t h_{t-1} + b_t  and  L = sum_t dy_t h_t + dhT h_{T-1}          */
/* the gradient reaching h_t is                                              */
/*   delta_t = dy_t + a_{t+1} delta_{t+1},  delta_{T-1} = dy_{T-1} + dhT,    */
/* dL/db_t = delta_t, dL/da_t = delta_t h_{t-1}, dL/dh_{-1} = a_0 delta_0.   */
/* a, dy, delta: [B][T][D]; dhT, dh0: [B][D] (dhT NULL = zeros, dh0 NULL =   */
/* skipped). ``a`` holds a_t, or log a_t when a_is_log.                      */
/* ------------------------------------------------------------------------ */
void oracle_scan_adjoint(int B, int T, int D, int a_is_log, const double *a,
                         const double *dy, const double *dhT, double *delta,
                         double *dh0) {
  for (int b = 0; b < B; ++b) {
    for (int d = 0; d < D; ++d) {
      double s = dhT ? dhT[(size_t)b * D + d] : 0.0;  /* a_{t+1} delta_{t+1} */
      for (int t = T - 1; t >= 0; --t) {
        const size_t o = ((size_t)b * T + t) * D + d;
        const double dl = dy[o] + s;
        delta[o] = dl;
        s = (a_is_log ? exp(a[o]) : a[o]) * dl;
      }
      if (dh0) dh0[(size_t)b * D + d] = s;
    }
  }
}

/* ------------------------------------------------------------------------ */
/* The recurrent block's merge (Section 2.3, "Recurrent block"): the output  */
/* of the RG-LRU branch is multiplied element by element with GeLU of the    */
/* other branch.  GeLU(z) = z * Phi(z) with Phi the standard normal CDF (the */
/* definition of the cited reference); approx != 0 selects that reference's  */
/* tanh form, 0.5 z (1 + tanh(sqrt(2/pi) (z + 0.044715 z^3))).               */
/* ------------------------------------------------------------------------ */
double oracle_gelu(double z, int approx) {
  if (approx) {
    const double k = sqrt(2.0 / PI) * (z + 0.044715 * z * z * z);
    return 0.5 * z * (1.0 + tanh(k));
  }
  return 0.5 * z * (1.0 + erf(z / sqrt(2.0)));
}

/* d GeLU / dz: Phi(z) + z phi(z), or the derivative of the tanh form */
double oracle_gelu_grad(double z, int approx) {
  if (approx) {
    const double s = sqrt(2.0 / PI);
    const double th = tanh(s * (z + 0.044715 * z * z * z));
    return 0.5 * (1.0 + th) +
           0.5 * z * (1.0 - th * th) * s * (1.0 + 3.0 * 0.044715 * z * z);
  }
  return 0.5 * (1.0 + erf(z / sqrt(2.0))) +
         z * exp(-0.5 * z * z) / sqrt(2.0 * PI);
}

/* out = y * GeLU(branch), n elements */
void oracle_merge(size_t n, int approx, const double *y, const double *branch,
                  double *out) {
  for (size_t i = 0; i < n; ++i) out[i] = y[i] * oracle_gelu(branch[i], approx);
}

/* adjoint of oracle_merge: dy = dout * GeLU(branch),                        */
/* dbranch = dout * y * GeLU'(branch)                                        */
void oracle_merge_backward(size_t n, int approx, const double *y,
                           const double *branch, const double *dout,
                           double *dy, double *dbranch) {
  for (size_t i = 0; i < n; ++i) {
    dy[i] = dout[i] * oracle_gelu(branch[i], approx);
    dbranch[i] = dout[i] * y[i] * oracle_gelu_grad(branch[i], approx);
  }
}

/* Conv1D followed by the RG-LRU: the whole forward path. */
void oracle_forward(int B, int T, int D, int nb, int K, double c,
                    const double *u, const double *W_a, const double *W_x,
                    const double *b_a, const double *b_x, const double *Lambda,
                    const double *conv_w, const double *conv_b,
                    const double *h0, const double *state_in, double *y,
                    double *hT, double *state_out, const unsigned char *reset) {
  double *x = (double *)malloc((size_t)B * T * D * sizeof(double));
  oracle_conv1d(B, T, D, K, u, conv_w, conv_b, state_in, x, state_out, reset);
  oracle_rglru(B, T, D, nb, c, x, W_a, W_x, b_a, b_x, Lambda, h0, y, hT, NULL,
               NULL, NULL, NULL, reset);
  free(x);
}

/* ------------------------------------------------------------------------ */
/* One decode step (Section 5 / Appendix F): the same equations for a single */
/* new token per sequence.  Written on its own, with a chronological shift   */
/* buffer, so that it cross-checks both oracle_forward and any ring-buffer   */
/* convention used elsewhere.  h and state are updated in place.             */
/* ------------------------------------------------------------------------ */
void oracle_decode_step(int B, int D, int nb, int K, double c,
                        const double *u_t, const double *W_a,
                        const double *W_x, const double *b_a,
                        const double *b_x, const double *Lambda,
                        const double *conv_w, const double *conv_b, double *h,
                        double *state, double *y_t) {
  const int bs = D / nb, S = K - 1;
  double *x = (double *)malloc((size_t)D * sizeof(double));
  for (int b = 0; b < B; ++b) {
    double *st = state + (size_t)b * S * D;
    for (int d = 0; d < D; ++d) {
      double acc = conv_b ? conv_b[d] : 0.0;
      acc += conv_w[d] * u_t[(size_t)b * D + d]; /* lag 0 */
      for (int k = 1; k < K; ++k)                /* lag k is row S-k */
        acc += conv_w[(size_t)k * D + d] * st[(size_t)(S - k) * D + d];
      x[d] = acc;
    }
    for (int d = 0; d < D; ++d) {
      const int g = d / bs, j = d % bs;
      double p = b_a[d], q = b_x[d];
      for (int k = 0; k < bs; ++k) {
        p += W_a[((size_t)g * bs + j) * bs + k] * x[g * bs + k];
        q += W_x[((size_t)g * bs + j) * bs + k] * x[g * bs + k];
      }
      const double r = sigmoid(p), i = sigmoid(q);
      const double la = -c * softplus(-Lambda[d]) * r;
      const double a = exp(la), m = sqrt(-expm1(2.0 * la));
      const double hn = a * h[(size_t)b * D + d] + m * (i * x[d]);
      h[(size_t)b * D + d] = hn;
      y_t[(size_t)b * D + d] = hn;
    }
    /* shift the window: drop the oldest row, append the new token */
    for (int s = 0; s + 1 < S; ++s)
      memcpy(st + (size_t)s * D, st + (size_t)(s + 1) * D, D * sizeof(double));
    if (S > 0)
      memcpy(st + (size_t)(S - 1) * D, u_t + (size_t)b * D, D * sizeof(double));
  }
  free(x);
}

/* ------------------------------------------------------------------------ */
/* Backward of the forward path: the adjoint of Section 2.4 eqs. (1)-(4) and */
/* of the Conv1D, for the scalar loss L = sum dy.y + sum dhT.hT.             */
/*                                                                          */
/* With g_t = i_t x_t, s = softplus(-Lambda), la_t = -c s r_t, a_t = e^la_t, */
/* m_t = sqrt(1-a_t^2):                                                     */
/*   delta_t = dy_t + a_{t+1} delta_{t+1}   (delta_{T-1} = dy_{T-1} + dhT)   */
/*   dh0     = a_0 delta_0                                                  */
/*   dla_t   = delta_t a_t (h_{t-1} - a_t g_t / m_t)      (dm/da = -a/m)     */
/*   dg_t    = delta_t m_t ;  di_t = dg_t x_t ;  dx_t = dg_t i_t  (direct)   */
/*   dr_t    = -c s dla_t ;   dLambda += dla_t c r_t (1 - sigmoid(Lambda))   */
/*   dp_t    = dr_t r_t (1-r_t) ;  dq_t = di_t i_t (1-i_t)                   */
/*   db_a += dp_t ; db_x += dq_t ; dW_a[g,j,k] += dp_t[j] x_t[k] (same W_x)  */
/*   dx_t[k] += sum_j W_a[g,j,k] dp_t[j] + W_x[g,j,k] dq_t[j]                */
/*   du_{t-k} += w[k] dx_t ;  dw[k] += dx_t u_{t-k} ;  dconv_b += dx_t       */
/* Inputs before the sequence start (the carried conv state) receive no     */
/* gradient.  Parameter gradients are overwritten (summed over B and T).    */
/* Any of dhT, dh0, dconv_b may be NULL.                                    */
/* With document boundaries (reset, see the top of this file) nothing flows  */
/* across a boundary at step t: a_t delta_t does not reach step t-1 (nor     */
/* dh0 when t = 0), h_{t-1} counts as zero in dla_t, and the Conv1D adjoint   */
/* skips every (step, lag) pair whose input lies before the boundary.        */
/* ------------------------------------------------------------------------ */
void oracle_backward(int B, int T, int D, int nb, int K, double c,
                     const double *u, const double *W_a, const double *W_x,
                     const double *b_a, const double *b_x,
                     const double *Lambda, const double *conv_w,
                     const double *conv_b, const double *h0,
                     const double *state_in, const double *dy,
                     const double *dhT, double *du, double *dh0, double *dW_a,
                     double *dW_x, double *db_a, double *db_x, double *dLambda,
                     double *dconv_w, double *dconv_b,
                     const unsigned char *reset) {
  const int bs = D / nb, S = K - 1;
  const size_t N = (size_t)B * T * D;
  double *x = (double *)malloc(N * sizeof(double));
  double *y = (double *)malloc(N * sizeof(double));
  double *r = (double *)malloc(N * sizeof(double));
  double *ig = (double *)malloc(N * sizeof(double));
  double *a = (double *)malloc(N * sizeof(double));
  double *m = (double *)malloc(N * sizeof(double));
  double *dp = (double *)malloc(N * sizeof(double));
  double *dq = (double *)malloc(N * sizeof(double));
  double *dx = (double *)malloc(N * sizeof(double));

  /* forward, keeping every intermediate */
  oracle_conv1d(B, T, D, K, u, conv_w, conv_b, state_in, x, NULL, reset);
  oracle_rglru(B, T, D, nb, c, x, W_a, W_x, b_a, b_x, Lambda, h0, y, NULL, r,
               ig, a, m, reset);

  memset(dW_a, 0, (size_t)nb * bs * bs * sizeof(double));
  memset(dW_x, 0, (size_t)nb * bs * bs * sizeof(double));
  memset(db_a, 0, (size_t)D * sizeof(double));
  memset(db_x, 0, (size_t)D * sizeof(double));
  memset(dLambda, 0, (size_t)D * sizeof(double));
  memset(dconv_w, 0, (size_t)K * D * sizeof(double));
  if (dconv_b) memset(dconv_b, 0, (size_t)D * sizeof(double));
  memset(du, 0, N * sizeof(double));

  /* reverse scan and pointwise adjoints */
  for (int b = 0; b < B; ++b) {
    for (int d = 0; d < D; ++d) {
      const double s = softplus(-Lambda[d]);
      const double one_minus_sig = 1.0 - sigmoid(Lambda[d]);
      double delta_next = 0.0, a_next = 0.0;
      for (int t = T - 1; t >= 0; --t) {
        const size_t o = ((size_t)b * T + t) * D + d;
        double delta = dy[o] + a_next * delta_next;
        if (t == T - 1 && dhT) delta += dhT[(size_t)b * D + d];
        const int fresh = reset && reset[(size_t)b * T + t]; /* new document */
        const double h_prev =
            fresh ? 0.0
                  : (t > 0 ? y[o - D] : (h0 ? h0[(size_t)b * D + d] : 0.0));
        const double g = ig[o] * x[o];
        const double dla = delta * a[o] * (h_prev - a[o] * g / m[o]);
        const double dg = delta * m[o];
        const double di = dg * x[o];
        dx[o] = dg * ig[o];
        const double dr = -c * s * dla;
        dLambda[d] += dla * c * r[o] * one_minus_sig;
        dp[o] = dr * r[o] * (1.0 - r[o]);
        dq[o] = di * ig[o] * (1.0 - ig[o]);
        db_a[d] += dp[o];
        db_x[d] += dq[o];
        delta_next = delta;
        a_next = fresh ? 0.0 : a[o]; /* nothing reaches the step before */
      }
      if (dh0) dh0[(size_t)b * D + d] = a_next * delta_next;
    }
  }

  /* gate projections: weight gradients and the gradient reaching x */
  for (int b = 0; b < B; ++b) {
    for (int t = 0; t < T; ++t) {
      const size_t row = ((size_t)b * T + t) * D;
      for (int g = 0; g < nb; ++g) {
        for (int j = 0; j < bs; ++j) {
          const double dpj = dp[row + g * bs + j];
          const double dqj = dq[row + g * bs + j];
          const size_t wrow = ((size_t)g * bs + j) * bs;
          for (int k = 0; k < bs; ++k) {
            dW_a[wrow + k] += dpj * x[row + g * bs + k];
            dW_x[wrow + k] += dqj * x[row + g * bs + k];
            dx[row + g * bs + k] += W_a[wrow + k] * dpj + W_x[wrow + k] * dqj;
          }
        }
      }
    }
  }

  /* Conv1D adjoint */
  for (int b = 0; b < B; ++b) {
    for (int t = 0; t < T; ++t) {
      for (int d = 0; d < D; ++d) {
        const double dxt = dx[((size_t)b * T + t) * D + d];
        if (dconv_b) dconv_b[d] += dxt;
        for (int k = 0; k < K; ++k) {
          const int sidx = t - k;
          double v;
          if (boundary_between(reset, T, b, sidx, t)) continue;
          if (sidx >= 0) {
            const size_t o = ((size_t)b * T + sidx) * D + d;
            du[o] += conv_w[(size_t)k * D + d] * dxt;
            v = u[o];
          } else if (state_in) {
            v = state_in[((size_t)b * S + (S + sidx)) * D + d];
          } else {
            v = 0.0;
          }
          dconv_w[(size_t)k * D + d] += dxt * v;
        }
      }
    }
  }

  free(x); free(y); free(r); free(ig); free(a); free(m);
  free(dp); free(dq); free(dx);
}
