/* Memory-safety check of the oracle's C code (test infrastructure): calls every entry point
 * of rglru_oracle.c on small, exactly sized heap buffers, with and without the optional
 * arguments, ragged shapes and document boundaries. Built together with rglru_oracle.c under
 * -fsanitize=address,undefined by tests/test_sanitizers.py; any out-of-bounds access,
 * misaligned or undefined operation aborts the run. Prints "ok" when every call returned. */
#include <stdio.h>
#include <stdlib.h>

void oracle_set_threads(int n);
void oracle_conv1d(int B, int T, int D, int K, const double *u, const double *w, const double *bias,
                   const double *state_in, double *x, double *state_out, const unsigned char *reset);
void oracle_rglru(int B, int T, int D, int nb, double c, const double *x, const double *W_a,
                  const double *W_x, const double *b_a, const double *b_x, const double *Lambda,
                  const double *h0, double *y, double *hT, double *r_out, double *i_out, double *a_out,
                  double *m_out, const unsigned char *reset);
void oracle_scan(int B, int T, int D, int a_is_log, int normalize, const double *a, const double *g,
                 const double *h0, double *h, double *hT);
void oracle_scan_adjoint(int B, int T, int D, int a_is_log, const double *a, const double *dh,
                         const double *dhT, double *delta, double *d0);
void oracle_merge(size_t n, int approx, const double *y, const double *branch, double *out);
void oracle_merge_backward(size_t n, int approx, const double *y, const double *branch, const double *dout,
                           double *dy, double *dbranch);
void oracle_forward(int B, int T, int D, int nb, int K, double c, const double *u, const double *W_a,
                    const double *W_x, const double *b_a, const double *b_x, const double *Lambda,
                    const double *conv_w, const double *conv_b, const double *h0, const double *state_in,
                    double *y, double *hT, double *state_out, const unsigned char *reset);
void oracle_decode_step(int B, int D, int nb, int K, double c, const double *u_t, const double *W_a,
                        const double *W_x, const double *b_a, const double *b_x, const double *Lambda,
                        const double *conv_w, const double *conv_b, double *h, double *state, double *y_t);
void oracle_backward(int B, int T, int D, int nb, int K, double c, const double *u, const double *W_a,
                     const double *W_x, const double *b_a, const double *b_x, const double *Lambda,
                     const double *conv_w, const double *conv_b, const double *h0, const double *state_in,
                     const double *dy, const double *dhT, double *du, double *dh0, double *dW_a, double *dW_x,
                     double *db_a, double *db_x, double *dLambda, double *dconv_w, double *dconv_b,
                     const unsigned char *reset);

static unsigned long long lcg = 88172645463325252ULL;
static double draw(void) {   /* xorshift, values in (-1, 1) */
  lcg ^= lcg << 13; lcg ^= lcg >> 7; lcg ^= lcg << 17;
  return (double)(lcg % 2000001ULL) / 1000000.0 - 1.0;
}
static double *vec(size_t n) {   /* exactly n doubles: one element more is out of bounds */
  double *p = (double *)malloc((n ? n : 1) * sizeof(double));
  for (size_t i = 0; i < n; ++i) p[i] = draw();
  return p;
}

static void one_case(int B, int T, int D, int nb, int with_opt, int with_reset) {
  const int K = 4, bs = D / nb;
  const size_t N = (size_t)B * T * D, BD = (size_t)B * D;
  double *u = vec(N), *Wa = vec((size_t)nb * bs * bs), *Wx = vec((size_t)nb * bs * bs);
  double *ba = vec(D), *bx = vec(D), *lam = vec(D), *cw = vec((size_t)K * D), *cb = vec(D);
  double *h0 = vec(BD), *st = vec(BD * (K - 1)), *dy = vec(N), *dhT = vec(BD);
  double *x = vec(N), *y = vec(N), *hT = vec(BD), *sto = vec(BD * (K - 1));
  double *r = vec(N), *ig = vec(N), *a = vec(N), *m = vec(N);
  double *du = vec(N), *dh0 = vec(BD), *dWa = vec((size_t)nb * bs * bs), *dWx = vec((size_t)nb * bs * bs);
  double *dba = vec(D), *dbx = vec(D), *dlam = vec(D), *dcw = vec((size_t)K * D), *dcb = vec(D);
  unsigned char *reset = (unsigned char *)malloc((size_t)B * T ? (size_t)B * T : 1);
  for (size_t i = 0; i < (size_t)B * T; ++i) reset[i] = (unsigned char)(draw() > 0.4);
  const unsigned char *rs = with_reset ? reset : NULL;
  const double *o_cb = with_opt ? cb : NULL, *o_h0 = with_opt ? h0 : NULL, *o_st = with_opt ? st : NULL;

  oracle_conv1d(B, T, D, K, u, cw, o_cb, o_st, x, with_opt ? sto : NULL, rs);
  oracle_rglru(B, T, D, nb, 8.0, x, Wa, Wx, ba, bx, lam, o_h0, y, hT, with_opt ? r : NULL,
               with_opt ? ig : NULL, with_opt ? a : NULL, with_opt ? m : NULL, rs);
  oracle_forward(B, T, D, nb, K, 8.0, u, Wa, Wx, ba, bx, lam, cw, o_cb, o_h0, o_st, y, hT, sto, rs);
  if (T >= 1)
    oracle_backward(B, T, D, nb, K, 8.0, u, Wa, Wx, ba, bx, lam, cw, o_cb, o_h0, o_st, dy, with_opt ? dhT : NULL, du,
                    with_opt ? dh0 : NULL, dWa, dWx, dba, dbx, dlam, dcw, with_opt ? dcb : NULL, rs);
  for (size_t i = 0; i < N; ++i) a[i] = 0.5 + 0.49 * a[i];   /* decays in (0, 1) */
  oracle_scan(B, T, D, 0, 1, a, x, o_h0, y, hT);
  oracle_scan(B, T, D, 0, 0, a, x, o_h0, y, with_opt ? hT : NULL);
  oracle_scan_adjoint(B, T, D, 0, a, dy, with_opt ? dhT : NULL, du, with_opt ? dh0 : NULL);
  oracle_merge(N, with_opt, y, x, du);
  oracle_merge_backward(N, with_opt, y, x, dy, du, r);
  oracle_decode_step(B, D, nb, K, 8.0, u, Wa, Wx, ba, bx, lam, cw, o_cb, h0, st, hT);   /* u: first [B][D] only if T >= 1 */

  free(u); free(Wa); free(Wx); free(ba); free(bx); free(lam); free(cw); free(cb); free(h0); free(st);
  free(dy); free(dhT); free(x); free(y); free(hT); free(sto); free(r); free(ig); free(a); free(m);
  free(du); free(dh0); free(dWa); free(dWx); free(dba); free(dbx); free(dlam); free(dcw); free(dcb);
  free(reset);
}

int main(void) {
  const int shapes[][4] = {{1, 1, 4, 1}, {2, 7, 12, 3}, {3, 2, 8, 8}, {2, 33, 6, 2}, {1, 3, 5, 5}};
  for (int threads = 1; threads <= 3; threads += 2) {
    oracle_set_threads(threads);
    for (unsigned s = 0; s < sizeof(shapes) / sizeof(shapes[0]); ++s)
      for (int opt = 0; opt < 2; ++opt)
        for (int rs = 0; rs < 2; ++rs) one_case(shapes[s][0], shapes[s][1], shapes[s][2], shapes[s][3], opt, rs);
  }
  puts("ok");
  return 0;
}
