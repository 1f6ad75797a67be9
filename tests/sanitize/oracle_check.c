/* Runs the fp64 oracle (oracle/entmax_oracle.c, compiled into this program with
 * -fsanitize=address,undefined) over small shapes that exercise every branch: the three
 * scale layouts, both log-n modes, causal and not, Nq != Nk, rows without keys, the
 * closed-form and the generic threshold solvers.  Prints "ok" on success. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

typedef struct {
  int32_t B, H, Nq, Nk, D;
  int32_t causal, scale_layout, logn_mode, bias_mode;
  double alpha, delta;
} oracle_params;

void oracle_entmax_row(const double*, int, double, int, double*, double*, int*);
int oracle_attn_fwd(const oracle_params*, const double*, const double*, const double*, const double*, const double*,
                    const double*, double*, double*, int32_t*, double*);
int oracle_attn_bwd(const oracle_params*, const double*, const double*, const double*, const double*, const double*,
                    const double*, const double*, double*, double*, double*, double*, double*, double*);
int oracle_tile_map(const oracle_params*, const double*, const double*, const double*, const double*, const double*,
                    int, int, uint8_t*, uint8_t*);

static uint64_t state = 88172645463325252ull;
static double rnd(void) { /* xorshift in [-1, 1) */
  state ^= state << 13;
  state ^= state >> 7;
  state ^= state << 17;
  return (double)(state >> 11) / 4503599627370496.0 - 1.0;
}
static double* fill(size_t n, double scale) {
  double* a = (double*)malloc(sizeof(double) * (n ? n : 1));
  for (size_t i = 0; i < n; ++i) a[i] = scale * rnd();
  return a;
}

int main(void) {
  const double alphas[] = {1.25, 1.5, 2.0, 1.7};
  int runs = 0;
  for (int ai = 0; ai < 4; ++ai)
    for (int layout = 0; layout <= 2; ++layout)
      for (int causal = 0; causal <= 1; ++causal)
        for (int shape = 0; shape < 4; ++shape) {
          oracle_params P;
          P.B = 2; P.H = 2; P.D = 8;
          P.Nq = shape == 0 ? 9 : shape == 1 ? 5 : shape == 2 ? 13 : 1;
          P.Nk = shape == 0 ? 9 : shape == 1 ? 12 : shape == 2 ? 6 : 1;
          P.causal = causal; P.scale_layout = layout; P.logn_mode = (ai + shape) & 1;
          P.alpha = alphas[ai]; P.delta = layout == 0 ? 1.0 : 0.5;
          P.bias_mode = (ai + layout) & 1;
          double slopes_buf[2] = {0.25, 0.0};
          const double* slopes = (shape + causal) & 1 ? slopes_buf : NULL; /* with and without the positional bias */
          size_t nq = (size_t)P.B * P.H * P.Nq, nk = (size_t)P.B * P.H * P.Nk;
          double *Q = fill(nq * P.D, 2.0), *K = fill(nk * P.D, 2.0), *V = fill(nk * P.D, 1.0), *dO = fill(nq * P.D, 1.0);
          size_t ns = layout == 1 ? (size_t)P.H : nq;
          double *beta = fill(ns, 1.0), *gamma = fill(ns, 1.0);
          double *O = fill(nq * P.D, 0.0), *tau = fill(nq, 0.0), *Pf = fill(nq * P.Nk, 0.0);
          int32_t* sup = (int32_t*)malloc(sizeof(int32_t) * nq);
          oracle_attn_fwd(&P, Q, K, V, layout ? beta : NULL, layout ? gamma : NULL, slopes, O, tau, sup, Pf);
          for (size_t r = 0; r < nq; ++r) {
            double s = 0.0;
            for (int j = 0; j < P.Nk; ++j) s += Pf[r * P.Nk + j];
            if (sup[r] > 0 && fabs(s - 1.0) > 1e-9) { fprintf(stderr, "row %zu sums to %g\n", r, s); return 1; }
          }
          double *dQ = fill(nq * P.D, 0.0), *dK = fill(nk * P.D, 0.0), *dV = fill(nk * P.D, 0.0);
          double *db = fill(ns, 0.0), *dg = fill(ns, 0.0), *dsc = fill(nq, 0.0);
          oracle_attn_bwd(&P, Q, K, V, layout ? beta : NULL, layout ? gamma : NULL, slopes, dO, dQ, dK, dV, layout ? db : NULL,
                          layout ? dg : NULL, dsc);
          int nti = (P.Nq + 3) / 4, ntj = (P.Nk + 3) / 4;
          uint8_t* map = (uint8_t*)malloc((size_t)P.B * P.H * nti * ntj + 1);
          uint8_t* vis = (uint8_t*)malloc((size_t)P.B * P.H * nti * ntj + 1);
          oracle_tile_map(&P, Q, K, layout ? beta : NULL, layout ? gamma : NULL, slopes, 4, 4, map, vis);
          free(Q); free(K); free(V); free(dO); free(beta); free(gamma); free(O); free(tau); free(Pf); free(sup);
          free(dQ); free(dK); free(dV); free(db); free(dg); free(dsc); free(map); free(vis);
          ++runs;
        }
  /* the row routine on its own, generic solver forced, ties and a single element included */
  double s[7] = {0.3, 0.3, -1.0, 2.0, 2.0, 2.0, -5.0}, p[7], t;
  int k;
  for (int n = 1; n <= 7; ++n)
    for (int ai = 0; ai < 4; ++ai)
      for (int fg = 0; fg <= 1; ++fg) oracle_entmax_row(s, n, alphas[ai], fg, p, &t, &k);
  printf("ok %d\n", runs);
  return 0;
}
