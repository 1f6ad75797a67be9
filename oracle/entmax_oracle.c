/*
 * entmax_oracle.c -- fp64 CPU oracle for alpha-entmax / ASEntmax attention.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
 * GPU library is checked against.  It shares no code with the HIP path, and
 * nothing in the product path may call it.  Only the tests, the smoke check
 * and the benchmark's cpu_baseline leg load it.
 *
 * What it follows (paper sections / equations, stated in our own words):
 *   - Sec. 2.1: causal attention head, logits z_ij = <q_i,k_j>/sqrt(d),
 *     weights p_ij = pi(z_i)_j over the visible keys j <= i, output
 *     u_i = sum_j p_ij v_j (the norm and residual are the caller's).
 *   - Sec. 2.2 eq. (entmax) and App. A: p_j = [(alpha-1) z_j - tau]_+^(1/(alpha-1))
 *     with tau fixed by sum_j p_j = 1; entries with (alpha-1) z_j <= tau are
 *     exactly zero.
 *   - App. A ("alpha-entmax computation"): order-based exact solutions exist
 *     for alpha = 2 and alpha = 1.5; the support is found here by sorting.
 *   - Sec. 4.1 eq. (asentmax): logits are multiplied by delta + beta (log n)^gamma
 *     before entmax; beta, gamma per head (or per query), natural logarithm.
 *   - Sec. 4.2, App. B and the ALiBi definition of the positional-encoding appendix:
 *     an optional per-head linear distance bias b_ij = m_h (j - i) for keys at or
 *     before the query's position (0 for later keys), added to the logit
 *     z_ij = <q_i,k_j>/sqrt(d).  A slope of 0 is NoPE; NAPE is a slope array in which
 *     half of the heads have slope 0.  The paper writes the bias as part of z, which
 *     eq. (asentmax) then multiplies by the scale (bias_mode 0); the other reading adds
 *     the bias after the scale (bias_mode 1).  Slopes are fixed numbers: no gradient.
 *   - The backward is the exact derivative of eq. (entmax): on the support
 *     p^(alpha-1) = (alpha-1) s - tau, hence dp = g (ds - dtau/(alpha-1)) with
 *     g = p^(2-alpha); sum_j dp_j = 0 gives dtau/(alpha-1) = sum g ds / sum g.
 *
 * No blocking, fusion or reordering: every row is handled on its own, in the
 * order the definition states.  Every function is pinned by tests that do not
 * go through this file's own formulas (closed forms from the paper, brute
 * force over supports, finite differences, the sparsemax and softmax limits).
 *
 * Layout: all tensors contiguous fp64, Q [B,H,Nq,D], K and V [B,H,Nk,D].
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
  int32_t B, H, Nq, Nk, D;
  int32_t causal;       /* 1: key j visible to query i iff j <= i + (Nk - Nq) */
  int32_t scale_layout; /* 0: scale = delta; 1: beta,gamma [H]; 2: beta,gamma [B,H,Nq] */
  int32_t logn_mode;    /* 0: n = Nk for every row; 1: n = number of visible keys of the row */
  int32_t bias_mode;    /* with slopes: 0: s = scale (z + b); 1: s = scale z + b */
  double alpha;         /* 1 < alpha <= 2 */
  double delta;
} oracle_params;

static int cmp_desc(const void* a, const void* b) {
  double x = *(const double*)a, y = *(const double*)b;
  return (x < y) - (x > y);
}

/* t^r for t >= 0, r = 1/(alpha-1); plain products where r is a small integer. */
static double pow_r(double t, double alpha) {
  if (t <= 0.0) return 0.0;
  if (alpha == 2.0) return t;
  if (alpha == 1.5) return t * t;
  return pow(t, 1.0 / (alpha - 1.0));
}

/* F_k = sum_{j<k} [(alpha-1)(s_(j) - s_(k))]^r on the descending-sorted scores
 * (k is 1-based).  Element k belongs to the support iff F_k < 1: F_k is the
 * total mass the larger elements would carry if the threshold sat exactly at
 * element k, and the mass is decreasing in the threshold. */
static double mass_above(const double* sorted, int k, double alpha) {
  double acc = 0.0;
  double sk = sorted[k - 1];
  for (int j = 0; j < k - 1; ++j) acc += pow_r((alpha - 1.0) * (sorted[j] - sk), alpha);
  return acc;
}

/*
 * Exact alpha-entmax of one score vector (eq. (entmax)).
 * s[n] scores, p[n] probabilities out, *tau threshold out (the convention of
 * eq. (entmax): p = [(alpha-1)s - tau]_+^r), *support = number of non-zeros.
 * force_generic != 0 skips the alpha = 1.5 / 2 closed forms and solves the
 * fixed-support equation by bisection (used to cross-check the closed forms).
 */
void oracle_entmax_row(const double* s, int n, double alpha, int force_generic, double* p, double* tau,
                       int* support) {
  double* sorted = (double*)malloc(sizeof(double) * (size_t)n);
  memcpy(sorted, s, sizeof(double) * (size_t)n);
  qsort(sorted, (size_t)n, sizeof(double), cmp_desc);

  /* F_k is non-decreasing in k (each term grows and one term is added when
   * s_(k) drops), F_1 = 0, so the support is a prefix 1..k*: binary search for
   * the last k with F_k < 1. */
  int lo = 1, hi = n;
  while (lo < hi) {
    int mid = lo + (hi - lo + 1) / 2;
    if (mass_above(sorted, mid, alpha) < 1.0)
      lo = mid;
    else
      hi = mid - 1;
  }
  int k = lo;

  double t;
  double a1 = alpha - 1.0;
  if (alpha == 2.0 && !force_generic) {
    double sum = 0.0;
    for (int j = 0; j < k; ++j) sum += sorted[j];
    t = (sum - 1.0) / k;
  } else if (alpha == 1.5 && !force_generic) {
    double mean = 0.0;
    for (int j = 0; j < k; ++j) mean += 0.5 * sorted[j];
    mean /= k;
    double ss = 0.0;
    for (int j = 0; j < k; ++j) {
      double dlt = 0.5 * sorted[j] - mean;
      ss += dlt * dlt;
    }
    double rad = (1.0 - ss) / k;
    if (rad < 0.0) rad = 0.0;
    t = mean - sqrt(rad);
  } else {
    /* On the fixed support, f(t) = sum_{j<=k} (a1 s_(j) - t)^r - 1 is smooth
     * and strictly decreasing between the two ends below; f >= 0 at the left
     * end, f < 0 at the right end. */
    double left = a1 * sorted[0] - 1.0;
    if (k < n && a1 * sorted[k] > left) left = a1 * sorted[k];
    double right = a1 * sorted[k - 1];
    for (int it = 0; it < 200; ++it) {
      double mid = 0.5 * (left + right);
      double f = -1.0;
      for (int j = 0; j < k; ++j) f += pow_r(a1 * sorted[j] - mid, alpha);
      if (f >= 0.0)
        left = mid;
      else
        right = mid;
    }
    t = 0.5 * (left + right);
  }
  int cnt = 0;
  for (int j = 0; j < n; ++j) {
    p[j] = pow_r(a1 * s[j] - t, alpha);
    cnt += (p[j] > 0.0);
  }
  *tau = t;
  if (support) *support = cnt;
  free(sorted);
}

/* Number of keys query row i may attend to, and whether key j is one of them. */
static int visible_count(const oracle_params* P, int i) {
  if (!P->causal) return P->Nk;
  int c = i + (P->Nk - P->Nq) + 1;
  if (c < 0) c = 0;
  if (c > P->Nk) c = P->Nk;
  return c;
}

/* ASEntmax multiplier delta + beta * (ln n)^gamma of eq. (asentmax) for one
 * row; also returns L^gamma and ln L (needed by the parameter gradients).
 * A row whose n is 1 has ln n = 0: the multiplier is defined as delta there
 * and the parameter gradients as zero. */
static double row_scale(const oracle_params* P, const double* beta, const double* gamma, int b, int h, int i,
                        double* Lg_out, double* lnL_out, double* beta_out) {
  double Lg = 0.0, lnL = 0.0, bt = 0.0;
  double scale = P->delta;
  if (P->scale_layout != 0) {
    size_t idx = (P->scale_layout == 1) ? (size_t)h : ((size_t)b * P->H + h) * P->Nq + i;
    bt = beta[idx];
    double gm = gamma[idx];
    int n = (P->logn_mode == 0) ? P->Nk : visible_count(P, i);
    if (n > 1) {
      double L = log((double)n);
      Lg = pow(L, gm);
      lnL = log(L);
      scale = P->delta + bt * Lg;
    }
  }
  if (Lg_out) *Lg_out = Lg;
  if (lnL_out) *lnL_out = lnL;
  if (beta_out) *beta_out = bt;
  return scale;
}

/* ALiBi bias of key j for query row i of head h: -m_h * distance, where the query sits at position
 * i + (Nk - Nq) of the key sequence and keys after it get no bias. */
static double alibi_bias(const oracle_params* P, const double* slopes, int h, int i, int j) {
  if (!slopes) return 0.0;
  int dist = i + (P->Nk - P->Nq) - j;
  if (dist < 0) dist = 0;
  return -slopes[h] * (double)dist;
}

/* Entmax input s_ij from the logit z_ij, the row's scale and the positional bias. */
static double scaled_logit(const oracle_params* P, double scale, double z, double b) {
  return P->bias_mode == 0 ? scale * (z + b) : scale * z + b;
}

static double dot(const double* a, const double* b, int d) {
  double acc = 0.0;
  for (int t = 0; t < d; ++t) acc += a[t] * b[t];
  return acc;
}

/*
 * Forward (Sec. 2.1 with pi = alpha-entmax, logits scaled per eq. (asentmax)).
 * O [B,H,Nq,D], tau [B,H,Nq], support [B,H,Nq] (may be NULL),
 * Pfull [B,H,Nq,Nk] (may be NULL; zero on masked keys).
 * A row with no visible key gets O = 0, tau = 0, support = 0.
 */
int oracle_attn_fwd(const oracle_params* P, const double* Q, const double* K, const double* V, const double* beta,
                    const double* gamma, const double* slopes, double* O, double* tau, int32_t* support,
                    double* Pfull) {
  const int B = P->B, H = P->H, Nq = P->Nq, Nk = P->Nk, D = P->D;
  const double inv_sqrt_d = 1.0 / sqrt((double)D);
  const long rows = (long)B * H * Nq;
#pragma omp parallel
  {
    double* s = (double*)malloc(sizeof(double) * (size_t)Nk);
    double* p = (double*)malloc(sizeof(double) * (size_t)Nk);
#pragma omp for schedule(dynamic, 16)
    for (long row = 0; row < rows; ++row) {
      int i = (int)(row % Nq);
      int h = (int)((row / Nq) % H);
      int b = (int)(row / ((long)Nq * H));
      const double* q = Q + (size_t)row * D;
      const double* Kh = K + ((size_t)b * H + h) * (size_t)Nk * D;
      const double* Vh = V + ((size_t)b * H + h) * (size_t)Nk * D;
      double* o = O + (size_t)row * D;
      for (int t = 0; t < D; ++t) o[t] = 0.0;
      if (Pfull)
        for (int j = 0; j < Nk; ++j) Pfull[(size_t)row * Nk + j] = 0.0;
      int nv = visible_count(P, i);
      if (nv == 0) {
        tau[row] = 0.0;
        if (support) support[row] = 0;
        continue;
      }
      double scale = row_scale(P, beta, gamma, b, h, i, NULL, NULL, NULL);
      for (int j = 0; j < nv; ++j)
        s[j] = scaled_logit(P, scale, dot(q, Kh + (size_t)j * D, D) * inv_sqrt_d, alibi_bias(P, slopes, h, i, j));
      double t;
      int cnt;
      oracle_entmax_row(s, nv, P->alpha, 0, p, &t, &cnt);
      tau[row] = t;
      if (support) support[row] = cnt;
      for (int j = 0; j < nv; ++j) {
        if (p[j] > 0.0)
          for (int c = 0; c < D; ++c) o[c] += p[j] * Vh[(size_t)j * D + c];
        if (Pfull) Pfull[(size_t)row * Nk + j] = p[j];
      }
    }
    free(s);
    free(p);
  }
  return 0;
}

/*
 * Backward.  Given dO, recomputes each row's exact probabilities and applies
 *   g_j  = p_j^(2-alpha) on the support, 0 off it,
 *   dP_j = <dO_i, v_j>,  mu = sum g dP / sum g,  dS_j = g_j (dP_j - mu),
 *   dV_j += p_j dO_i,  dQ_i = (scale/sqrt d) sum_j dS_j k_j,
 *   dK_j += (scale/sqrt d) dS_j q_i,  dscale_i = sum_j dS_j ds_j/dscale  (= z_j, or z_j + b_j when the
 *   positional bias sits inside the scaled logit),
 *   dbeta = dscale L^gamma,  dgamma = dscale beta L^gamma ln L   (L = ln n),
 * the last two summed over (batch, row) for the per-head layout.
 * dQ,dK,dV as Q,K,V; dbeta,dgamma in beta/gamma's layout (ignored when the
 * layout is 0; may be NULL then); dscale [B,H,Nq] may be NULL.
 */
int oracle_attn_bwd(const oracle_params* P, const double* Q, const double* K, const double* V, const double* beta,
                    const double* gamma, const double* slopes, const double* dO, double* dQ, double* dK, double* dV,
                    double* dbeta, double* dgamma, double* dscale) {
  const int B = P->B, H = P->H, Nq = P->Nq, Nk = P->Nk, D = P->D;
  const double inv_sqrt_d = 1.0 / sqrt((double)D);
  const double alpha = P->alpha;
  memset(dK, 0, sizeof(double) * (size_t)B * H * Nk * D);
  memset(dV, 0, sizeof(double) * (size_t)B * H * Nk * D);
  memset(dQ, 0, sizeof(double) * (size_t)B * H * Nq * D);
  double* dbeta_bh = NULL;
  double* dgamma_bh = NULL;
  if (P->scale_layout == 1) {
    dbeta_bh = (double*)calloc((size_t)B * H, sizeof(double));
    dgamma_bh = (double*)calloc((size_t)B * H, sizeof(double));
  }
#pragma omp parallel
  {
    double* z = (double*)malloc(sizeof(double) * (size_t)Nk);
    double* s = (double*)malloc(sizeof(double) * (size_t)Nk);
    double* p = (double*)malloc(sizeof(double) * (size_t)Nk);
#pragma omp for schedule(dynamic, 1)
    for (int bh = 0; bh < B * H; ++bh) {
      int b = bh / H, h = bh % H;
      const double* Kh = K + (size_t)bh * Nk * D;
      const double* Vh = V + (size_t)bh * Nk * D;
      double* dKh = dK + (size_t)bh * Nk * D;
      double* dVh = dV + (size_t)bh * Nk * D;
      for (int i = 0; i < Nq; ++i) {
        size_t row = (size_t)bh * Nq + i;
        const double* q = Q + row * D;
        const double* go = dO + row * D;
        double* dq = dQ + row * D;
        if (dscale) dscale[row] = 0.0;
        int nv = visible_count(P, i);
        if (nv == 0) continue;
        double Lg, lnL, bt;
        double scale = row_scale(P, beta, gamma, b, h, i, &Lg, &lnL, &bt);
        for (int j = 0; j < nv; ++j) {
          double bj = alibi_bias(P, slopes, h, i, j);
          double zj = dot(q, Kh + (size_t)j * D, D) * inv_sqrt_d;
          s[j] = scaled_logit(P, scale, zj, bj);
          z[j] = P->bias_mode == 0 ? zj + bj : zj; /* d s_j / d scale */
        }
        double t;
        oracle_entmax_row(s, nv, alpha, 0, p, &t, NULL);
        double sum_g = 0.0, sum_gdp = 0.0;
        for (int j = 0; j < nv; ++j) {
          if (p[j] > 0.0) {
            double g = pow(p[j], 2.0 - alpha);
            double dp = dot(go, Vh + (size_t)j * D, D);
            sum_g += g;
            sum_gdp += g * dp;
          }
        }
        double mu = sum_gdp / sum_g;
        double dsc = 0.0;
        for (int j = 0; j < nv; ++j) {
          if (p[j] > 0.0) {
            double g = pow(p[j], 2.0 - alpha);
            double dp = dot(go, Vh + (size_t)j * D, D);
            double ds = g * (dp - mu);
            dsc += ds * z[j];
            for (int c = 0; c < D; ++c) {
              dVh[(size_t)j * D + c] += p[j] * go[c];
              dq[c] += scale * inv_sqrt_d * ds * Kh[(size_t)j * D + c];
              dKh[(size_t)j * D + c] += scale * inv_sqrt_d * ds * q[c];
            }
          }
        }
        if (dscale) dscale[row] = dsc;
        if (P->scale_layout == 1) {
          dbeta_bh[bh] += dsc * Lg;
          dgamma_bh[bh] += dsc * bt * Lg * lnL;
        } else if (P->scale_layout == 2) {
          dbeta[row] = dsc * Lg;
          dgamma[row] = dsc * bt * Lg * lnL;
        }
      }
    }
    free(z);
    free(s);
    free(p);
  }
  if (P->scale_layout == 1) {
    for (int h = 0; h < H; ++h) {
      dbeta[h] = 0.0;
      dgamma[h] = 0.0;
      for (int b = 0; b < B; ++b) {
        dbeta[h] += dbeta_bh[b * H + h];
        dgamma[h] += dgamma_bh[b * H + h];
      }
    }
    free(dbeta_bh);
    free(dgamma_bh);
  }
  return 0;
}

/*
 * Block sparsity of the exact attention matrix: map[b,h,ti,tj] = 1 iff some
 * p_ij > 0 with i in query tile ti (tq rows) and j in key tile tj (tk keys).
 * visible[b,h,ti,tj] = 1 iff the tile holds at least one unmasked (i,j) pair.
 * Both arrays are [B,H,ceil(Nq/tq),ceil(Nk/tk)] bytes.
 */
int oracle_tile_map(const oracle_params* P, const double* Q, const double* K, const double* beta,
                    const double* gamma, const double* slopes, int tq, int tk, uint8_t* map, uint8_t* visible) {
  const int B = P->B, H = P->H, Nq = P->Nq, Nk = P->Nk, D = P->D;
  const int nti = (Nq + tq - 1) / tq, ntj = (Nk + tk - 1) / tk;
  const double inv_sqrt_d = 1.0 / sqrt((double)D);
  memset(map, 0, (size_t)B * H * nti * ntj);
  memset(visible, 0, (size_t)B * H * nti * ntj);
  const long rows = (long)B * H * Nq;
#pragma omp parallel
  {
    double* s = (double*)malloc(sizeof(double) * (size_t)Nk);
    double* p = (double*)malloc(sizeof(double) * (size_t)Nk);
    /* static chunks of tq rows: one thread owns all rows of a query tile */
#pragma omp for schedule(dynamic, 1)
    for (long tile = 0; tile < (long)B * H * nti; ++tile) {
      long bh = tile / nti;
      int ti = (int)(tile % nti);
      int b = (int)(bh / H), h = (int)(bh % H);
      const double* Kh = K + (size_t)bh * Nk * D;
      for (int i = ti * tq; i < (ti + 1) * tq && i < Nq; ++i) {
        long row = bh * Nq + i;
        const double* q = Q + (size_t)row * D;
        int nv = visible_count(P, i);
        if (nv == 0) continue;
        double scale = row_scale(P, beta, gamma, b, h, i, NULL, NULL, NULL);
        for (int j = 0; j < nv; ++j)
          s[j] = scaled_logit(P, scale, dot(q, Kh + (size_t)j * D, D) * inv_sqrt_d, alibi_bias(P, slopes, h, i, j));
        double t;
        oracle_entmax_row(s, nv, P->alpha, 0, p, &t, NULL);
        for (int j = 0; j < nv; ++j) {
          size_t m = ((size_t)tile) * ntj + j / tk;
          visible[m] = 1;
          if (p[j] > 0.0) map[m] = 1;
        }
      }
    }
    free(s);
    free(p);
  }
  (void)rows;
  return 0;
}

/* ---------------------------------------------------------------------------
 * ASEntmax scale projections (Sec. 4.1, the two equations after eq. (asentmax)): for every token x_t of
 * X [B,N,E] and every head h with projection vectors w_beta,h, w_gamma,h (rows of Wb, Wg [H,E]),
 *     beta[b,h,i]  = softplus(<x_{b,i}, w_beta,h>)  = ln(1 + e^u)
 *     gamma[b,h,i] = s * tanh(<x_{b,i}, w_gamma,h>)
 * written in the per-query layout [B,H,N] the attention takes.  The paper gives no value for s: an argument.
 * ------------------------------------------------------------------------- */
int oracle_scale_proj_fwd(int B, int H, int N, int E, double s, const double* X, const double* Wb, const double* Wg,
                          double* beta, double* gamma) {
  for (int b = 0; b < B; ++b)
    for (int h = 0; h < H; ++h)
      for (int i = 0; i < N; ++i) {
        const double* x = X + ((size_t)b * N + i) * E;
        double u = dot(x, Wb + (size_t)h * E, E), v = dot(x, Wg + (size_t)h * E, E);
        /* ln(1 + e^u) without overflow: max(u, 0) + ln(1 + e^-|u|) */
        beta[((size_t)b * H + h) * N + i] = (u > 0 ? u : 0) + log1p(exp(-fabs(u)));
        gamma[((size_t)b * H + h) * N + i] = s * tanh(v);
      }
  return 0;
}

/* Chain rule through the projections: with u = <x, w_beta>, v = <x, w_gamma>,
 *     d beta / du = e^u / (1 + e^u),   d gamma / dv = s (1 - tanh^2 v),
 * dWb[h] = sum_{b,i} dbeta du/.. x_{b,i},  dWg[h] likewise,  dX[b,i] = sum_h (du w_beta,h + dv w_gamma,h). */
int oracle_scale_proj_bwd(int B, int H, int N, int E, double s, const double* X, const double* Wb, const double* Wg,
                          const double* dbeta, const double* dgamma, double* dX, double* dWb, double* dWg) {
  for (size_t k = 0; k < (size_t)B * N * E; ++k) dX[k] = 0.0;
  for (size_t k = 0; k < (size_t)H * E; ++k) dWb[k] = dWg[k] = 0.0;
  for (int b = 0; b < B; ++b)
    for (int h = 0; h < H; ++h)
      for (int i = 0; i < N; ++i) {
        const double* x = X + ((size_t)b * N + i) * E;
        double* dx = dX + ((size_t)b * N + i) * E;
        const double* wb = Wb + (size_t)h * E;
        const double* wg = Wg + (size_t)h * E;
        double u = dot(x, wb, E), v = dot(x, wg, E);
        double sig = u >= 0 ? 1.0 / (1.0 + exp(-u)) : exp(u) / (1.0 + exp(u));
        double th = tanh(v);
        double du = dbeta[((size_t)b * H + h) * N + i] * sig;
        double dv = dgamma[((size_t)b * H + h) * N + i] * s * (1.0 - th * th);
        for (int k = 0; k < E; ++k) {
          dWb[(size_t)h * E + k] += du * x[k];
          dWg[(size_t)h * E + k] += dv * x[k];
          dx[k] += du * wb[k] + dv * wg[k];
        }
      }
  return 0;
}

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}
