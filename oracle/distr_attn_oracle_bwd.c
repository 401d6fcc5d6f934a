/*
 * CPU oracle, backward pass -- TEST INFRASTRUCTURE ONLY (see distr_attn_oracle.h).
 *
 * The paper trains through the approximation (Sec. 4.3, 4.4) without giving the gradient. The
 * reading implemented here: the gradient of what the forward computes with the grouping held
 * fixed. The permutation of a Q block is a piecewise-constant function of Q (sign bits of
 * Sec. 3.2), so almost everywhere the forward of a block is the smooth map
 *     O = softmax(scale * Q_r K_f^T) V,   Q_r[:, j] = Q[:, first member of group j],
 *                                          K_f[:, j] = sum of K's columns in group j   (Eq. 2)
 * and the chain rule gives, with P = softmax(S^), dP = dO V^T, D_i = sum_c dO_ic O_ic and
 * dS^ = P o (dP - D):
 *     dV = P^T dO
 *     dQ[:, first member of group j] = scale * (dS^ K_f)[:, j],  every other column of the block 0
 *     dK[:, c] = scale * sum over Q blocks of (dS^T Q_r)[:, group of c in that block]
 * Exact attention (Sec. 2.1) is the case of one column per group.
 * Plain two-pass arithmetic in double, no tiling. Shares no code with the GPU library.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include "distr_attn_oracle.h"

static int keys_of(const oracle_params *p) { return p->Nk > 0 ? p->Nk : p->N; }

static int bwd_params_ok(const oracle_params *p, int distr) {
  if (!p || p->B <= 0 || p->H <= 0 || p->Hkv <= 0 || p->N <= 0 || p->d <= 0 || p->d > 256) return 0;
  if (p->H % p->Hkv != 0) return 0;
  if (p->causal && keys_of(p) < p->N) return 0;
  if (distr) {
    if (p->side != 0) return 0; /* the mirrored form has no backward here */
    if (p->Br <= 0 || p->n_groups <= 0 || p->d % p->n_groups != 0) return 0;
  }
  return 1;
}

/* Scores of query row qi against keys 0..n_vis-1 through the grouping (perm == NULL: exact). */
static void score_row(const float *qi, const float *kh, int n_vis, int d, const uint8_t *perm,
                      int n_groups, double scale, double *s) {
  const int G = perm ? d / n_groups : 1;
  for (int n = 0; n < n_vis; ++n) {
    const float *kn = kh + (size_t)n * d;
    double acc = 0.0;
    if (!perm) {
      for (int c = 0; c < d; ++c) acc += (double)qi[c] * (double)kn[c];
    } else {
      for (int j = 0; j < n_groups; ++j) {
        double kf = 0.0;
        for (int g = 0; g < G; ++g) kf += (double)kn[perm[j * G + g]];
        acc += (double)qi[perm[j * G]] * kf;
      }
    }
    s[n] = scale * acc;
  }
}

static int grouping_table(const float *q, const oracle_params *p, const float *R,
                          const uint8_t *perm_in, uint8_t **owned, const uint8_t **table) {
  *owned = NULL;
  if (perm_in) {
    *table = perm_in;
    return 0;
  }
  const int Tq = (p->N + p->Br - 1) / p->Br;
  uint8_t *t = (uint8_t *)malloc((size_t)p->B * p->H * Tq * p->d);
  if (!t) return -2;
  float *Rown = NULL;
  if (!R) {
    Rown = (float *)malloc(sizeof(float) * (size_t)p->n_planes * p->Br);
    if (!Rown) {
      free(t);
      return -2;
    }
    oracle_hyperplanes(p->lsh_seed, p->n_planes, p->Br, Rown);
    R = Rown;
  }
  int rc = oracle_lsh_group(q, p, R, NULL, t, NULL);
  free(Rown);
  if (rc) {
    free(t);
    return rc;
  }
  *owned = t;
  *table = t;
  return 0;
}

int oracle_lse(const float *q, const float *k, double *lse, const oracle_params *p, const float *R,
               const uint8_t *perm_in, int distr) {
  if (!q || !k || !lse || !bwd_params_ok(p, distr)) return -1;
  const int N = p->N, d = p->d, Nk = keys_of(p), shift = Nk - N, rep = p->H / p->Hkv;
  const int Br = distr ? p->Br : N, Tq = (N + Br - 1) / Br;
  uint8_t *owned = NULL;
  const uint8_t *table = NULL;
  if (distr) {
    int rc = grouping_table(q, p, R, perm_in, &owned, &table);
    if (rc) return rc;
  }
  int failed = 0;
#pragma omp parallel
  {
    double *s = (double *)malloc(sizeof(double) * (size_t)Nk);
    if (!s) {
#pragma omp atomic write
      failed = 1;
    }
#pragma omp barrier
    if (!failed) {
#pragma omp for schedule(dynamic, 1)
      for (long bh = 0; bh < (long)p->B * p->H; ++bh) {
        const int b = (int)(bh / p->H), h = (int)(bh % p->H);
        const float *qh = q + (size_t)bh * N * d;
        const float *kh = k + ((size_t)b * p->Hkv + h / rep) * Nk * d;
        for (int i = 0; i < N; ++i) {
          const uint8_t *perm = distr ? table + ((size_t)bh * Tq + i / Br) * d : NULL;
          const int n_vis = p->causal ? i + shift + 1 : Nk;
          score_row(qh + (size_t)i * d, kh, n_vis, d, perm, p->n_groups, p->scale, s);
          double m = s[0];
          for (int n = 1; n < n_vis; ++n)
            if (s[n] > m) m = s[n];
          double sum = 0.0;
          for (int n = 0; n < n_vis; ++n) sum += exp(s[n] - m);
          lse[(size_t)bh * N + i] = m + log(sum);
        }
      }
    }
    free(s);
  }
  free(owned);
  return failed ? -2 : 0;
}

static int run_bwd(const float *q, const float *k, const float *v, const float *dout, double *dq,
                   double *dk, double *dv, const oracle_params *p, const float *R,
                   const uint8_t *perm_in, int distr) {
  if (!q || !k || !v || !dout || !dq || !dk || !dv || !bwd_params_ok(p, distr)) return -1;
  const int N = p->N, d = p->d, Nk = keys_of(p), shift = Nk - N, rep = p->H / p->Hkv;
  const int Br = distr ? p->Br : N, Tq = (N + Br - 1) / Br;
  const int ng = distr ? p->n_groups : d, G = d / ng;
  uint8_t *owned = NULL;
  const uint8_t *table = NULL;
  if (distr) {
    int rc = grouping_table(q, p, R, perm_in, &owned, &table);
    if (rc) return rc;
  }
  int failed = 0;
#pragma omp parallel
  {
    double *s = (double *)malloc(sizeof(double) * (size_t)Nk);         /* scores, then probabilities */
    double *kf = (double *)malloc(sizeof(double) * (size_t)Nk * ng);   /* fused keys of the block */
    double *dkf = (double *)malloc(sizeof(double) * (size_t)Nk * ng);  /* their gradient */
    double *o = (double *)malloc(sizeof(double) * (size_t)d);
    double *dqr = (double *)malloc(sizeof(double) * (size_t)ng);
    if (!s || !kf || !dkf || !o || !dqr) {
#pragma omp atomic write
      failed = 1;
    }
#pragma omp barrier
    if (!failed) {
      /* one kv head at a time per thread: its dK and dV collect from rep query heads */
#pragma omp for schedule(dynamic, 1)
      for (long bk = 0; bk < (long)p->B * p->Hkv; ++bk) {
        const int b = (int)(bk / p->Hkv), hk = (int)(bk % p->Hkv);
        const float *kh = k + (size_t)bk * Nk * d;
        const float *vh = v + (size_t)bk * Nk * d;
        double *dkh = dk + (size_t)bk * Nk * d;
        double *dvh = dv + (size_t)bk * Nk * d;
        memset(dkh, 0, sizeof(double) * (size_t)Nk * d);
        memset(dvh, 0, sizeof(double) * (size_t)Nk * d);
        for (int h = hk * rep; h < (hk + 1) * rep; ++h) {
          const size_t bh = (size_t)b * p->H + h;
          const float *qh = q + bh * N * d;
          const float *doh = dout + bh * N * d;
          double *dqh = dq + bh * N * d;
          for (int t = 0; t < Tq; ++t) {
            const int r0 = t * Br, rows = N - r0 < Br ? N - r0 : Br;
            uint8_t perm[256];
            if (distr) memcpy(perm, table + (bh * Tq + t) * d, d);
            else
              for (int c = 0; c < d; ++c) perm[c] = (uint8_t)c;
            const int n_keys = p->causal ? r0 + rows + shift : Nk;
            for (int n = 0; n < n_keys; ++n)
              for (int j = 0; j < ng; ++j) {
                double acc = 0.0;
                for (int g = 0; g < G; ++g) acc += (double)kh[(size_t)n * d + perm[j * G + g]];
                kf[(size_t)n * ng + j] = acc;
                dkf[(size_t)n * ng + j] = 0.0;
              }
            for (int r = 0; r < rows; ++r) {
              const int i = r0 + r;
              const int n_vis = p->causal ? i + shift + 1 : Nk;
              const float *qi = qh + (size_t)i * d;
              const float *doi = doh + (size_t)i * d;
              double m = -INFINITY, denom = 0.0;
              for (int n = 0; n < n_vis; ++n) {
                double acc = 0.0;
                for (int j = 0; j < ng; ++j) acc += (double)qi[perm[j * G]] * kf[(size_t)n * ng + j];
                s[n] = p->scale * acc;
                if (s[n] > m) m = s[n];
              }
              for (int n = 0; n < n_vis; ++n) {
                s[n] = exp(s[n] - m);
                denom += s[n];
              }
              for (int c = 0; c < d; ++c) o[c] = 0.0;
              for (int n = 0; n < n_vis; ++n) {
                s[n] /= denom; /* P[i][n] */
                for (int c = 0; c < d; ++c) o[c] += s[n] * (double)vh[(size_t)n * d + c];
              }
              double D = 0.0;
              for (int c = 0; c < d; ++c) D += (double)doi[c] * o[c];
              for (int j = 0; j < ng; ++j) dqr[j] = 0.0;
              for (int n = 0; n < n_vis; ++n) {
                double dp = 0.0;
                for (int c = 0; c < d; ++c) {
                  dp += (double)doi[c] * (double)vh[(size_t)n * d + c];
                  dvh[(size_t)n * d + c] += s[n] * (double)doi[c];
                }
                const double ds = s[n] * (dp - D);
                for (int j = 0; j < ng; ++j) {
                  dqr[j] += ds * kf[(size_t)n * ng + j];
                  dkf[(size_t)n * ng + j] += ds * (double)qi[perm[j * G]];
                }
              }
              for (int c = 0; c < d; ++c) dqh[(size_t)i * d + c] = 0.0;
              for (int j = 0; j < ng; ++j) dqh[(size_t)i * d + perm[j * G]] = p->scale * dqr[j];
            }
            /* every member of a group receives the gradient of the group's fused column */
            for (int n = 0; n < n_keys; ++n)
              for (int j = 0; j < ng; ++j)
                for (int g = 0; g < G; ++g)
                  dkh[(size_t)n * d + perm[j * G + g]] += p->scale * dkf[(size_t)n * ng + j];
          }
        }
      }
    }
    free(s);
    free(kf);
    free(dkf);
    free(o);
    free(dqr);
  }
  free(owned);
  return failed ? -2 : 0;
}

int oracle_exact_bwd(const float *q, const float *k, const float *v, const float *dout, double *dq,
                     double *dk, double *dv, const oracle_params *p) {
  return run_bwd(q, k, v, dout, dq, dk, dv, p, NULL, NULL, 0);
}

int oracle_distr_bwd(const float *q, const float *k, const float *v, const float *dout, double *dq,
                     double *dk, double *dv, const oracle_params *p, const float *R,
                     const uint8_t *perm) {
  return run_bwd(q, k, v, dout, dq, dk, dv, p, R, perm, 1);
}
