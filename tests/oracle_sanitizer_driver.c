/* Calls every entry point of the CPU oracle on small ragged problems; built with
 * -fsanitize=address,undefined by tests/test_oracle_sanitized.py, which fails on any report. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "distr_attn_oracle.h"

static float *filled(size_t n, int mul, int mod, float scale) {
  float *x = (float *)malloc(sizeof(float) * n);
  for (size_t i = 0; i < n; ++i) x[i] = (float)((int)((i * (size_t)mul) % (size_t)mod) - mod / 2) * scale;
  return x;
}

static int run(oracle_params p) {
  const int Nk = p.Nk > 0 ? p.Nk : p.N;
  const size_t nq = (size_t)p.B * p.H * p.N * p.d, nk = (size_t)p.B * p.Hkv * Nk * p.d;
  const int Tq = (p.N + p.Br - 1) / p.Br, Tk = (Nk + p.Bc - 1) / p.Bc;
  float *q = filled(nq, 37, 11, 0.25f), *k = filled(nk, 13, 7, 0.5f), *v = filled(nk, 5, 9, 0.125f);
  float *dout = filled(nq, 3, 13, 0.1f);
  double *o = (double *)malloc(sizeof(double) * nq), *dq = (double *)malloc(sizeof(double) * nq);
  double *dk = (double *)malloc(sizeof(double) * nk), *dv = (double *)malloc(sizeof(double) * nk);
  double *lse = (double *)malloc(sizeof(double) * (size_t)p.B * p.H * p.N);
  double *s1 = (double *)malloc(sizeof(double) * (size_t)p.N * Nk), *s2 = (double *)malloc(sizeof(double) * (size_t)p.N * Nk);
  const size_t n_tab = p.side == 1 ? (size_t)p.B * p.Hkv * Tk * p.d : (size_t)p.B * p.H * Tq * p.d;
  uint8_t *perm = (uint8_t *)malloc(n_tab);
  uint32_t *hash = (uint32_t *)malloc(sizeof(uint32_t) * n_tab);
  float *R = (float *)malloc(sizeof(float) * (size_t)p.n_planes * (p.side == 1 ? p.Bc : p.Br));
  int rc = 0;
  rc |= oracle_hyperplanes(p.lsh_seed, p.n_planes, p.side == 1 ? p.Bc : p.Br, R);
  rc |= oracle_exact_fwd(q, k, v, o, &p);
  rc |= oracle_distr_fwd(q, k, v, o, &p, NULL, NULL);
  rc |= oracle_distr_fwd(q, k, v, o, &p, R, NULL);
  rc |= oracle_scores(q, k, s1, s2, &p, NULL, NULL, p.B - 1, p.H - 1);
  if (p.side == 0) {
    rc |= oracle_lsh_group(q, &p, R, hash, perm, NULL);
    rc |= oracle_sort_channels(hash, p.d, perm);
    rc |= oracle_lsh_group(q, &p, R, NULL, perm, NULL);
    rc |= oracle_distr_fwd(q, k, v, o, &p, NULL, perm);
    int tiles[6] = {0, 0, 0, p.B - 1, p.H - 1, Tq - 1};
    double *ot = (double *)malloc(sizeof(double) * 2 * (size_t)p.Br * p.d);
    rc |= oracle_exact_fwd_tiles(q, k, v, ot, &p, tiles, 2);
    rc |= oracle_distr_fwd_tiles(q, k, v, ot, &p, NULL, NULL, tiles, 2);
    free(ot);
    rc |= oracle_lse(q, k, lse, &p, NULL, NULL, 1);
    rc |= oracle_lse(q, k, lse, &p, NULL, NULL, 0);
    rc |= oracle_distr_bwd(q, k, v, dout, dq, dk, dv, &p, NULL, NULL);
    rc |= oracle_distr_bwd(q, k, v, dout, dq, dk, dv, &p, NULL, perm);
    rc |= oracle_exact_bwd(q, k, v, dout, dq, dk, dv, &p);
  }
  printf("B%d H%d Hkv%d N%d Nk%d d%d Br%d Bc%d k%d causal%d side%d: rc %d, o[0] %.6g, dq[last] %.6g\n", p.B, p.H, p.Hkv,
         p.N, Nk, p.d, p.Br, p.Bc, p.n_groups, p.causal, p.side, rc, o[0], p.side == 0 ? dq[nq - 1] : 0.0);
  free(q); free(k); free(v); free(dout); free(o); free(dq); free(dk); free(dv); free(lse); free(s1); free(s2);
  free(perm); free(hash); free(R);
  return rc;
}

int main(void) {
  int rc = 0;
  /*                    B  H Hkv  N   d  Br  k causal planes gray seed scale  Nk side Bc */
  rc |= run((oracle_params){1, 2, 1, 37, 16, 8, 4, 1, 8, 0, 3, 0.25, 45, 0, 8});
  rc |= run((oracle_params){2, 4, 2, 21, 32, 16, 8, 0, 16, 1, 0, 0.2, 0, 0, 8});
  rc |= run((oracle_params){1, 3, 3, 1, 8, 4, 8, 1, 1, 0, 9, 1.0, 5, 0, 4});       /* one query, groups of one channel */
  rc |= run((oracle_params){1, 2, 2, 19, 16, 8, 2, 0, 32, 0, 1, 0.5, 7, 0, 8});     /* fewer keys than queries, 32 planes */
  rc |= run((oracle_params){1, 2, 1, 26, 16, 8, 4, 1, 4, 0, 5, 0.25, 33, 1, 8});    /* mirrored form */
  rc |= run((oracle_params){2, 2, 2, 10, 8, 16, 1, 0, 2, 1, 2, 0.3, 0, 1, 4});      /* mirrored, one group */
  return rc != 0;
}
