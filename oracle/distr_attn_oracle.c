/*
 * CPU oracle for DistrAttention (arXiv 2507.17245) -- TEST INFRASTRUCTURE ONLY.
 * See distr_attn_oracle.h for the contract. Nothing in the GPU library includes,
 * links or calls this file.
 *
 * The approximation is an algorithm, not a closed form, so the code below takes
 * the paper's steps in the paper's order:
 *   Sec. 3.2 "similar columns identification": project each column of the Q block
 *            onto N' random directions, keep the signs, map the sign word through
 *            the Gray table -> one integer per channel;
 *   Sec. 3.2 / Fig. 5: sort the integers, read off the index permutation, cut it
 *            into runs of G* -> groups;
 *   Sec. 3.2 "sampling" and "fusion": one Q column per group, the sum of the
 *            group's K columns;
 *   Eq. 2:   S^ = sum_j q^_j (sum_{i in G_j} k_i)^T;
 *   Sec. 3.3: all of the above once per Q block, the block's grouping applied to
 *            every key;
 *   Sec. 2.1: P = softmax(S^) row-wise, O = P V with the full V.
 * The mirrored form (Sec. 3.1 last sentence of the Eq. 2 paragraph, Fig. 4 right side,
 * Sec. 3.3 "(sum q_i) k^T"): the same steps with the roles of Q and K^T exchanged -- the
 * grouping comes from the channel columns of a K block, one K column per group is sampled and
 * the group's Q columns are summed.
 */
#include "distr_attn_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

static int n_keys_of(const oracle_params *p) { return p->Nk > 0 ? p->Nk : p->N; }

static int check_params(const oracle_params *p) {
  if (!p) return -1;
  if (p->B <= 0 || p->H <= 0 || p->Hkv <= 0 || p->N <= 0 || p->d <= 0 || p->Nk < 0) return -1;
  if (p->H % p->Hkv != 0) return -1;
  if (p->causal && n_keys_of(p) < p->N) return -1; /* the first queries would see no key */
  return 0;
}

static int check_distr_params(const oracle_params *p) {
  if (check_params(p)) return -1;
  if (p->Br <= 0 || p->n_groups <= 0 || p->d % p->n_groups != 0) return -1;
  if (p->d > 256) return -1; /* perm entries are bytes */
  if (p->n_planes < 1 || p->n_planes > 32) return -1;
  if (p->gray_mode != 0 && p->gray_mode != 1) return -1;
  if (p->side != 0 && p->side != 1) return -1;
  if (p->side == 1 && p->Bc <= 0) return -1;
  return 0;
}

/* ---- projection matrix ---------------------------------------------------
 * The paper only says the matrix is random and fixed in advance (Sec. 3.2).
 * Entry (p, r) is a function of (seed, p, r) alone: a 64-bit counter is mixed
 * (two multiply-xorshift rounds), its four 16-bit fields are summed and
 * centred. The result is an integer in [-131070, 131070] times 2^-16: a
 * symmetric, bell-shaped value in [-2, 2] that a float holds exactly.
 */
static uint64_t mix64(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
  return z ^ (z >> 31);
}

int oracle_hyperplanes(uint64_t seed, int n_planes, int Br, float *R) {
  if (!R || n_planes < 1 || n_planes > 32 || Br < 1) return -1;
  for (int p = 0; p < n_planes; ++p) {
    for (int r = 0; r < Br; ++r) {
      uint64_t counter = ((uint64_t)(uint32_t)p << 32) + (uint64_t)(uint32_t)r + 1u;
      uint64_t z = mix64(seed + 0x9E3779B97F4A7C15ULL * counter);
      long sum = (long)(z & 0xFFFF) + (long)((z >> 16) & 0xFFFF) + (long)((z >> 32) & 0xFFFF) +
                 (long)((z >> 48) & 0xFFFF);
      R[(size_t)p * Br + r] = (float)(sum - 2L * 65535L) / 65536.0f;
    }
  }
  return 0;
}

/* ---- Gray map -------------------------------------------------------------
 * mode 1: the sign word indexes the table of Gray codes, table[i] = i ^ (i >> 1).
 * mode 0: the sign word is read as a Gray codeword and the hash is its position
 *         in the Gray sequence (prefix xor from the top bit), so that hashes
 *         that differ by one belong to sign words that differ in one plane.
 */
uint32_t oracle_gray_hash(uint32_t code, int n_planes, int gray_mode) {
  (void)n_planes;
  if (gray_mode == 1) return code ^ (code >> 1);
  uint32_t rank = 0;
  for (uint32_t g = code; g; g >>= 1) rank ^= g;
  return rank;
}

/* Ascending, stable sort of channels by hash: ties keep ascending channel index.
 * perm[s] = channel at sorted position s (Fig. 5). */
static void sort_channels(const uint32_t *hash, int d, uint8_t *perm) {
  int idx[256];
  for (int c = 0; c < d; ++c) idx[c] = c;
  for (int i = 1; i < d; ++i) { /* insertion sort: stable */
    int ci = idx[i];
    int j = i - 1;
    while (j >= 0 && hash[idx[j]] > hash[ci]) {
      idx[j + 1] = idx[j];
      --j;
    }
    idx[j + 1] = ci;
  }
  for (int s = 0; s < d; ++s) perm[s] = (uint8_t)idx[s];
}

int oracle_sort_channels(const uint32_t *hash, int d, uint8_t *perm) {
  if (!hash || !perm || d < 1 || d > 256) return -1;
  sort_channels(hash, d, perm);
  return 0;
}

/* LSH of one Q block: rows r0 .. r0+rows-1 of one head (qh points at row 0 of the head). */
static void lsh_block(const float *qh, int d, int r0, int rows, const float *R, int Br,
                      int n_planes, int gray_mode, uint32_t *hash, uint8_t *perm, float *proj) {
  for (int c = 0; c < d; ++c) {
    uint32_t code = 0;
    for (int pl = 0; pl < n_planes; ++pl) {
      float acc = 0.0f;
      for (int r = 0; r < rows; ++r) /* float, fused, ascending rows: fixes the sign bit for bit */
        acc = fmaf(qh[(size_t)(r0 + r) * d + c], R[(size_t)pl * Br + r], acc);
      if (proj) proj[(size_t)c * n_planes + pl] = acc;
      uint32_t bit = (acc > 0.0f) ? 1u : 0u; /* positive -> 1, everything else -> 0 */
      code |= bit << (n_planes - 1 - pl);    /* plane 0 is the most significant bit */
    }
    hash[c] = oracle_gray_hash(code, n_planes, gray_mode);
  }
  sort_channels(hash, d, perm);
}

int oracle_lsh_group(const float *q, const oracle_params *p, const float *R, uint32_t *hash_out,
                     uint8_t *perm_out, float *proj_out) {
  if (!q || !R || check_distr_params(p)) return -1;
  const int Tq = (p->N + p->Br - 1) / p->Br;
  const long units = (long)p->B * p->H * Tq;
#pragma omp parallel for schedule(dynamic, 4)
  for (long u = 0; u < units; ++u) {
    int t = (int)(u % Tq);
    long bh = u / Tq;
    const float *qh = q + (size_t)bh * p->N * p->d;
    int r0 = t * p->Br;
    int rows = p->N - r0 < p->Br ? p->N - r0 : p->Br;
    uint32_t hash[256];
    uint8_t perm[256];
    lsh_block(qh, p->d, r0, rows, R, p->Br, p->n_planes, p->gray_mode, hash, perm,
              proj_out ? proj_out + (size_t)u * p->d * p->n_planes : NULL);
    if (hash_out) memcpy(hash_out + (size_t)u * p->d, hash, sizeof(uint32_t) * p->d);
    if (perm_out) memcpy(perm_out + (size_t)u * p->d, perm, p->d);
  }
  return 0;
}

/* softmax(s[0..n_vis-1]) . V  -> out[d]; two passes with the row maximum taken out. */
static void softmax_pv(double *s, int n_vis, const float *vh, int d, double *out) {
  double m = s[0];
  for (int n = 1; n < n_vis; ++n)
    if (s[n] > m) m = s[n];
  double denom = 0.0;
  for (int n = 0; n < n_vis; ++n) {
    s[n] = exp(s[n] - m);
    denom += s[n];
  }
  for (int c = 0; c < d; ++c) out[c] = 0.0;
  for (int n = 0; n < n_vis; ++n) {
    double pn = s[n] / denom;
    const float *vr = vh + (size_t)n * d;
    for (int c = 0; c < d; ++c) out[c] += pn * (double)vr[c];
  }
}

/* Exact attention for rows r0..r0+rows-1 of one head. */
static void exact_block(const float *qh, const float *kh, const float *vh, int Nk, int shift, int d,
                        int r0, int rows, int causal, double scale, double *o_rows, double *s) {
  for (int r = 0; r < rows; ++r) {
    int i = r0 + r;
    int n_vis = causal ? i + shift + 1 : Nk; /* shift = Nk - N: last query sees every key */
    const float *qi = qh + (size_t)i * d;
    for (int n = 0; n < n_vis; ++n) {
      const float *kn = kh + (size_t)n * d;
      double acc = 0.0;
      for (int c = 0; c < d; ++c) acc += (double)qi[c] * (double)kn[c];
      s[n] = scale * acc;
    }
    softmax_pv(s, n_vis, vh, d, o_rows + (size_t)r * d);
  }
}

/* Fusion (Sec. 3.2): kf[n][j] = sum over the members of group j of K[n][member], members
 * taken in sorted order. */
static void fuse_keys(const float *kh, int n_keys, int d, const uint8_t *perm, int n_groups,
                      double *kf) {
  const int G = d / n_groups;
  for (int n = 0; n < n_keys; ++n) {
    const float *kn = kh + (size_t)n * d;
    for (int j = 0; j < n_groups; ++j) {
      double acc = 0.0;
      for (int g = 0; g < G; ++g) acc += (double)kn[perm[j * G + g]];
      kf[(size_t)n * n_groups + j] = acc;
    }
  }
}

/* DistrAttention for one Q block given its permutation. kf and s are scratch. */
static void distr_block(const float *qh, const float *kh, const float *vh, int Nk, int shift, int d,
                        int r0, int rows, int causal, double scale, const uint8_t *perm,
                        int n_groups, double *o_rows, double *kf, double *s) {
  const int G = d / n_groups;
  int n_keys = causal ? r0 + rows + shift : Nk; /* keys any row of the block can see */
  fuse_keys(kh, n_keys, d, perm, n_groups, kf);
  for (int r = 0; r < rows; ++r) {
    int i = r0 + r;
    int n_vis = causal ? i + shift + 1 : Nk;
    const float *qi = qh + (size_t)i * d;
    for (int n = 0; n < n_vis; ++n) {
      const double *kfn = kf + (size_t)n * n_groups;
      double acc = 0.0;
      for (int j = 0; j < n_groups; ++j) /* sampling: the group's first column in sorted order */
        acc += (double)qi[perm[j * G]] * kfn[j];
      s[n] = scale * acc;
    }
    softmax_pv(s, n_vis, vh, d, o_rows + (size_t)r * d);
  }
}

/* The mirrored form for one Q block: for every K block (Bc rows) its own grouping
 * perm_k[tb] (from that K block's channel columns); S^[i][n] = scale * sum_j
 * (sum_{g} Q[i][member g of group j]) * K[n][first member of group j]  for n in block tb.
 * qf is scratch of n_groups doubles. */
static void distr_block_kside(const float *qh, const float *kh, const float *vh, int Nk, int shift,
                              int d, int r0, int rows, int causal, double scale,
                              const uint8_t *perm_k, int Bc, int n_groups, double *o_rows,
                              double *qf, double *s) {
  const int G = d / n_groups;
  for (int r = 0; r < rows; ++r) {
    int i = r0 + r;
    int n_vis = causal ? i + shift + 1 : Nk;
    const float *qi = qh + (size_t)i * d;
    for (int n0 = 0; n0 < n_vis; n0 += Bc) {
      const uint8_t *perm = perm_k + (size_t)(n0 / Bc) * d;
      for (int j = 0; j < n_groups; ++j) { /* fusion of the query's channels, in sorted order */
        double acc = 0.0;
        for (int g = 0; g < G; ++g) acc += (double)qi[perm[j * G + g]];
        qf[j] = acc;
      }
      int n1 = n0 + Bc < n_vis ? n0 + Bc : n_vis;
      for (int n = n0; n < n1; ++n) {
        const float *kn = kh + (size_t)n * d;
        double acc = 0.0;
        for (int j = 0; j < n_groups; ++j) /* sampling: the group's first K column in sorted order */
          acc += qf[j] * (double)kn[perm[j * G]];
        s[n] = scale * acc;
      }
    }
    softmax_pv(s, n_vis, vh, d, o_rows + (size_t)r * d);
  }
}

/* Groupings of every K block of one kv head: perm_k[tb][d]. */
static void lsh_key_blocks(const float *kh, int Nk, int d, const float *R, int Bc, int n_planes,
                           int gray_mode, uint8_t *perm_k) {
  for (int n0 = 0; n0 < Nk; n0 += Bc) {
    uint32_t hash[256];
    int rows = Nk - n0 < Bc ? Nk - n0 : Bc;
    lsh_block(kh, d, n0, rows, R, Bc, n_planes, gray_mode, hash, perm_k + (size_t)(n0 / Bc) * d, NULL);
  }
}

static int run_tiles(const float *q, const float *k, const float *v, double *o,
                     const oracle_params *p, const float *R, const uint8_t *perm_in,
                     const int *tiles, long n_units, int distr, int packed_out) {
  if (!q || !k || !v || !o) return -1;
  if (distr ? check_distr_params(p) : check_params(p)) return -1;
  if (!distr && p->Br <= 0 && tiles) return -1;
  const int N = p->N, d = p->d, Nk = n_keys_of(p), shift = Nk - N;
  const int Br = (p->Br > 0) ? p->Br : N;
  const int Tq = (N + Br - 1) / Br;
  const int rep = p->H / p->Hkv;
  const int kside = distr && p->side == 1;
  const int Tk = kside ? (Nk + p->Bc - 1) / p->Bc : 0;
  const int lsh_rows = kside ? p->Bc : Br; /* rows of the blocks the LSH runs on */
  float *Rown = NULL;
  if (distr && !perm_in && !R) {
    Rown = (float *)malloc(sizeof(float) * (size_t)p->n_planes * lsh_rows);
    if (!Rown) return -2;
    oracle_hyperplanes(p->lsh_seed, p->n_planes, lsh_rows, Rown);
    R = Rown;
  }
  if (tiles) {
    for (long u = 0; u < n_units; ++u) {
      if (tiles[3 * u] < 0 || tiles[3 * u] >= p->B || tiles[3 * u + 1] < 0 ||
          tiles[3 * u + 1] >= p->H || tiles[3 * u + 2] < 0 || tiles[3 * u + 2] >= Tq) {
        free(Rown);
        return -1;
      }
    }
  }
  int failed = 0;
#pragma omp parallel
  {
    double *s = (double *)malloc(sizeof(double) * (size_t)Nk);
    double *kf = (distr && !kside) ? (double *)malloc(sizeof(double) * (size_t)Nk * p->n_groups) : NULL;
    double *qf = kside ? (double *)malloc(sizeof(double) * (size_t)p->n_groups) : NULL;
    uint8_t *perm_k = kside ? (uint8_t *)malloc((size_t)Tk * d) : NULL;
    if (!s || (distr && !kside && !kf) || (kside && (!qf || !perm_k))) {
#pragma omp atomic write
      failed = 1;
    }
#pragma omp barrier
    if (!failed) {
#pragma omp for schedule(dynamic, 1)
      for (long u = 0; u < n_units; ++u) {
        int b, h, t;
        if (tiles) {
          b = tiles[3 * u];
          h = tiles[3 * u + 1];
          t = tiles[3 * u + 2];
        } else {
          t = (int)(u % Tq);
          h = (int)((u / Tq) % p->H);
          b = (int)(u / ((long)Tq * p->H));
        }
        const float *qh = q + ((size_t)b * p->H + h) * N * d;
        const float *kh = k + ((size_t)b * p->Hkv + h / rep) * Nk * d;
        const float *vh = v + ((size_t)b * p->Hkv + h / rep) * Nk * d;
        int r0 = t * Br;
        int rows = N - r0 < Br ? N - r0 : Br;
        double *o_rows = packed_out ? o + (size_t)u * Br * d
                                    : o + (((size_t)b * p->H + h) * N + r0) * d;
        if (!distr) {
          exact_block(qh, kh, vh, Nk, shift, d, r0, rows, p->causal, p->scale, o_rows, s);
        } else if (kside) {
          const uint8_t *pk = perm_k;
          if (perm_in) pk = perm_in + ((size_t)b * p->Hkv + h / rep) * Tk * d;
          else lsh_key_blocks(kh, Nk, d, R, p->Bc, p->n_planes, p->gray_mode, perm_k);
          distr_block_kside(qh, kh, vh, Nk, shift, d, r0, rows, p->causal, p->scale, pk, p->Bc,
                            p->n_groups, o_rows, qf, s);
        } else {
          uint8_t perm[256];
          size_t unit = ((size_t)b * p->H + h) * Tq + t;
          if (perm_in) {
            memcpy(perm, perm_in + unit * d, d);
          } else {
            uint32_t hash[256];
            lsh_block(qh, d, r0, rows, R, Br, p->n_planes, p->gray_mode, hash, perm, NULL);
          }
          distr_block(qh, kh, vh, Nk, shift, d, r0, rows, p->causal, p->scale, perm, p->n_groups,
                      o_rows, kf, s);
        }
      }
    }
    free(s);
    free(kf);
    free(qf);
    free(perm_k);
  }
  free(Rown);
  return failed ? -2 : 0;
}

int oracle_exact_fwd(const float *q, const float *k, const float *v, double *o,
                     const oracle_params *p) {
  if (check_params(p)) return -1;
  const int Br = (p->Br > 0) ? p->Br : p->N;
  const int Tq = (p->N + Br - 1) / Br;
  return run_tiles(q, k, v, o, p, NULL, NULL, NULL, (long)p->B * p->H * Tq, 0, 0);
}

int oracle_distr_fwd(const float *q, const float *k, const float *v, double *o,
                     const oracle_params *p, const float *R, const uint8_t *perm) {
  if (check_distr_params(p)) return -1;
  const int Tq = (p->N + p->Br - 1) / p->Br;
  return run_tiles(q, k, v, o, p, R, perm, NULL, (long)p->B * p->H * Tq, 1, 0);
}

int oracle_exact_fwd_tiles(const float *q, const float *k, const float *v, double *o_tiles,
                           const oracle_params *p, const int *tiles, int n_tiles) {
  if (!tiles || n_tiles < 0 || check_params(p) || p->Br <= 0) return -1;
  return run_tiles(q, k, v, o_tiles, p, NULL, NULL, tiles, n_tiles, 0, 1);
}

int oracle_distr_fwd_tiles(const float *q, const float *k, const float *v, double *o_tiles,
                           const oracle_params *p, const float *R, const uint8_t *perm,
                           const int *tiles, int n_tiles) {
  if (!tiles || n_tiles < 0 || check_distr_params(p)) return -1;
  return run_tiles(q, k, v, o_tiles, p, R, perm, tiles, n_tiles, 1, 1);
}

int oracle_scores(const float *q, const float *k, double *s_hat, double *s,
                  const oracle_params *p, const float *R, const uint8_t *perm_in, int b, int h) {
  if (!q || !k || check_distr_params(p)) return -1;
  if (b < 0 || b >= p->B || h < 0 || h >= p->H) return -1;
  const int N = p->N, d = p->d, Br = p->Br, G = d / p->n_groups, Nk = n_keys_of(p);
  const int Tq = (N + Br - 1) / Br;
  const int rep = p->H / p->Hkv;
  const int kside = p->side == 1;
  const int lsh_rows = kside ? p->Bc : Br;
  const float *qh = q + ((size_t)b * p->H + h) * N * d;
  const float *kh = k + ((size_t)b * p->Hkv + h / rep) * Nk * d;
  float *Rown = NULL;
  if (s_hat && !perm_in && !R) {
    Rown = (float *)malloc(sizeof(float) * (size_t)p->n_planes * lsh_rows);
    if (!Rown) return -2;
    oracle_hyperplanes(p->lsh_seed, p->n_planes, lsh_rows, Rown);
    R = Rown;
  }
  if (s) {
    for (int i = 0; i < N; ++i)
      for (int n = 0; n < Nk; ++n) {
        double acc = 0.0;
        for (int c = 0; c < d; ++c) acc += (double)qh[(size_t)i * d + c] * (double)kh[(size_t)n * d + c];
        s[(size_t)i * Nk + n] = p->scale * acc;
      }
  }
  if (s_hat && kside) {
    const int Tk = (Nk + p->Bc - 1) / p->Bc;
    uint8_t *perm_k = (uint8_t *)malloc((size_t)Tk * d);
    if (!perm_k) {
      free(Rown);
      return -2;
    }
    if (perm_in) memcpy(perm_k, perm_in + ((size_t)b * p->Hkv + h / rep) * Tk * d, (size_t)Tk * d);
    else lsh_key_blocks(kh, Nk, d, R, p->Bc, p->n_planes, p->gray_mode, perm_k);
    for (int i = 0; i < N; ++i)
      for (int n = 0; n < Nk; ++n) {
        const uint8_t *perm = perm_k + (size_t)(n / p->Bc) * d;
        double acc = 0.0;
        for (int j = 0; j < p->n_groups; ++j) {
          double qsum = 0.0;
          for (int g = 0; g < G; ++g) qsum += (double)qh[(size_t)i * d + perm[j * G + g]];
          acc += qsum * (double)kh[(size_t)n * d + perm[j * G]];
        }
        s_hat[(size_t)i * Nk + n] = p->scale * acc;
      }
    free(perm_k);
  } else if (s_hat) {
    double *kf = (double *)malloc(sizeof(double) * (size_t)Nk * p->n_groups);
    if (!kf) {
      free(Rown);
      return -2;
    }
    for (int t = 0; t < Tq; ++t) {
      int r0 = t * Br;
      int rows = N - r0 < Br ? N - r0 : Br;
      uint8_t perm[256];
      if (perm_in) {
        memcpy(perm, perm_in + (((size_t)b * p->H + h) * Tq + t) * d, d);
      } else {
        uint32_t hash[256];
        lsh_block(qh, d, r0, rows, R, Br, p->n_planes, p->gray_mode, hash, perm, NULL);
      }
      fuse_keys(kh, Nk, d, perm, p->n_groups, kf);
      for (int r = 0; r < rows; ++r) {
        int i = r0 + r;
        for (int n = 0; n < Nk; ++n) {
          double acc = 0.0;
          for (int j = 0; j < p->n_groups; ++j)
            acc += (double)qh[(size_t)i * d + perm[j * G]] * kf[(size_t)n * p->n_groups + j];
          s_hat[(size_t)i * Nk + n] = p->scale * acc;
        }
      }
    }
    free(kf);
  }
  free(Rown);
  return 0;
}
