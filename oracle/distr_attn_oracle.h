/*
 * CPU oracle for DistrAttention (arXiv 2507.17245) -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, fp64 implementation of
 *   - exact attention, S = QK^T -> softmax -> PV                       (Sec. 2.1)
 *   - the DistrAttention approximation: LSH over the channel columns of
 *     each Q block, sort, fixed-size groups, sample one Q column per
 *     group, sum the group's K columns, S^ = Q_r K_f^T                 (Sec. 3.1 Eq. 2,
 *     Sec. 3.2, Sec. 3.3)
 * It shares no code with the GPU library and is only called from the
 * tests, the smoke check and the benchmark's cpu_baseline leg.
 *
 * All pointers are host pointers. q and o are [B][H][N][d], k and v are
 * [B][Hkv][Nk][d] (Nk = N unless oracle_params.Nk says otherwise), contiguous, d fastest. Inputs are float (bf16 workloads
 * pass bf16-representable floats), every dot product, sum and softmax is
 * taken in double, outputs are double. The one exception is the LSH
 * projection, whose sign decides an integer: it is taken in float with one
 * fused multiply-add per row in ascending row order, the precision and
 * order the GPU kernel uses, so the group tables can be compared bit by bit.
 *
 * Every function returns 0 on success and a negative value on bad arguments.
 */
#ifndef DISTR_ATTN_ORACLE_H
#define DISTR_ATTN_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
  int B, H, Hkv, N, d;
  int Br;         /* rows of a Q block (the paper's l): one grouping per block (Sec. 3.3) */
  int n_groups;   /* k = d / G*                                            (Sec. 3.2)  */
  int causal;     /* key n visible to query i iff n <= i */
  int n_planes;   /* the paper's N' (16 in Sec. 3.2), 1..32 */
  int gray_mode;  /* 0: hash = rank of the sign word read as a Gray codeword; 1: hash = sign word Gray-encoded */
  uint64_t lsh_seed;
  double scale;   /* multiplies S before softmax */
  int Nk;         /* number of keys / values per head; 0 means N. With causal != 0 (needs Nk >= N)
                     the last query is aligned with the last key: key n is visible to query i
                     iff n <= i + (Nk - N) */
  int side;       /* 0: sample Q columns, fuse K columns, one grouping per Q block of Br rows
                        (the form the paper builds, Sec. 3.2-3.3);
                     1: the mirrored form of Sec. 3.1 / Fig. 4 right: sample K columns, fuse Q
                        columns, one grouping per K block of Bc rows, taken from that K block */
  int Bc;         /* rows of a K block; only side 1 depends on it */
} oracle_params;

/* Projection matrix R[n_planes][Br] from the seed (counter-based, exactly representable floats). */
int oracle_hyperplanes(uint64_t seed, int n_planes, int Br, float *R);

/* Gray map of one sign word. */
uint32_t oracle_gray_hash(uint32_t code, int n_planes, int gray_mode);

/* Ascending stable sort of d hashes (ties keep ascending channel index): perm[s] = channel at
 * sorted position s (Fig. 5). */
int oracle_sort_channels(const uint32_t *hash, int d, uint8_t *perm);

/* LSH grouping of every Q block with an explicit projection matrix R[n_planes][Br].
 * hash_out, perm_out: [B][H][Tq][d], Tq = ceil(N/Br); either may be NULL.
 * proj_out (may be NULL): [B][H][Tq][d][n_planes] float projections. */
int oracle_lsh_group(const float *q, const oracle_params *p, const float *R,
                     uint32_t *hash_out, uint8_t *perm_out, float *proj_out);

/* Exact attention, all rows. */
int oracle_exact_fwd(const float *q, const float *k, const float *v, double *o,
                     const oracle_params *p);

/* DistrAttention, all rows. R may be NULL (then it comes from p->lsh_seed).
 * perm (may be NULL) overrides the LSH grouping: [B][H][Tq][d] (side 1: [B][Hkv][Tk][d], and R is
 * [n_planes][Bc]). */
int oracle_distr_fwd(const float *q, const float *k, const float *v, double *o,
                     const oracle_params *p, const float *R, const uint8_t *perm);

/* The same two, restricted to a list of Q blocks: tiles[3*i+0..2] = (b, h, t).
 * o_tiles is [n_tiles][Br][d]; rows past N in a ragged block are left untouched. */
int oracle_exact_fwd_tiles(const float *q, const float *k, const float *v, double *o_tiles,
                           const oracle_params *p, const int *tiles, int n_tiles);
int oracle_distr_fwd_tiles(const float *q, const float *k, const float *v, double *o_tiles,
                           const oracle_params *p, const float *R, const uint8_t *perm,
                           const int *tiles, int n_tiles);

/* Unnormalised score blocks for one (b, h): s_hat and s are [N][Nk] doubles
 * (scale applied, no mask). Either may be NULL. For side 1, R is [n_planes][Bc] and perm is the
 * table of the K blocks, [B][Hkv][ceil(Nk/Bc)][d]. */
int oracle_scores(const float *q, const float *k, double *s_hat, double *s,
                  const oracle_params *p, const float *R, const uint8_t *perm, int b, int h);

/* Row statistics of the forward: lse[b][h][i] = log of the sum over the visible keys of
 * exp(score), scores = S^ (distr != 0; R and perm as for oracle_distr_fwd) or S (distr == 0).
 * lse is [B][H][N]. Side 0 only. */
int oracle_lse(const float *q, const float *k, double *lse, const oracle_params *p, const float *R,
               const uint8_t *perm, int distr);

/* Backward pass (distr_attn_oracle_bwd.c): gradients of sum(dout * O) with respect to q, k, v.
 * The paper gives no gradient (Sec. 4.3-4.4 only train through the method); this is the
 * derivative of the forward with every Q block's grouping held fixed: only the sampled Q columns
 * of a block receive a gradient, every member of a K group receives its group's. dout is
 * [B][H][N][d]; dq [B][H][N][d], dk and dv [B][Hkv][Nk][d] are overwritten. Side 0 only. */
int oracle_exact_bwd(const float *q, const float *k, const float *v, const float *dout, double *dq,
                     double *dk, double *dv, const oracle_params *p);
int oracle_distr_bwd(const float *q, const float *k, const float *v, const float *dout, double *dq,
                     double *dk, double *dv, const oracle_params *p, const float *R,
                     const uint8_t *perm);

/* Threads the parallel loops will use. */
int oracle_num_threads(void);

#ifdef __cplusplus
}
#endif
#endif
