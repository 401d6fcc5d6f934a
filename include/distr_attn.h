/*
 * distr_attn -- DistrAttention block-wise attention forward pass for AMD MI355X (gfx950).
 *
 * C ABI of libdistr_attn.so. Method: "DistrAttention: An Efficient and Flexible
 * Self-Attention Mechanism on Modern GPUs" (arXiv 2507.17245), cited below by section.
 *
 * Conventions for every entry point
 *   - q, k, v, o and every pointer named *_out / workspace are DEVICE pointers owned by the
 *     caller; `const da_params*` and `float* host_out` are HOST pointers.
 *   - Layout: q and o are [B][H][N][d]; k and v are [B][Hkv][Nk][d] (Nk = N unless da_params.Nk
 *     says otherwise); contiguous, d fastest. Query head h reads key/value head h / (H / Hkv).
 *     Element type is bf16 or float (da_dtype).
 *   - q, k, v are never written. o must not alias an input. Base pointers must be 16-byte aligned.
 *   - Calls only enqueue work on the stream (asynchronous); they never synchronise the device
 *     (distr_attn_release does). Debugging aid: with DISTR_ATTN_DEBUG=1 in the environment when the
 *     library is first called, every launch is followed by a device synchronisation and a fault is
 *     reported by the call that caused it, naming the launch (launches into a stream under capture are not waited for).
 *   - Return value: DA_OK or a negative da_status. All argument checks run on the host before
 *     anything is launched; on error nothing has been enqueued. distr_attn_last_error() gives a
 *     message for the last failure on the calling thread.
 *   - Notation: Tq = ceil(N / Br) query blocks; Tk = ceil(Nk / Bc) key blocks; G* = d / n_groups
 *     channels per group.
 */
#ifndef DISTR_ATTN_H
#define DISTR_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  DA_OK = 0,
  DA_ERR_INVALID_ARG = -1, /* null pointer, non-positive size, H % Hkv != 0, d % n_groups != 0, misaligned */
  DA_ERR_UNSUPPORTED = -2, /* valid for the method, outside what the kernels are built for */
  DA_ERR_WORKSPACE = -3,   /* caller workspace too small, or the library could not allocate its own */
  DA_ERR_HIP = -4          /* a HIP runtime call failed */
} da_status;

typedef enum { DA_BF16 = 0, DA_F32 = 1 } da_dtype;

/*
 * Full parameter block (host memory).
 *
 * Supported by the kernels: d in {64, 128}; Br in {64, 128, 256}; Bc in {32, 64, 128}; for bf16
 * n_groups in {4, 8, 16, 32, 64, 128} with G* = d / n_groups <= 16 (4 and 8 zero-pad the contraction
 * to one MFMA step of 16, and need Bc = 64), for float any divisor of d; 1 <= n_planes <= 32;
 * N, Nk >= 1 arbitrary (ragged last blocks are masked), N * d * 4 and Nk * d * 4 < 2^31; at most
 * 2^31 - 1 query blocks.
 * bf16 DistrAttention path: the reduced product S^ = Q_r K_f^T runs in half precision on
 * Q_r * softmax_scale * log2(e) and on K. Full precision needs magnitudes inside half's normal
 * range: |q| * softmax_scale * log2(e) beyond 65504 and |k| beyond 65504 / G* are clamped; below
 * 2^-14 (6.1e-5) values keep fewer significand bits (absolute step 2^-24) and below 2^-25 they
 * become 0. The exact path and the float path have no such limit.
 */
typedef struct {
  int B, H, Hkv, N, d;
  int Br;               /* rows of a query block, the paper's l; one LSH grouping per block (Sec. 3.3) */
  int Bc;               /* rows of a key/value block, the paper's m (Sec. 2.2.2)                     */
  int n_groups;         /* k = d / G*: contraction length of S^ = Q_r K_f^T (Sec. 3.1 Eq. 2, Sec. 3.2) */
  int causal;           /* 0 / 1: key n is visible to query i iff n <= i                            */
  uint64_t lsh_seed;    /* seed of the random projection matrix (Sec. 3.2)                          */
  int dtype;            /* da_dtype of q, k, v, o                                                   */
  int n_planes;         /* number of projections N' (Sec. 3.2 uses 16); 0 means 16                  */
  float softmax_scale;  /* multiplies S before softmax; 0 means 1/sqrt(d)                           */
  int gray_mode;        /* Gray map of the sign word (Sec. 3.2): 0 = position of the word in the Gray
                           sequence, 1 = Gray code of the word                                     */
  void *stream;         /* hipStream_t; NULL = the stream set by distr_attn_set_stream (default: null stream) */
  void *workspace;      /* device scratch of >= distr_attn_workspace_bytes(), 256-byte aligned; NULL =
                           library-owned, one per device, grown on demand (hipMalloc on first use /
                           growth; outgrown buffers are kept until distr_attn_release; growing
                           while the stream is being captured into a graph is refused). Calls that
                           may overlap in time on different streams must each bring their own
                           workspace. Only what the call writes is needed: no K^T part with kt_in,
                           no table with perm_in / perm_out or when the attention kernel does the
                           LSH stage itself.                                                        */
  size_t workspace_bytes;
  uint8_t *perm_out;    /* optional device [B][H][Tq][d]: channel at sorted position s of each block */
  uint32_t *hash_out;   /* optional device [B][H][Tq][d]: hash of each channel of each block          */
  const uint8_t *perm_in; /* optional device [B][H][Tq][d]: use this grouping and skip the LSH stage
                             (each row must be a permutation of 0..d-1; it is not checked)          */
  const void *kt_in;      /* optional device buffer written by distr_attn_key_prepass for this k and
                             n_groups: skip the key pre-pass (bf16 only)                            */
  int Nk;               /* keys / values per head; 0 means N. N != Nk covers decoding against a cache
                           and cross attention (Sec. 2.1 with an N x Nk score matrix). With causal = 1
                           (needs Nk >= N) the last query is aligned with the last key: key n is
                           visible to query i iff n <= i + (Nk - N)                                */
  int side;             /* 0: sample Q columns, fuse K columns, one grouping per Q block (Sec. 3.2-3.3,
                           the form the paper builds). 1: the mirrored form of Sec. 3.1 / Fig. 4 right:
                           sample K columns, fuse Q columns, one grouping per K block of Bc rows taken
                           from that K block; Bc in {32, 64, 128}; float arithmetic on the vector ALUs
                           for both dtypes (bf16 tensors are converted on load); perm_in / perm_out /
                           hash_out are then [B][Hkv][Tk][d]                                        */
  float *lse_out;       /* optional device [B][H][N] float: natural logarithm of the sum over the visible
                           keys of exp(score) of every query row -- the row statistics of the softmax
                           (Sec. 2.2.2), which a backward pass needs; scores are S^ for the
                           DistrAttention calls and S for the exact ones. side = 0 only              */
} da_params;

/*
 * DistrAttention forward (Sec. 3.1-3.3): per query block, hash the d channel columns with
 * random-projection LSH, sort the hashes, cut the sorted order into groups of G*, take the first
 * channel of each group from Q and the sum of the group's channels from K, S^ = Q_r K_f^T, then
 * online softmax and P V over the full V. bf16, 16 projections, scale 1/sqrt(d), current stream.
 */
int distr_attn_fwd(const void *q, const void *k, const void *v, void *o, int B, int H, int Hkv,
                   int N, int d, int Br, int Bc, int n_groups, uint64_t lsh_seed, int causal);

/* Exact attention forward, O = softmax(scale * Q K^T) V (Sec. 2.1), tiled the same way (Sec. 2.2.2). */
int distr_attn_exact_fwd(const void *q, const void *k, const void *v, void *o, int B, int H,
                         int Hkv, int N, int d, int Br, int Bc, int causal);

/* The same two operations with every option of da_params. In the bf16 forward with at most 16
 * projections and neither perm_in nor hash_out, the attention kernel runs the LSH stage of each
 * query block in that block's own workgroup (same arithmetic and tables as distr_attn_lsh_group;
 * the table is written only if perm_out is given, e.g. to hand it to the backward pass as
 * perm_in); otherwise the stage is a kernel of its own. */
int distr_attn_fwd_ex(const void *q, const void *k, const void *v, void *o, const da_params *p);
int distr_attn_exact_fwd_ex(const void *q, const void *k, const void *v, void *o, const da_params *p);

/*
 * Backward pass of the two calls above (side = 0). The paper trains through the method (Sec. 4.3,
 * 4.4) without giving a gradient; computed here is the derivative of the forward with every query
 * block's grouping held fixed (the grouping is a piecewise-constant function of q): with
 * P = softmax(S^), dP = dout V^T, D_i = sum_c dout_ic o_ic and dS^ = P o (dP - D),
 * dv = P^T dout;  dq[:, first channel of group j] = scale (dS^ K_f)[:, j] and 0 in the block's
 * other columns;  dk[:, c] = scale * sum over query blocks of (dS^T Q_r)[:, group of c in that
 * block]  (Q_r, K_f: sampled and fused columns, Sec. 3.2, Eq. 2). The exact call is the case of
 * one channel per group (Sec. 2.1).
 * bf16 tensors: matrix-core kernels (bf16 operands, fp32 accumulate; P and dS^ are rounded to bf16
 * before the products that take them), d in {64, 128}, any n_groups that divides d. float tensors:
 * float arithmetic on the vector ALUs (a reference-precision path).
 * q, k, v, p: as given to the forward; o: its output; lse: its lse_out; dout [B][H][N][d]: gradient
 * of the loss with respect to o, same dtype. Written: dq [B][H][N][d], dk and dv [B][Hkv][Nk][d]
 * (p->dtype, device, 16-byte aligned, distinct from every input and from each other). The grouping is recomputed
 * from q (same seed and options give the forward's table) unless p->perm_in brings it. Scratch
 * (the table, and for bf16 tensors D and a copy of q, see distr_attn_bwd_workspace_bytes) comes
 * from p->workspace, else from the library-owned buffer as in the forward. No atomics: results
 * are the same on every run.
 * Errors: as the forward; DA_ERR_UNSUPPORTED for side = 1.
 */
int distr_attn_bwd_ex(const void *q, const void *k, const void *v, const void *o, const void *dout,
                      const float *lse, void *dq, void *dk, void *dv, const da_params *p);
int distr_attn_exact_bwd_ex(const void *q, const void *k, const void *v, const void *o,
                            const void *dout, const float *lse, void *dq, void *dk, void *dv,
                            const da_params *p);

/* Bytes of p->workspace the backward calls need at most for p (0 for invalid parameters):
 * the grouping table and, for bf16 tensors, 8 bytes per query row, a copy of q and (grouped-query
 * shapes with few kv heads) float partial sums of dk and dv per query head of a kv head. */
size_t distr_attn_bwd_workspace_bytes(const da_params *p);

/*
 * LSH hash-and-group stage alone (Sec. 3.2 "similar columns identification", Fig. 5): writes
 * p->perm_out and/or p->hash_out (at least one must be given). Projections are accumulated in
 * float with one fused multiply-add per row, rows ascending; bit of plane 0 is the most
 * significant; channels are sorted by (hash, channel index) ascending. With p->side = 1 the
 * tensor is K ([B][Hkv][Nk][d]) and the blocks are its K blocks of Bc rows.
 */
int distr_attn_lsh_group(const void *q, const da_params *p);

/*
 * Key pre-pass of the bf16 DistrAttention path alone: k [B][Hkv][Nk][d] bf16 -> kt_out
 * [B][Hkv][d][Npad] half, keys fastest, Npad = Nk rounded up to 128, tail zero-filled, values
 * clamped to +-65504/G* so that a group's sum (Sec. 3.2 fusion) stays finite in half. The fusion
 * then adds whole channel rows. Behind the copy it leaves, in 19 KB, the projection matrix of the
 * LSH stage (Sec. 3.2) for p's lsh_seed, n_planes and Br, which the attention kernel's own LSH stage
 * loads instead of generating it in every workgroup; a forward whose seed, projection count or
 * block rows differ from the table's header ignores the table, so a kt_in made with other values
 * of those three stays valid. distr_attn_fwd_ex runs the pre-pass into its workspace unless kt_in
 * is given. kt_out: device, distr_attn_kt_bytes(p) bytes, 256-byte aligned.
 */
int distr_attn_key_prepass(const void *k, void *kt_out, const da_params *p);
size_t distr_attn_kt_bytes(const da_params *p);

/* Bytes of device scratch distr_attn_fwd_ex needs for p: permutation table + transposed keys
 * (0 on invalid p). */
size_t distr_attn_workspace_bytes(const da_params *p);

/*
 * The projection matrix the GPU path uses for (seed, n_planes, Br): host_out[n_planes][Br] floats
 * (host memory). Entry (p, r) depends on (seed, p, r) only. Sec. 3.2 asks for a fixed random
 * matrix; the generator is a counter-based integer mixer whose outputs are exact dyadic floats.
 */
int distr_attn_hyperplanes(uint64_t seed, int n_planes, int Br, float *host_out);

/*
 * distr_attn_fwd_ex for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc. Same arguments, same kernels, same
 * result; the scratch the forward needs (the transposed copy of K, and the permutation table
 * when the LSH stage runs as a kernel of its own) lives in a fixed device array of
 * DISTR_ATTN_NOALLOC_MAX_BYTES inside the library instead of a workspace, so the call allocates
 * and frees nothing (p->workspace is ignored). Each GPU the library runs on holds its own copy
 * of the array until the process ends. A problem whose scratch exceeds the array is refused
 * with DA_ERR_WORKSPACE before anything is launched (kt_in removes the K^T part of the need).
 * All calls on one GPU share the array: calls that overlap in time on one GPU race; calls
 * queued on one stream do not.
 */
#define DISTR_ATTN_NOALLOC_MAX_BYTES (32u << 20)
int distr_attn_fwd_noalloc(const void *q, const void *k, const void *v, void *o, const da_params *p);
size_t distr_attn_noalloc_max_bytes(void);

/* Stream used when da_params.stream is NULL and by the short-form entry points (process-wide). */
int distr_attn_set_stream(void *hip_stream);

/* Frees the library-owned device workspace (synchronises the device first). */
int distr_attn_release(void);

const char *distr_attn_last_error(void);
const char *distr_attn_version(void);

#ifdef __cplusplus
}
#endif
#endif
