// Attention forward (exact and DistrAttention) in float arithmetic for gfx950: the reference-precision
// path, for float tensors and (the mirrored form only) for bf16 tensors converted on load.
//
// Same steps as the bf16 kernel (Sec. 2.2.2 tiling; Sec. 3.2 sampling and fusion per Q block,
// Sec. 3.3; Eq. 2), in plain float FMAs on the vector ALUs. Four adjacent lanes share one query
// row: each takes every fourth (sampled) channel of the score product, the partial sums are
// added across the four lanes, and each lane accumulates a quarter of the output channels.
// K/V tiles of 32 rows go through LDS; the fused tile K_f is built in LDS once per (Q block,
// K tile) and shared by the block's rows; the softmax is online per tile (Sec. 2.2.2).
// Built for accuracy checks on small problems.
//
// side = 1 is the mirrored form of Sec. 3.1 (last sentence of the Eq. 2 paragraph, Fig. 4 right
// side): the grouping belongs to the K block (Bc rows, table [B][Hkv][Tk][d] from the LSH
// stage run on K), one K column per group is sampled and the group's Q columns are summed.
// Every K block then needs its own permutation and its own fused queries -- the reloading
// Sec. 3.3 gives as the reason for sampling Q instead.
#include "da_common.h"

namespace da {

constexpr int kF32Tile = 32;  // key rows per LDS tile of this kernel
constexpr int kF32Lanes = 4;  // lanes per query row

template <typename E, int D, int BR>
__global__ __launch_bounds__(BR * kF32Lanes) void attn_f32_kernel(
    const E* __restrict__ q, const E* __restrict__ k, const E* __restrict__ v,
    E* __restrict__ o, const uint8_t* __restrict__ perm, int H, int Hkv, int N, int Nk, int Tq,
    int n_groups, int causal, float scale, int distr, int side, int Bc, float* __restrict__ lse) {
  constexpr int T = BR * kF32Lanes;
  constexpr int QS = D / kF32Lanes;            // most channels of the score product one lane takes
  constexpr int CS = D / kF32Lanes;            // output channels per lane
  __shared__ float k_lds[kF32Tile][D + 1];     // raw key tile
  __shared__ float kf_lds[kF32Tile][D + 1];    // fused key tile (distr only)
  __shared__ __attribute__((aligned(16))) float v_lds[kF32Tile][D];
  __shared__ uint8_t perm_lds[D];

  const int tid = threadIdx.x;
  const int row = tid / kF32Lanes;             // query row of the block
  const int part = tid % kF32Lanes;
  const int t = blockIdx.x % Tq;
  const int bh = blockIdx.x / Tq;
  const int b = bh / H, h = bh % H;
  const int hk = h / (H / Hkv);
  const int r0 = t * BR;
  const int rows = min(BR, N - r0);
  const int kred = distr ? n_groups : D;
  const int G = D / kred;

  const E* qh = q + ((size_t)bh * N + r0) * D;
  const E* kh = k + ((size_t)(b * Hkv + hk) * Nk) * D;
  const E* vh = v + ((size_t)(b * Hkv + hk) * Nk) * D;
  const int shift = Nk - N;   // causal: key n is visible to query i iff n <= i + shift
  const bool mirrored = distr && side == 1;
  const int Tk = (Nk + Bc - 1) / Bc;

  if (distr && !mirrored)
    // D is a power of two: an out-of-range entry of a caller's table cannot index past a row
    for (int i = tid; i < D; i += T) perm_lds[i] = perm[(size_t)blockIdx.x * D + i] & (D - 1);
  __syncthreads();
  const bool active = row < rows;
  const int i_abs = r0 + row;
  // sampling: column j of Q_r is the first channel of group j in sorted order; this lane keeps
  // columns part, part + 4, ...
  float qreg[QS];
#pragma unroll
  for (int i = 0; i < QS; ++i) {
    const int j = part + kF32Lanes * i;
    qreg[i] = (active && j < kred && !mirrored) ? (float)qh[(size_t)row * D + (distr ? perm_lds[j * G] : j)] : 0.0f;
  }

  float acc[CS];
#pragma unroll
  for (int c = 0; c < CS; ++c) acc[c] = 0.0f;
  float m_run = -INFINITY, l_run = 0.0f;
  const int n_end = causal ? min(Nk, r0 + rows + shift) : Nk;

  for (int n0 = 0; n0 < n_end; n0 += kF32Tile) {
    const int tn = min(kF32Tile, n_end - n0);
    __syncthreads();
    if (mirrored && n0 % Bc == 0) {
      // a new K block: its permutation, and the queries fused by it (members in sorted order)
      const size_t pbase = (((size_t)(b * Hkv + hk)) * Tk + n0 / Bc) * D;
      for (int i = tid; i < D; i += T) perm_lds[i] = perm[pbase + i] & (D - 1);
      __syncthreads();
#pragma unroll
      for (int i = 0; i < QS; ++i) {
        const int j = part + kF32Lanes * i;
        float s = 0.0f;
        if (active && j < kred)
          for (int g = 0; g < G; ++g) s += (float)qh[(size_t)row * D + perm_lds[j * G + g]];
        qreg[i] = s;
      }
    }
    for (int i = tid; i < tn * D; i += T) {
      int n = i / D, c = i % D;
      k_lds[n][c] = (float)kh[(size_t)(n0 + n) * D + c];
      v_lds[n][c] = (float)vh[(size_t)(n0 + n) * D + c];
    }
    __syncthreads();
    if (mirrored) {  // sampling on the K side: the group's first channel in sorted order
      for (int i = tid; i < tn * kred; i += T) {
        int n = i / kred, j = i % kred;
        kf_lds[n][j] = k_lds[n][perm_lds[j * G]];
      }
      __syncthreads();
    } else if (distr) {  // fusion: sum the group's key channels, members in sorted order
      for (int i = tid; i < tn * kred; i += T) {
        int n = i / kred, j = i % kred;
        float s = 0.0f;
        for (int g = 0; g < G; ++g) s += k_lds[n][perm_lds[j * G + g]];
        kf_lds[n][j] = s;
      }
      __syncthreads();
    }
    const float(*kx)[D + 1] = distr ? kf_lds : k_lds;
    // scores of the tile: partial dot products, summed over the row's four lanes
    float sc[kF32Tile];
    float m_tile = -INFINITY;
#pragma unroll
    for (int n = 0; n < kF32Tile; ++n) {
      float s = 0.0f;
      if (n < tn) {
#pragma unroll
        for (int i = 0; i < QS; ++i) {
          const int j = part + kF32Lanes * i;
          if (j < kred) s = __builtin_fmaf(qreg[i], kx[n][j], s);
        }
      }
      s += __shfl_xor(s, 1);
      s += __shfl_xor(s, 2);
      s *= scale;
      if (n >= tn || (causal && n0 + n > i_abs + shift)) s = -INFINITY;
      sc[n] = s;
      m_tile = fmaxf(m_tile, s);
    }
    // online softmax step for the tile (Sec. 2.2.2); a row whose keys of this tile are all
    // masked keeps its state (its first tile always holds key 0, so m_run is finite by then)
    const float m_new = fmaxf(m_run, m_tile);
    const float alpha = (m_new == -INFINITY) ? 1.0f : expf(m_run - m_new);   // exp(-inf) = 0 on the first tile
    float psum = 0.0f;
#pragma unroll
    for (int n = 0; n < kF32Tile; ++n) {
      sc[n] = (sc[n] == -INFINITY) ? 0.0f : expf(sc[n] - m_new);
      psum += sc[n];
    }
    l_run = l_run * alpha + psum;
    m_run = m_new;
#pragma unroll
    for (int c = 0; c < CS; ++c) acc[c] *= alpha;
#pragma unroll
    for (int n = 0; n < kF32Tile; ++n) {
      if (n < tn) {
        const float p = sc[n];
#pragma unroll
        for (int c = 0; c < CS; ++c) acc[c] = __builtin_fmaf(p, v_lds[n][part * CS + c], acc[c]);
      }
    }
  }
  if (active) {
    if (lse && part == 0) lse[(size_t)bh * N + i_abs] = m_run + logf(l_run);   // row statistics for a backward pass
    float inv = 1.0f / l_run;
    E* orow = o + ((size_t)bh * N + i_abs) * D + part * CS;
#pragma unroll
    for (int c = 0; c < CS; ++c) orow[c] = (E)(acc[c] * inv);
  }
}

template <typename E>
static hipError_t launch_f32_typed(const void* q, const void* k, const void* v, void* o, const uint8_t* perm,
                                   const Problem& pb, int distr, hipStream_t stream) {
  const int Tq = (pb.N + pb.Br - 1) / pb.Br;
  const long long units = (long long)pb.B * pb.H * Tq;
  dim3 grid((unsigned)units);
#define DA_F32_LAUNCH(DD, BB)                                                                          \
  hipLaunchKernelGGL((attn_f32_kernel<E, DD, BB>), grid, dim3(BB * kF32Lanes), 0, stream, (const E*)q,  \
                     (const E*)k, (const E*)v, (E*)o, perm, pb.H, pb.Hkv, pb.N, pb.Nk, Tq, pb.n_groups, \
                     pb.causal, pb.scale, distr, pb.side, pb.Bc, pb.lse)
  if (pb.d == 64 && pb.Br == 64) DA_F32_LAUNCH(64, 64);
  else if (pb.d == 64 && pb.Br == 128) DA_F32_LAUNCH(64, 128);
  else if (pb.d == 128 && pb.Br == 64) DA_F32_LAUNCH(128, 64);
  else if (pb.d == 128 && pb.Br == 128) DA_F32_LAUNCH(128, 128);
  else if (pb.d == 64 && pb.Br == 256) DA_F32_LAUNCH(64, 256);
  else if (pb.d == 128 && pb.Br == 256) DA_F32_LAUNCH(128, 256);
  else return hipErrorInvalidValue;
#undef DA_F32_LAUNCH
  return hipGetLastError();
}

// dtype 0: bf16 tensors (converted on load, rounded on store), 1: float tensors; float arithmetic either way
hipError_t launch_attn_f32(const void* q, const void* k, const void* v, void* o, const uint8_t* perm,
                           const Problem& pb, int dtype, int distr, hipStream_t stream) {
  return dtype == 0 ? launch_f32_typed<bf16>(q, k, v, o, perm, pb, distr, stream)
                    : launch_f32_typed<float>(q, k, v, o, perm, pb, distr, stream);
}

}  // namespace da
