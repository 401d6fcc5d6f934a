// Float attention forward (exact and DistrAttention) for gfx950: the reference-precision path.
//
// Same steps as the bf16 kernel (Sec. 2.2.2 tiling; Sec. 3.2 sampling and fusion per Q block,
// Sec. 3.3; Eq. 2), in plain float FMAs: one thread owns one query row, K/V tiles of 32 rows go
// through LDS, the fused tile K_f is built in LDS once per (Q block, K tile) and shared by the
// block's rows. Built for accuracy checks on small problems, not for speed.
#include "da_common.h"

namespace da {

constexpr int kF32Tile = 32;  // key rows per LDS tile of this kernel

template <int D, int BR>
__global__ __launch_bounds__(BR) void attn_f32_kernel(
    const float* __restrict__ q, const float* __restrict__ k, const float* __restrict__ v,
    float* __restrict__ o, const uint8_t* __restrict__ perm, int H, int Hkv, int N, int Tq,
    int n_groups, int causal, float scale, int distr) {
  __shared__ float q_lds[BR][D + 1];           // sampled (or full) query rows
  __shared__ float k_lds[kF32Tile][D + 1];     // raw key tile
  __shared__ float kf_lds[kF32Tile][D + 1];    // fused key tile (distr only)
  __shared__ float v_lds[kF32Tile][D];
  __shared__ uint8_t perm_lds[D];

  const int tid = threadIdx.x;
  const int t = blockIdx.x % Tq;
  const int bh = blockIdx.x / Tq;
  const int b = bh / H, h = bh % H;
  const int hk = h / (H / Hkv);
  const int r0 = t * BR;
  const int rows = min(BR, N - r0);
  const int kred = distr ? n_groups : D;
  const int G = D / kred;

  const float* qh = q + ((size_t)bh * N + r0) * D;
  const float* kh = k + ((size_t)(b * Hkv + hk) * N) * D;
  const float* vh = v + ((size_t)(b * Hkv + hk) * N) * D;

  if (distr)
    for (int i = tid; i < D; i += BR) perm_lds[i] = perm[(size_t)blockIdx.x * D + i];
  __syncthreads();
  // sampling: column j of Q_r is the first channel of group j in sorted order
  for (int i = tid; i < rows * kred; i += BR) {
    int r = i / kred, j = i % kred;
    q_lds[r][j] = qh[(size_t)r * D + (distr ? perm_lds[j * G] : j)];
  }

  float acc[D];
#pragma unroll
  for (int c = 0; c < D; ++c) acc[c] = 0.0f;
  float m_run = -INFINITY, l_run = 0.0f;
  const int i_abs = r0 + tid;
  const bool active = tid < rows;
  const int n_end = causal ? min(N, r0 + rows) : N;

  for (int n0 = 0; n0 < n_end; n0 += kF32Tile) {
    const int tn = min(kF32Tile, n_end - n0);
    __syncthreads();
    for (int i = tid; i < tn * D; i += BR) {
      int n = i / D, c = i % D;
      k_lds[n][c] = kh[(size_t)(n0 + n) * D + c];
      v_lds[n][c] = vh[(size_t)(n0 + n) * D + c];
    }
    __syncthreads();
    if (distr) {  // fusion: sum the group's key channels, members in sorted order
      for (int i = tid; i < tn * kred; i += BR) {
        int n = i / kred, j = i % kred;
        float s = 0.0f;
        for (int g = 0; g < G; ++g) s += k_lds[n][perm_lds[j * G + g]];
        kf_lds[n][j] = s;
      }
      __syncthreads();
    }
    if (active) {
      const float(*kx)[D + 1] = distr ? kf_lds : k_lds;
      for (int n = 0; n < tn; ++n) {
        if (causal && n0 + n > i_abs) break;
        float s = 0.0f;
        for (int j = 0; j < kred; ++j) s = __builtin_fmaf(q_lds[tid][j], kx[n][j], s);
        s *= scale;
        float m_new = fmaxf(m_run, s);
        float alpha = expf(m_run - m_new);   // exp(-inf) = 0 on the first key
        float p = expf(s - m_new);
        l_run = l_run * alpha + p;
        m_run = m_new;
#pragma unroll
        for (int c = 0; c < D; ++c) acc[c] = __builtin_fmaf(p, v_lds[n][c], acc[c] * alpha);
      }
    }
  }
  if (active) {
    float inv = 1.0f / l_run;
    float* orow = o + ((size_t)bh * N + i_abs) * D;
#pragma unroll
    for (int c = 0; c < D; ++c) orow[c] = acc[c] * inv;
  }
}

hipError_t launch_attn_f32(const void* q, const void* k, const void* v, void* o, const uint8_t* perm,
                           const Problem& pb, int distr, hipStream_t stream) {
  const int Tq = (pb.N + pb.Br - 1) / pb.Br;
  const long long units = (long long)pb.B * pb.H * Tq;
  dim3 grid((unsigned)units);
#define DA_F32_LAUNCH(DD, BB)                                                                      \
  hipLaunchKernelGGL((attn_f32_kernel<DD, BB>), grid, dim3(BB), 0, stream, (const float*)q,        \
                     (const float*)k, (const float*)v, (float*)o, perm, pb.H, pb.Hkv, pb.N, Tq,    \
                     pb.n_groups, pb.causal, pb.scale, distr)
  if (pb.d == 64 && pb.Br == 64) DA_F32_LAUNCH(64, 64);
  else if (pb.d == 64 && pb.Br == 128) DA_F32_LAUNCH(64, 128);
  else if (pb.d == 128 && pb.Br == 64) DA_F32_LAUNCH(128, 64);
  else if (pb.d == 128 && pb.Br == 128) DA_F32_LAUNCH(128, 128);
  else return hipErrorInvalidValue;
#undef DA_F32_LAUNCH
  return hipGetLastError();
}

}  // namespace da
