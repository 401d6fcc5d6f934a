// Backward of the attention forward (exact and DistrAttention) for gfx950 in float arithmetic on
// the vector ALUs: the reference-precision path, for float tensors (bf16 tensors take the
// matrix-core kernels of attn_bf16_bwd.hip); two kernels, no atomics (results do not depend on the run).
//
// The paper trains through the approximation (Sec. 4.3, 4.4) and gives no gradient. Computed
// here: the derivative of the forward with every Q block's grouping held fixed (the permutation
// is a piecewise-constant function of Q). With P = softmax(S^) rebuilt from the saved row
// statistics, dP = dO V^T, D_i = sum_c dO_ic O_ic and dS^ = P o (dP - D):
//   dV = P^T dO
//   dQ[:, first channel of group j] = scale * (dS^ K_f)[:, j]; the other columns of the block 0
//   dK[:, c] = scale * sum over Q blocks of (dS^T Q_r)[:, group of c in that block]
// (Eq. 2 with Q_r the sampled and K_f the fused columns of Sec. 3.2; one grouping per Q block,
// Sec. 3.3). Exact attention is the case of one channel per group.
//
// Kernel 1 (dQ): one workgroup per Q block, four lanes per query row as in the forward; K/V tiles
// of 32 rows through LDS, the fused tile K_f rebuilt per tile.
// Kernel 2 (dK, dV): one workgroup per (kv head, 32 keys), four lanes per key; it walks every
// query head of the kv head and every Q block that sees the keys, rebuilds that block's fused
// keys in registers, and un-fuses the block's dK_f into a dK tile in LDS through the block's
// permutation (the mirror image of the forward's fusion).
#include "da_common.h"

namespace da {

constexpr int kBwdTile = 32;   // key rows per tile (both kernels)
constexpr int kBwdLanes = 4;   // lanes per query row (kernel 1) / per key (kernel 2)
constexpr int kBwdChunk = 16;  // query rows staged at a time by kernel 2

__device__ inline float quad_sum(float x) {
  x += __shfl_xor(x, 1);
  x += __shfl_xor(x, 2);
  return x;
}

template <typename E, int D, int BR>
__global__ __launch_bounds__(BR * kBwdLanes) void attn_f32_bwd_dq_kernel(
    const E* __restrict__ q, const E* __restrict__ k, const E* __restrict__ v,
    const E* __restrict__ o, const E* __restrict__ dout, const float* __restrict__ lse,
    E* __restrict__ dq, const uint8_t* __restrict__ perm, int H, int Hkv, int N, int Nk, int Tq,
    int n_groups, int causal, float scale, int distr) {
  constexpr int T = BR * kBwdLanes;
  constexpr int QS = D / kBwdLanes;   // most columns of the score product one lane takes
  constexpr int CS = D / kBwdLanes;   // channels of dO, O and V per lane
  __shared__ float k_lds[kBwdTile][D + 1];
  __shared__ float kf_lds[kBwdTile][D + 1];
  __shared__ __attribute__((aligned(16))) float v_lds[kBwdTile][D];
  __shared__ uint8_t perm_lds[D];
  __shared__ uint8_t sampled_lds[D];   // 1 where the channel is its group's first in sorted order

  const int tid = threadIdx.x;
  const int row = tid / kBwdLanes, part = tid % kBwdLanes;
  const int t = blockIdx.x % Tq;
  const int bh = blockIdx.x / Tq;
  const int b = bh / H, h = bh % H;
  const int hk = h / (H / Hkv);
  const int r0 = t * BR;
  const int rows = min(BR, N - r0);
  const int kred = distr ? n_groups : D;
  const int G = D / kred;
  const int shift = Nk - N;   // causal: key n is visible to query i iff n <= i + shift

  const E* kh = k + ((size_t)(b * Hkv + hk) * Nk) * D;
  const E* vh = v + ((size_t)(b * Hkv + hk) * Nk) * D;

  for (int i = tid; i < D; i += T) {
    perm_lds[i] = distr ? (perm[(size_t)blockIdx.x * D + i] & (D - 1)) : (uint8_t)i;
    sampled_lds[i] = 0;
  }
  __syncthreads();
  for (int j = tid; j < kred; j += T) sampled_lds[perm_lds[j * G]] = 1;
  __syncthreads();

  const bool active = row < rows;
  const int i_abs = r0 + row;
  const size_t row_off = ((size_t)bh * N + (active ? i_abs : r0)) * D;
  float qreg[QS], dqr[QS], doreg[CS];
#pragma unroll
  for (int i = 0; i < QS; ++i) {
    const int j = part + kBwdLanes * i;
    qreg[i] = (active && j < kred) ? (float)q[row_off + perm_lds[j * G]] : 0.0f;
    dqr[i] = 0.0f;
  }
  float dsum = 0.0f;
#pragma unroll
  for (int c = 0; c < CS; ++c) {
    doreg[c] = active ? (float)dout[row_off + part * CS + c] : 0.0f;
    dsum = __builtin_fmaf(doreg[c], active ? (float)o[row_off + part * CS + c] : 0.0f, dsum);
  }
  const float Drow = quad_sum(dsum);
  const float lse_row = active ? lse[(size_t)bh * N + i_abs] : 0.0f;
  const int n_end = causal ? min(Nk, r0 + rows + shift) : Nk;

  for (int n0 = 0; n0 < n_end; n0 += kBwdTile) {
    const int tn = min(kBwdTile, n_end - n0);
    __syncthreads();
    for (int i = tid; i < tn * D; i += T) {
      int n = i / D, c = i % D;
      k_lds[n][c] = (float)kh[(size_t)(n0 + n) * D + c];
      v_lds[n][c] = (float)vh[(size_t)(n0 + n) * D + c];
    }
    __syncthreads();
    for (int i = tid; i < tn * kred; i += T) {   // fusion, members in sorted order
      int n = i / kred, j = i % kred;
      float s = 0.0f;
      for (int g = 0; g < G; ++g) s += k_lds[n][perm_lds[j * G + g]];
      kf_lds[n][j] = s;
    }
    __syncthreads();
    for (int n = 0; n < tn; ++n) {
      float s = 0.0f, dp = 0.0f;
#pragma unroll
      for (int i = 0; i < QS; ++i) {
        const int j = part + kBwdLanes * i;
        if (j < kred) s = __builtin_fmaf(qreg[i], kf_lds[n][j], s);
      }
#pragma unroll
      for (int c = 0; c < CS; ++c) dp = __builtin_fmaf(doreg[c], v_lds[n][part * CS + c], dp);
      s = quad_sum(s) * scale;
      dp = quad_sum(dp);
      const bool visible = active && !(causal && n0 + n > i_abs + shift);
      const float p = visible ? expf(s - lse_row) : 0.0f;
      const float ds = p * (dp - Drow);
#pragma unroll
      for (int i = 0; i < QS; ++i) {
        const int j = part + kBwdLanes * i;
        if (j < kred) dqr[i] = __builtin_fmaf(ds, kf_lds[n][j], dqr[i]);
      }
    }
  }
  if (active) {
    E* dqrow = dq + row_off;
    // the row's four lanes write disjoint columns: zeros where the channel was not sampled,
    // the gradient of column j of Q_r at the channel it was sampled from
    for (int c = part; c < D; c += kBwdLanes)
      if (!sampled_lds[c]) dqrow[c] = (E)0.0f;
#pragma unroll
    for (int i = 0; i < QS; ++i) {
      const int j = part + kBwdLanes * i;
      if (j < kred) dqrow[perm_lds[j * G]] = (E)(scale * dqr[i]);
    }
  }
}

template <typename E, int D>
__global__ __launch_bounds__(kBwdTile * kBwdLanes) void attn_f32_bwd_dkv_kernel(
    const E* __restrict__ q, const E* __restrict__ k, const E* __restrict__ v,
    const E* __restrict__ o, const E* __restrict__ dout, const float* __restrict__ lse,
    E* __restrict__ dk, E* __restrict__ dv, const uint8_t* __restrict__ perm, int H, int Hkv,
    int N, int Nk, int Br, int Tq, int Tk, int n_groups, int causal, float scale, int distr) {
  constexpr int T = kBwdTile * kBwdLanes;
  constexpr int QS = D / kBwdLanes;
  constexpr int CS = D / kBwdLanes;
  __shared__ float k_lds[kBwdTile][D + 1];     // the keys of this workgroup
  __shared__ float dk_lds[kBwdTile][D + 1];    // their gradient, channel order
  __shared__ float qr_lds[kBwdChunk][D + 1];   // sampled query columns of the staged rows
  __shared__ float do_lds[kBwdChunk][D + 1];   // dO of the staged rows
  __shared__ float lse_lds[kBwdChunk];
  __shared__ float drow_lds[kBwdChunk];        // D_i = sum_c dO_ic O_ic
  __shared__ uint8_t perm_lds[D];

  const int tid = threadIdx.x;
  const int key = tid / kBwdLanes, part = tid % kBwdLanes;
  const int tk = blockIdx.x % Tk;
  const int bk = blockIdx.x / Tk;          // b * Hkv + hk
  const int b = bk / Hkv, hk = bk % Hkv;
  const int rep = H / Hkv;
  const int n0 = tk * kBwdTile;
  const int tn = min(kBwdTile, Nk - n0);
  const int n_abs = n0 + key;
  const bool valid = key < tn;
  const int kred = distr ? n_groups : D;
  const int G = D / kred;
  const int shift = Nk - N;

  const E* kh = k + ((size_t)bk * Nk + n0) * D;
  const E* vh = v + ((size_t)bk * Nk + n0) * D;
  for (int i = tid; i < kBwdTile * D; i += T) {
    int n = i / D, c = i % D;
    k_lds[n][c] = n < tn ? (float)kh[(size_t)n * D + c] : 0.0f;
    dk_lds[n][c] = 0.0f;
  }
  float vreg[CS], dvacc[CS];
#pragma unroll
  for (int c = 0; c < CS; ++c) {
    vreg[c] = valid ? (float)vh[(size_t)key * D + part * CS + c] : 0.0f;
    dvacc[c] = 0.0f;
  }
  // causal: the first Q block with a row that sees key n0 (row i sees it iff i >= n0 - shift)
  const int t_first = causal ? max(0, n0 - shift) / Br : 0;

  for (int h = hk * rep; h < (hk + 1) * rep; ++h) {
    const size_t bh = (size_t)b * H + h;
    for (int t = t_first; t < Tq; ++t) {
      const int r0 = t * Br;
      const int rows = min(Br, N - r0);
      __syncthreads();   // previous block's reads of perm_lds and the staging buffers are done
      for (int i = tid; i < D; i += T)
        perm_lds[i] = distr ? (perm[(bh * Tq + t) * D + i] & (D - 1)) : (uint8_t)i;
      __syncthreads();
      float kf[QS], dkf[QS];
#pragma unroll
      for (int i = 0; i < QS; ++i) {
        const int j = part + kBwdLanes * i;
        float s = 0.0f;
        if (j < kred)
          for (int g = 0; g < G; ++g) s += k_lds[key][perm_lds[j * G + g]];
        kf[i] = s;
        dkf[i] = 0.0f;
      }
      for (int c0 = 0; c0 < rows; c0 += kBwdChunk) {
        const int cr = min(kBwdChunk, rows - c0);
        __syncthreads();
        // stage the chunk: sampled query columns, dO, row statistics; eight threads per row
        // take the row's dO.O product
        const size_t base = (bh * N + r0 + c0) * D;
        for (int i = tid; i < cr * D; i += T) {
          int r = i / D, c = i % D;
          do_lds[r][c] = (float)dout[base + (size_t)r * D + c];
          if (c < kred) qr_lds[r][c] = (float)q[base + (size_t)r * D + perm_lds[c * G]];
        }
        {
          constexpr int TPR = T / kBwdChunk;   // threads per staged row
          const int r = tid / TPR, sub = tid % TPR;
          float acc = 0.0f;
          if (r < cr)
            for (int c = sub; c < D; c += TPR)
              acc = __builtin_fmaf((float)dout[base + (size_t)r * D + c], (float)o[base + (size_t)r * D + c], acc);
#pragma unroll
          for (int m = 1; m < TPR; m <<= 1) acc += __shfl_xor(acc, m);
          if (r < cr && sub == 0) {
            drow_lds[r] = acc;
            lse_lds[r] = lse[bh * N + r0 + c0 + r];
          }
        }
        __syncthreads();
        for (int r = 0; r < cr; ++r) {
          const int i_abs = r0 + c0 + r;
          float s = 0.0f, dp = 0.0f;
#pragma unroll
          for (int i = 0; i < QS; ++i) {
            const int j = part + kBwdLanes * i;
            if (j < kred) s = __builtin_fmaf(qr_lds[r][j], kf[i], s);
          }
#pragma unroll
          for (int c = 0; c < CS; ++c) dp = __builtin_fmaf(do_lds[r][part * CS + c], vreg[c], dp);
          s = quad_sum(s) * scale;
          dp = quad_sum(dp);
          const bool visible = valid && !(causal && n_abs > i_abs + shift);
          const float p = visible ? expf(s - lse_lds[r]) : 0.0f;
          const float ds = p * (dp - drow_lds[r]);
#pragma unroll
          for (int c = 0; c < CS; ++c) dvacc[c] = __builtin_fmaf(p, do_lds[r][part * CS + c], dvacc[c]);
#pragma unroll
          for (int i = 0; i < QS; ++i) {
            const int j = part + kBwdLanes * i;
            if (j < kred) dkf[i] = __builtin_fmaf(ds, qr_lds[r][j], dkf[i]);
          }
        }
      }
      // un-fuse: every member of group j receives the gradient of the fused column j. The four
      // lanes of a key hold different groups, hence different channels: no two threads meet.
#pragma unroll
      for (int i = 0; i < QS; ++i) {
        const int j = part + kBwdLanes * i;
        if (j < kred)
          for (int g = 0; g < G; ++g) dk_lds[key][perm_lds[j * G + g]] += dkf[i];
      }
    }
  }
  __syncthreads();
  E* dkh = dk + ((size_t)bk * Nk + n0) * D;
  E* dvh = dv + ((size_t)bk * Nk + n0) * D;
  for (int i = tid; i < tn * D; i += T) {
    int n = i / D, c = i % D;
    dkh[(size_t)n * D + c] = (E)(scale * dk_lds[n][c]);
  }
  if (valid) {
#pragma unroll
    for (int c = 0; c < CS; ++c) dvh[(size_t)key * D + part * CS + c] = (E)dvacc[c];
  }
}

template <typename T>
static hipError_t launch_bwd_typed(const void* q, const void* k, const void* v, const void* o, const void* dout,
                                   const float* lse, void* dq, void* dk, void* dv, const uint8_t* perm,
                                   const Problem& pb, int distr, hipStream_t stream) {
  const int Tq = (pb.N + pb.Br - 1) / pb.Br;
  const int Tk = (pb.Nk + kBwdTile - 1) / kBwdTile;
  const long long q_units = (long long)pb.B * pb.H * Tq;
  const long long k_units = (long long)pb.B * pb.Hkv * Tk;
  if (k_units > 0x7fffffffLL) return hipErrorInvalidValue;
#define DA_BWD_DQ(DD, BB)                                                                                       \
  hipLaunchKernelGGL((attn_f32_bwd_dq_kernel<T, DD, BB>), dim3((unsigned)q_units), dim3(BB * kBwdLanes), 0, stream, \
                     (const T*)q, (const T*)k, (const T*)v, (const T*)o, (const T*)dout, lse, (T*)dq, perm, pb.H, \
                     pb.Hkv, pb.N, pb.Nk, Tq, pb.n_groups, pb.causal, pb.scale, distr)
  if (pb.d == 64 && pb.Br == 64) DA_BWD_DQ(64, 64);
  else if (pb.d == 64 && pb.Br == 128) DA_BWD_DQ(64, 128);
  else if (pb.d == 64 && pb.Br == 256) DA_BWD_DQ(64, 256);
  else if (pb.d == 128 && pb.Br == 64) DA_BWD_DQ(128, 64);
  else if (pb.d == 128 && pb.Br == 128) DA_BWD_DQ(128, 128);
  else if (pb.d == 128 && pb.Br == 256) DA_BWD_DQ(128, 256);
  else return hipErrorInvalidValue;
#undef DA_BWD_DQ
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
#define DA_BWD_DKV(DD)                                                                                            \
  hipLaunchKernelGGL((attn_f32_bwd_dkv_kernel<T, DD>), dim3((unsigned)k_units), dim3(kBwdTile * kBwdLanes), 0, stream, \
                     (const T*)q, (const T*)k, (const T*)v, (const T*)o, (const T*)dout, lse, (T*)dk, (T*)dv, perm,  \
                     pb.H, pb.Hkv, pb.N, pb.Nk, pb.Br, Tq, Tk, pb.n_groups, pb.causal, pb.scale, distr)
  if (pb.d == 64) DA_BWD_DKV(64);
  else DA_BWD_DKV(128);
#undef DA_BWD_DKV
  return hipGetLastError();
}

hipError_t launch_attn_f32_bwd(const void* q, const void* k, const void* v, const void* o, const void* dout,
                               const float* lse, void* dq, void* dk, void* dv, const uint8_t* perm,
                               const Problem& pb, int distr, hipStream_t stream) {
  return launch_bwd_typed<float>(q, k, v, o, dout, lse, dq, dk, dv, perm, pb, distr, stream);
}

}  // namespace da
