// Key pre-pass of the DistrAttention path: K [B][Hkv][Nk][d] (bf16, d fastest) is rewritten once
// per forward as K^T [B][Hkv][d][Npad] in half precision (keys fastest, Npad = Nk rounded up to
// the largest key tile, 128, tail zero-filled).
//
// Why: the fusion step of Sec. 3.2 sums, for every (Q block, K tile) pair, the key channels of a
// group chosen by that Q block's permutation. With keys fastest a channel is one contiguous
// row, so "sum the group's channels" becomes whole-row vector adds (16-byte LDS reads, packed
// half adds) instead of 2-byte gathers across a row-major tile. The pre-pass costs one read and
// one write of K; the fusion it speeds up runs N/Br times over the same data.
//
// bf16 -> half is exact inside half's range (8 vs 11 significand bits). Values are clamped to
// +-65504/G so that the sum of a group's G channels cannot overflow half.
#include "da_common.h"

namespace da {

typedef _Float16 f16;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;

constexpr int kKtThreads = 256;

// The projection matrix for (seed, n_planes, Br), as two bf16 pieces with r1 + r2 = R exactly (an
// entry is an integer of 17 bits times 2^-16), in the layout the attention kernel loads it in.
// Written by one extra workgroup of the pre-pass (a launch of its own would cost more than the
// table saves).
__device__ inline void write_rtab(char* __restrict__ rtab, uint64_t seed, int n_planes, int Br) {
  const int rpad = Br + 8;
  bf16* rp1 = (bf16*)(rtab + kRtabHead);
  bf16* rp2 = (bf16*)(rtab + kRtabHead + rtab_piece_bytes(Br));
  for (int i = threadIdx.x; i < 16 * Br; i += kKtThreads) {
    const int r = i % Br, pl = i / Br;
    const float rv = pl < n_planes ? hyperplane_entry(seed, (uint32_t)pl, (uint32_t)r) : 0.0f;
    const bf16 r1 = (bf16)rv;
    rp1[pl * rpad + r] = r1;
    rp2[pl * rpad + r] = (bf16)(rv - (float)r1);
  }
  if (threadIdx.x == 0) {
    RtabHeader* hd = (RtabHeader*)rtab;
    hd->seed = seed;
    hd->n_planes = n_planes;
    hd->Br = Br;
  }
}

template <int D>
__global__ __launch_bounds__(kKtThreads) void kt_prepass_kernel(const bf16* __restrict__ k,
                                                                f16* __restrict__ kt, int N, int Npad,
                                                                int Tk, float limit, int units, char* __restrict__ rtab,
                                                                uint64_t seed, int n_planes, int Br) {
  if ((int)blockIdx.x == units) {   // the extra workgroup
    write_rtab(rtab, seed, n_planes, Br);
    return;
  }
  // tile[key][channel], row stride D + 2 halves (odd number of dwords: the column reads below
  // hit distinct banks)
  __shared__ f16 tile[kBc][D + 2];
  const int tid = threadIdx.x;
  const int tk = blockIdx.x % Tk;
  const size_t head = blockIdx.x / Tk;
  const int n0 = tk * kBc;
  const bf16* kh = k + head * (size_t)N * D;
  f16* kth = kt + head * (size_t)D * Npad;

  constexpr int CH = D / 8;   // 16-byte chunks per key row
  for (int id = tid; id < kBc * CH; id += kKtThreads) {
    const int row = id / CH, col = (id % CH) * 8;
    bf16x8 x;
    if (n0 + row < N) x = *(const bf16x8*)(kh + (size_t)(n0 + row) * D + col);
    else
#pragma unroll
      for (int j = 0; j < 8; ++j) x[j] = (bf16)0.0f;
#pragma unroll
    for (int j = 0; j < 8; ++j)
      tile[row][col + j] = (f16)__builtin_amdgcn_fmed3f((float)x[j], -limit, limit);
  }
  __syncthreads();
  // output chunk (channel c, 8 consecutive keys)
  for (int id = tid; id < D * (kBc / 8); id += kKtThreads) {
    const int c = id / (kBc / 8), kc = (id % (kBc / 8)) * 8;
    f16x8 y;
#pragma unroll
    for (int j = 0; j < 8; ++j) y[j] = tile[kc + j][c];
    *(f16x8*)(kth + (size_t)c * Npad + n0 + kc) = y;
  }
}

hipError_t launch_kt_prepass(const void* k, void* kt, const Problem& pb, hipStream_t stream) {
  const int Npad = (pb.Nk + kKtPad - 1) / kKtPad * kKtPad;
  const int Tk = Npad / kBc;   // tiles past the last key are written as zeros
  const long long units = (long long)pb.B * pb.Hkv * Tk;
  const float limit = 65504.0f / (float)(pb.d / pb.n_groups);
  if (units >= 0x7fffffffLL) return hipErrorInvalidValue;
  char* rtab = (char*)kt + kt_copy_bytes(pb.B, pb.Hkv, pb.d, pb.Nk);
  const bool with_table = pb.Br <= 256;   // the largest block the table is laid out for
  dim3 grid((unsigned)units + (with_table ? 1u : 0u)), block(kKtThreads);
  if (pb.d == 64)
    hipLaunchKernelGGL((kt_prepass_kernel<64>), grid, block, 0, stream, (const bf16*)k, (f16*)kt, pb.Nk, Npad, Tk, limit,
                       (int)units, rtab, pb.seed, pb.n_planes, pb.Br);
  else if (pb.d == 128)
    hipLaunchKernelGGL((kt_prepass_kernel<128>), grid, block, 0, stream, (const bf16*)k, (f16*)kt, pb.Nk, Npad, Tk, limit,
                       (int)units, rtab, pb.seed, pb.n_planes, pb.Br);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace da
