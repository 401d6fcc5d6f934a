// LSH hash-and-group kernel (arXiv 2507.17245, Sec. 3.2 "similar columns identification" and
// Fig. 5; once per Q block as in Sec. 3.3).
//
// One workgroup per (batch, head, Q block). For every channel column of the block:
//   projection onto n_planes random directions -> sign bits -> Gray map -> integer hash;
// then the d hashes are ranked (ascending, ties by channel index) and the inverse of the rank
// is written as the block's channel permutation.
//
// The sign of a projection decides an integer, so the sum is taken in a fixed order that a CPU
// can repeat bit for bit: float, one fused multiply-add per row, rows ascending, starting at +0.
// That is why this stage runs on the vector ALUs and not on the matrix cores, although the
// paper picked N' = 16 with tensor cores in mind.
#include "da_common.h"

namespace da {

constexpr int kLshThreads = 256;
constexpr int kMaxLshRows = 256;   // largest block the stage hashes (Q blocks up to 256 rows, K blocks up to 128)

template <typename T>
__device__ inline float to_float(T x);
template <>
__device__ inline float to_float<float>(float x) { return x; }
template <>
__device__ inline float to_float<bf16>(bf16 x) { return (float)x; }

// Accumulate JMAX planes for one channel over the block's rows.
template <typename T, int D, int JMAX>
__device__ inline uint32_t project_bits(const T* __restrict__ qcol, int rows, const float* R_lds,
                                        int pg, int n_planes) {
  constexpr int NPG = kLshThreads / D;
  float acc[JMAX];
#pragma unroll
  for (int j = 0; j < JMAX; ++j) acc[j] = 0.0f;
  const float* Rt = R_lds + pg * (kMaxPlanes / NPG);
#pragma unroll 4
  for (int r = 0; r < rows; ++r) {
    float x = to_float<T>(qcol[(size_t)r * D]);
#pragma unroll
    for (int j = 0; j < JMAX; ++j) acc[j] = __builtin_fmaf(x, Rt[r * kMaxPlanes + j], acc[j]);
  }
  uint32_t bits = 0;
#pragma unroll
  for (int j = 0; j < JMAX; ++j) {
    int p = j * NPG + pg;  // plane handled in slot j of this thread
    if (p < n_planes && acc[j] > 0.0f) bits |= 1u << (n_planes - 1 - p);  // plane 0 = top bit
  }
  return bits;
}

template <typename T, int D>
__global__ __launch_bounds__(kLshThreads) void lsh_group_kernel(
    const T* __restrict__ q, uint8_t* __restrict__ perm_out, uint32_t* __restrict__ hash_out,
    int N, int Br, int Tq, int n_planes, int gray_mode, uint64_t seed) {
  constexpr int NPG = kLshThreads / D;        // threads per channel, each takes planes p = j*NPG + pg
  constexpr int PPT = kMaxPlanes / NPG;       // plane slots per thread
  __shared__ float R_lds[kMaxLshRows * kMaxPlanes];   // [row][pg][j], zero where the plane does not exist
  __shared__ uint32_t code_lds[D];
  __shared__ __attribute__((aligned(16))) uint32_t hash_lds[D];
  __shared__ uint8_t perm_lds[D];

  const int tid = threadIdx.x;
  const int t = blockIdx.x % Tq;
  const size_t bh = blockIdx.x / Tq;
  const int r0 = t * Br;
  const int rows = min(Br, N - r0);

  for (int i = tid; i < Br * kMaxPlanes; i += kLshThreads) {
    int r = i / kMaxPlanes, rem = i % kMaxPlanes;
    int pg = rem / PPT, j = rem % PPT;
    int p = j * NPG + pg;
    R_lds[i] = (p < n_planes) ? hyperplane_entry(seed, (uint32_t)p, (uint32_t)r) : 0.0f;
  }
  if (tid < D) code_lds[tid] = 0;
  __syncthreads();

  const int c = tid % D;
  const int pg = tid / D;
  const T* qcol = q + (bh * N + r0) * D + c;
  const int slots = (n_planes + NPG - 1) / NPG;
  uint32_t bits;
  if (slots <= 4) bits = project_bits<T, D, (PPT < 4 ? PPT : 4)>(qcol, rows, R_lds, pg, n_planes);
  else if (slots <= 8) bits = project_bits<T, D, (PPT < 8 ? PPT : 8)>(qcol, rows, R_lds, pg, n_planes);
  else bits = project_bits<T, D, PPT>(qcol, rows, R_lds, pg, n_planes);
  if (bits) atomicOr(&code_lds[c], bits);
  __syncthreads();

  if (tid < D) {
    const uint32_t h = lsh_hash_of_code(code_lds[tid], gray_mode);
    hash_lds[tid] = h;
    code_lds[tid] = 0;   // from here on the channel's rank is counted in this word
    if (hash_out) hash_out[(size_t)blockIdx.x * D + tid] = h;
  }
  __syncthreads();
  {
    // Rank by counting = stable ascending sort; perm = inverse of the rank. Every thread counts a
    // slice of the other channels for its own (NPG threads per channel, hashes read four at a
    // time); the slices meet in an integer LDS add.
    constexpr int SL = D / NPG;
    uint32_t* rank_lds = code_lds;
    const int first = pg * SL;
    const uint32_t mine = hash_lds[c];
    uint32_t cnt = 0;
#pragma unroll
    for (int o4 = 0; o4 < SL; o4 += 4) {
      const u32x4 h = *(const u32x4*)&hash_lds[first + o4];
#pragma unroll
      for (int j = 0; j < 4; ++j) cnt += (h[j] < mine || (h[j] == mine && first + o4 + j < c)) ? 1u : 0u;
    }
    if (cnt) atomicAdd(&rank_lds[c], cnt);
    __syncthreads();
    if (tid < D) perm_lds[rank_lds[tid]] = (uint8_t)tid;
  }
  __syncthreads();
  if (perm_out && tid < D) perm_out[(size_t)blockIdx.x * D + tid] = perm_lds[tid];
}

hipError_t launch_lsh_group(const void* q, int dtype, const Problem& pb, uint8_t* perm_out,
                            uint32_t* hash_out, hipStream_t stream) {
  if (pb.Br < 1 || pb.Br > kMaxLshRows) return hipErrorInvalidValue;
  const int Tq = (pb.N + pb.Br - 1) / pb.Br;
  const long long units = (long long)pb.B * pb.H * Tq;
  dim3 grid((unsigned)units), block(kLshThreads);
#define DA_LSH_LAUNCH(T, DD)                                                                   \
  hipLaunchKernelGGL((lsh_group_kernel<T, DD>), grid, block, 0, stream, (const T*)q, perm_out, \
                     hash_out, pb.N, pb.Br, Tq, pb.n_planes, pb.gray_mode, pb.seed)
  if (dtype == 0 && pb.d == 64) DA_LSH_LAUNCH(bf16, 64);
  else if (dtype == 0 && pb.d == 128) DA_LSH_LAUNCH(bf16, 128);
  else if (dtype == 1 && pb.d == 64) DA_LSH_LAUNCH(float, 64);
  else if (dtype == 1 && pb.d == 128) DA_LSH_LAUNCH(float, 128);
  else return hipErrorInvalidValue;
#undef DA_LSH_LAUNCH
  return hipGetLastError();
}

}  // namespace da
