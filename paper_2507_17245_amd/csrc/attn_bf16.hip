// Tiled bf16 attention forward for gfx950 (CDNA4): exact attention (Sec. 2.1, tiled as in
// Sec. 2.2.2) and DistrAttention (Sec. 3.1 Eq. 2, Sec. 3.2 sampling and fusion, Sec. 3.3
// block-wise grouping) from one template.
//
// Work split. One workgroup owns one Q block of BR rows of one (batch, head); each of its
// BR/32 wavefronts owns 32 query rows for the whole inner loop over K/V tiles of 64 rows.
//
// Matrix-core mapping (v_mfma_f32_32x32x16_bf16, fp32 accumulate). Both products are taken
// transposed so that one lane owns one query row's softmax state:
//   S^T[kv][q] = sum_c  Kx[kv][c] * Qx[q][c]      A = Kx tile rows from LDS, B = Qx in registers
//   O^T[ch][q] = sum_kv V[kv][ch] * P^T[kv][q]    A = V^T via LDS transpose reads, B = P^T in registers
// The accumulator layout of the first product (lane = q, registers = kv) is, after conversion
// to bf16, exactly the B-operand layout of the second, so P never leaves registers; the
// contraction index kv is enumerated in the accumulator's order on both operands.
//   exact:  Kx = K tile,  Qx = Q,    contraction over d channels
//   distr:  Kx = K_f tile (Sec. 3.2 fusion: sum of the group's K channels, built once per
//           (Q block, K tile) in LDS by all waves together), Qx = Q_r (sampling: the group's
//           first channel in sorted order, gathered once per Q block), contraction over
//           n_groups = d / G*.
// Online softmax (running max, running sum, rescaled accumulator) follows the block-wise
// scheme of Sec. 2.2.2 in the exp2 domain.
#include <type_traits>

#include "da_common.h"

namespace da {

namespace {

typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef _Float16 f16;
typedef __attribute__((ext_vector_type(4))) _Float16 f16x4;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;

// Largest finite half; sampled queries and fused keys of the distr path are clamped to it.
constexpr float kHalfMax = 65504.0f;
__device__ inline f16 to_half_sat(float x) { return (f16)__builtin_amdgcn_fmed3f(x, -kHalfMax, kHalfMax); }

__device__ inline f32x16 mfma_32x32x16(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
__device__ inline f32x16 mfma_32x32x16(f16x8 a, f16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
}

__device__ inline bf16x8 lds_read_tr_pair(const bf16* p0, const bf16* p1) {
  // Two transposing LDS reads (ds_read_b64_tr_b16): within each group of 16 lanes, lane i
  // receives element (i % 4) of the 8-byte chunks addressed by lanes 4j + i/4, j = 0..3.
  s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p0);
  s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p1);
  s16x8 r = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
  return __builtin_bit_cast(bf16x8, r);
}

// Exchange between the wave halves: v_permlane32_swap swaps the upper 32 lanes of its first
// operand with the lower 32 lanes of its second; fed the same value twice it leaves, in every
// lane, the values of lanes l % 32 (first operand) and l % 32 + 32 (second operand). Written as
// inline asm with both registers read-write: the builtin's second result was dropped by the
// compiler when both inputs were the same value. The s_nop covers the VALU-write -> permlane
// read hazard, which the compiler cannot see inside an asm block.
__device__ inline void half_pair(float x, float& lo, float& hi) {
  float a = x, b = x;
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
  lo = a;
  hi = b;
}
__device__ inline float half_swap_max(float x) {
  float lo, hi;
  half_pair(x, lo, hi);
  return fmaxf(lo, hi);
}
__device__ inline float half_swap_sum(float x) {
  float lo, hi;
  half_pair(x, lo, hi);
  return lo + hi;
}

template <int D, int BR, int KRED, bool DISTR>
struct Cfg {
  static constexpr int NW = BR / 32;              // wavefronts per workgroup
  static constexpr int T = NW * 64;               // threads
  static constexpr int G = D / KRED;              // channels per group
  static constexpr int CH = D / 8;                // 16-byte chunks per row
  static constexpr int CPT = kBc * CH / T;        // chunks each thread stages per tile
  // LDS row strides in elements. Raw K of the distr path is only read by 2-byte gathers down a
  // column: an odd number of dwords per row keeps 64 rows on distinct banks. Rows read by
  // 16-byte accesses need 16-byte alignment; +8 elements shifts consecutive rows by 4 banks.
  // V is read by transposing 8-byte accesses, 4 rows x 64 bytes per half wave: +32 elements.
  static constexpr int KS = DISTR ? D + 2 : D + 8;
  static constexpr int KFS = KRED + 8;
  static constexpr int VS = D + 32;
  static constexpr int SP = KRED / NW;            // fused slots each wave builds per key row
  static constexpr int NGATHER = SP * G;          // 2-byte gathers per lane per tile (= D / NW)
};

template <int D, int BR, int KRED, bool DISTR>
__global__ __launch_bounds__(BR * 2, 2) void attn_bf16_kernel(
    const bf16* __restrict__ q, const bf16* __restrict__ k, const bf16* __restrict__ v,
    bf16* __restrict__ o, const uint8_t* __restrict__ perm, int H, int Hkv, int N, int Tq,
    int causal, float scale_log2e, int total_units) {
  using C = Cfg<D, BR, KRED, DISTR>;
  __shared__ __attribute__((aligned(16))) bf16 k_lds[kBc * C::KS];
  __shared__ __attribute__((aligned(16))) bf16 v_lds[kBc * C::VS];
  __shared__ __attribute__((aligned(16))) f16 kf_lds[DISTR ? kBc * C::KFS : 8];
  __shared__ uint8_t perm_lds[DISTR ? D : 4];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lq = lane & 31;   // query row of this lane inside the wave's 32 rows
  const int hh = lane >> 5;   // which half of each 8-wide contraction chunk this lane feeds

  // Workgroup -> (batch*head, Q block). Consecutive workgroup ids go round-robin over the 8
  // XCDs; remap so that each XCD walks a contiguous range of units and the Q blocks of one
  // head share that XCD's L2 for K and V. Causal blocks are taken longest first.
  int unit = blockIdx.x;
  if ((total_units & 7) == 0) unit = (blockIdx.x & 7) * (total_units >> 3) + (blockIdx.x >> 3);
  const int bh = unit / Tq;
  int t = unit % Tq;
  if (causal) t = Tq - 1 - t;
  const int b = bh / H, h = bh % H;
  const int hk = h / (H / Hkv);
  const int r0 = t * BR;

  const bf16* qh = q + (size_t)bh * N * D;
  const bf16* kh = k + (size_t)(b * Hkv + hk) * N * D;
  const bf16* vh = v + (size_t)(b * Hkv + hk) * N * D;

  const int qw0 = r0 + wave * 32;              // first query row of this wave
  const int q_abs = qw0 + lq;                  // this lane's query row
  const int q_ld = min(q_abs, N - 1);          // ragged block: load a valid row, never store it

  if constexpr (DISTR) {
    const size_t pbase = ((size_t)bh * Tq + t) * D;
    for (int i = tid; i < D; i += C::T) perm_lds[i] = perm[pbase + i];
    __syncthreads();
  }

  // ---- Q operands, held for the whole inner loop ------------------------------------------
  // distr: the reduced product runs on the f16 matrix path. A bf16 value converts to half
  // exactly (8 vs 11 significand bits) inside half's exponent range, and the fused keys, rounded
  // once from their float sum, keep 3 more bits than bf16 would: with bf16 K_f the logit error
  // on inputs with heavy-tailed channel scales exceeds what the output tolerance allows.
  using kx8 = typename std::conditional<DISTR, f16x8, bf16x8>::type;
  kx8 qop[KRED / 16];
  if constexpr (DISTR) {
    const bf16* qrow = qh + (size_t)q_ld * D;
#pragma unroll
    for (int s = 0; s < KRED / 16; ++s) {
#pragma unroll
      for (int j = 0; j < 8; ++j)
        qop[s][j] = to_half_sat((float)qrow[perm_lds[(16 * s + 8 * hh + j) * C::G]]);
    }
  } else {
#pragma unroll
    for (int s = 0; s < KRED / 16; ++s)
      qop[s] = *(const bf16x8*)(qh + (size_t)q_ld * D + 16 * s + 8 * hh);
  }

  // ---- fusion gather offsets (bytes into k_lds), fixed for the Q block ----------------------
  // Thread (row n = tid % 64, part = wave) builds K_f[n][part*SP .. part*SP+SP-1].
  int goff[DISTR ? C::NGATHER : 1];
  if constexpr (DISTR) {
#pragma unroll
    for (int i = 0; i < C::NGATHER; ++i)
      goff[i] = (lane * C::KS + perm_lds[wave * C::NGATHER + i]) * 2;
  }

  // ---- staging registers: global -> registers -> LDS -----------------------------------------
  u32x4 kst[C::CPT], vst[C::CPT];
  auto stage_load = [&](int n0) {
#pragma unroll
    for (int j = 0; j < C::CPT; ++j) {
      int id = tid + j * C::T;
      int row = min(n0 + id / C::CH, N - 1);
      int col = (id % C::CH) * 8;
      kst[j] = *(const u32x4*)(kh + (size_t)row * D + col);
      vst[j] = *(const u32x4*)(vh + (size_t)row * D + col);
    }
  };
  auto stage_store = [&]() {
#pragma unroll
    for (int j = 0; j < C::CPT; ++j) {
      int id = tid + j * C::T;
      int row = id / C::CH, col = (id % C::CH) * 8;
      if constexpr (DISTR) {
        unsigned* dst = (unsigned*)(k_lds + row * C::KS + col);
        dst[0] = kst[j][0]; dst[1] = kst[j][1]; dst[2] = kst[j][2]; dst[3] = kst[j][3];
      } else {
        *(u32x4*)(k_lds + row * C::KS + col) = kst[j];
      }
      *(u32x4*)(v_lds + row * C::VS + col) = vst[j];
    }
  };

  // ---- accumulators and softmax state ---------------------------------------------------------
  f32x16 oacc[D / 32];
#pragma unroll
  for (int mb = 0; mb < D / 32; ++mb)
#pragma unroll
    for (int i = 0; i < 16; ++i) oacc[mb][i] = 0.0f;
  float m_run = -INFINITY;   // running row max, in log2 units (already scaled)
  float l_run = 0.0f;        // running row sum over this lane's half of the keys

  const int n_end = causal ? min(N, r0 + BR) : N;
  const int n_tiles = (n_end + kBc - 1) / kBc;

  // LDS addresses that do not change across tiles
  using kx_t = typename std::conditional<DISTR, f16, bf16>::type;
  const kx_t* ka_base;
  if constexpr (DISTR) ka_base = kf_lds + lq * C::KFS + 8 * hh;
  else ka_base = k_lds + lq * C::KS + 8 * hh;
  const bf16* vt_base = v_lds + (((lane & 15) >> 2) + 4 * hh) * C::VS + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);

  stage_load(0);
  stage_store();
  __syncthreads();

  for (int it = 0; it < n_tiles; ++it) {
    const int n0 = it * kBc;
    if (it + 1 < n_tiles) stage_load(n0 + kBc);

    if constexpr (DISTR) {
      // ---- fusion (Sec. 3.2): K_f[n][j] = sum of the group's key channels, in float, rounded
      // to half once. The two members of a pair are gathered into one register and summed by a
      // bf16 dot product with (1, 1).
      const char* kraw = (const char*)k_lds;
      const bf16x2 ones = {(bf16)1.0f, (bf16)1.0f};
      f16 fused[C::SP];
#pragma unroll
      for (int sl = 0; sl < C::SP; ++sl) {
        if constexpr (C::G == 1) {
          fused[sl] = to_half_sat((float)*(const bf16*)(kraw + goff[sl]));
        } else {
          float acc = 0.0f;
#pragma unroll
          for (int g = 0; g < C::G; g += 2) {
            bf16x2 pr = {*(const bf16*)(kraw + goff[sl * C::G + g]),
                         *(const bf16*)(kraw + goff[sl * C::G + g + 1])};
            acc = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, acc, false);
          }
          fused[sl] = to_half_sat(acc);
        }
      }
      f16* dst = kf_lds + lane * C::KFS + wave * C::SP;
      if constexpr (C::SP % 8 == 0) {
#pragma unroll
        for (int c8 = 0; c8 < C::SP / 8; ++c8) {
          f16x8 pk;
#pragma unroll
          for (int j = 0; j < 8; ++j) pk[j] = fused[c8 * 8 + j];
          *(f16x8*)(dst + c8 * 8) = pk;
        }
      } else {
        static_assert(C::SP == 4, "fused slots per wave must be 4 or a multiple of 8");
        f16x4 pk = {fused[0], fused[1], fused[2], fused[3]};
        *(f16x4*)dst = pk;
      }
      __syncthreads();
    }

    // wave-uniform: does this wave see any key of the tile, and does it need masking?
    const bool wave_active = !causal || n0 <= qw0 + 31;
    if (wave_active) {
      // ---- S^T = Kx . Qx^T ---------------------------------------------------------------------
      f32x16 sacc[2];
#pragma unroll
      for (int mb = 0; mb < 2; ++mb) {
#pragma unroll
        for (int i = 0; i < 16; ++i) sacc[mb][i] = 0.0f;
#pragma unroll
        for (int s = 0; s < KRED / 16; ++s) {
          kx8 a = *(const kx8*)(ka_base + mb * 32 * (DISTR ? C::KFS : C::KS) + 16 * s);
          sacc[mb] = mfma_32x32x16(a, qop[s], sacc[mb]);
        }
      }
      // register i of block mb holds key  n0 + 32*mb + 8*(i/4) + 4*hh + i%4
      const bool need_mask = (n0 + kBc > N) || (causal && n0 + kBc - 1 > qw0);
      if (need_mask) {
        const int lim = causal ? min(q_abs, N - 1) : N - 1;  // last visible key of this row
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            int kv = n0 + 32 * mb + 8 * (i >> 2) + 4 * hh + (i & 3);
            if (kv > lim) sacc[mb][i] = -INFINITY;
          }
      }
      // ---- online softmax ---------------------------------------------------------------------
      float mt = sacc[0][0];
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int i = 0; i < 16; ++i) mt = fmaxf(mt, sacc[mb][i]);
      mt = half_swap_max(mt);
      const float m_new = fmaxf(m_run, mt * scale_log2e);
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
      m_run = m_new;
      float rs = 0.0f;
      bf16x8 pop[4];
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          float p = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[mb][i], scale_log2e, -m_new));
          rs += p;
          pop[mb * 2 + (i >> 3)][i & 7] = (bf16)p;
        }
      l_run = l_run * alpha + rs;
      if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
        for (int mb = 0; mb < D / 32; ++mb)
#pragma unroll
          for (int i = 0; i < 16; ++i) oacc[mb][i] *= alpha;
      }
      // ---- O^T += V^T . P^T ---------------------------------------------------------------------
      // step tt covers the 16 keys n0 + 16*tt + {8*(j/4) + 4*hh + j%4}: rows 16*tt + 4*hh + 0..3
      // and 16*tt + 8 + 4*hh + 0..3 of the V tile.
#pragma unroll
      for (int tt = 0; tt < 4; ++tt) {
#pragma unroll
        for (int mb = 0; mb < D / 32; ++mb) {
          const bf16* p0 = vt_base + (16 * tt) * C::VS + 32 * mb;
          bf16x8 a = lds_read_tr_pair(p0, p0 + 8 * C::VS);
          oacc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pop[tt], oacc[mb], 0, 0, 0);
        }
      }
    }
    __syncthreads();   // every wave is done reading this tile
    if (it + 1 < n_tiles) {
      stage_store();
      __syncthreads();
    }
  }

  // ---- epilogue: O = O_acc / l, bf16, 8-byte stores ---------------------------------------------
  const float l_tot = half_swap_sum(l_run);
  const float inv = 1.0f / l_tot;
  if (q_abs < N) {
    bf16* orow = o + ((size_t)bh * N + q_abs) * D;
#pragma unroll
    for (int mb = 0; mb < D / 32; ++mb)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        bf16x4 pk;
#pragma unroll
        for (int j = 0; j < 4; ++j) pk[j] = (bf16)(oacc[mb][4 * i4 + j] * inv);
        *(bf16x4*)(orow + 32 * mb + 8 * i4 + 4 * hh) = pk;
      }
  }
}

template <int D, int BR, int KRED, bool DISTR>
hipError_t launch_one(const void* q, const void* k, const void* v, void* o, const uint8_t* perm,
                      const Problem& pb, hipStream_t stream) {
  const int Tq = (pb.N + BR - 1) / BR;
  const long long units = (long long)pb.B * pb.H * Tq;
  const float scale_log2e = pb.scale * 1.4426950408889634f;
  hipLaunchKernelGGL((attn_bf16_kernel<D, BR, KRED, DISTR>), dim3((unsigned)units), dim3(BR * 2), 0,
                     stream, (const bf16*)q, (const bf16*)k, (const bf16*)v, (bf16*)o, perm, pb.H,
                     pb.Hkv, pb.N, Tq, pb.causal, scale_log2e, (int)units);
  return hipGetLastError();
}

template <int D, int BR>
hipError_t dispatch_kred(const void* q, const void* k, const void* v, void* o, const uint8_t* perm,
                         const Problem& pb, int distr, hipStream_t stream) {
  if (!distr) return launch_one<D, BR, D, false>(q, k, v, o, perm, pb, stream);
  switch (pb.n_groups) {
    case 16: return launch_one<D, BR, 16, true>(q, k, v, o, perm, pb, stream);
    case 32: return launch_one<D, BR, 32, true>(q, k, v, o, perm, pb, stream);
    case 64: return launch_one<D, BR, 64, true>(q, k, v, o, perm, pb, stream);
    case 128:
      if constexpr (D == 128) return launch_one<D, BR, 128, true>(q, k, v, o, perm, pb, stream);
      [[fallthrough]];
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

bool attn_bf16_supported(const Problem& pb, int distr) {
  if (pb.d != 64 && pb.d != 128) return false;
  if (pb.Br != 64 && pb.Br != 128) return false;
  if (distr) {
    const int kr = pb.n_groups;
    if (kr != 16 && kr != 32 && kr != 64 && kr != 128) return false;
    if (kr > pb.d || pb.d % kr != 0) return false;
    if (kr / (pb.Br / 32) < 4) return false;   // each wave builds at least 4 fused slots per key row
  }
  return true;
}

hipError_t launch_attn_bf16(const void* q, const void* k, const void* v, void* o, const uint8_t* perm,
                            const Problem& pb, int distr, hipStream_t stream) {
  if (!attn_bf16_supported(pb, distr)) return hipErrorInvalidValue;
  if (pb.d == 64 && pb.Br == 64) return dispatch_kred<64, 64>(q, k, v, o, perm, pb, distr, stream);
  if (pb.d == 64 && pb.Br == 128) return dispatch_kred<64, 128>(q, k, v, o, perm, pb, distr, stream);
  if (pb.d == 128 && pb.Br == 64) return dispatch_kred<128, 64>(q, k, v, o, perm, pb, distr, stream);
  return dispatch_kred<128, 128>(q, k, v, o, perm, pb, distr, stream);
}

}  // namespace da
