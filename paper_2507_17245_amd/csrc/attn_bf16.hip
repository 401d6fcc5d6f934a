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
  // LDS layouts.
  //  * V tiles, and K tiles of the exact path, arrive by direct global->LDS loads (each
  //    wave-level load drops 64 x 16 bytes contiguously), so rows are unpadded (D*2 bytes) and
  //    bank conflicts are avoided by swizzling where a 16-byte chunk sits inside its row:
  //      K (read with 16-byte accesses, 16 lanes = 16 rows at one logical chunk):
  //          chunk' = chunk ^ (row & 15)            (D = 128: 16 chunks per row)
  //          chunk' = chunk ^ ((row >> 1) & 7)      (D = 64: 8 chunks per row, two rows per 256 B)
  //      V (read with transposing 8-byte accesses, 4 rows x 32 bytes per 16 lanes):
  //          32-byte segment' = segment ^ (row & 7)         (D = 128)
  //          32-byte segment' = segment ^ ((row >> 1) & 3)  (D = 64)
  //    The loading lane fetches the global chunk that belongs at its LDS position.
  //  * The fused tile K_f of the distr path is written by the waves themselves: rows padded by
  //    8 elements (16-byte aligned, consecutive rows 4 banks apart).
  //  * The raw K tile of the distr path is only read by 2-byte gathers down a column: an odd
  //    number of dwords per row keeps the 64 rows of a wave on distinct banks.
  static constexpr int ROWB = D * 2;              // bytes of an unpadded row
  static constexpr int TILEB = kBc * ROWB;        // bytes of an unpadded 64-row tile
  static constexpr int KXS = KRED + 8;            // K_f row stride in elements (distr)
  static constexpr int KX_BYTES = DISTR ? kBc * KXS * 2 : TILEB;   // one Kx buffer
  static constexpr int KRS = D + 2;               // raw K tile row stride in elements (distr only)
  static constexpr int SP = KRED / NW;            // fused slots each wave builds per key row
  static constexpr int NGATHER = SP * G;          // 2-byte gathers per lane per tile (= D / NW)
  static constexpr int KSTEPS = KRED / 16;        // MFMA steps of the score product
};

// Tuning switches (compile-time; the defaults are what the library ships with).
#ifndef DA_HINTS
#define DA_HINTS 1          // 1: interleave MFMA / LDS / vector instructions with scheduling groups
#endif
#ifndef DA_KPF
#define DA_KPF 4            // LDS operand reads issued ahead of the first MFMA of a phase
#endif
#ifndef DA_WAVES_PER_EU
#define DA_WAVES_PER_EU 2   // occupancy target (waves per SIMD) given to the register allocator
#endif

// Rows whose running maximum moved by less than this (in log2 units) keep their old reference
// maximum: P is then at most 2^kTau, the sums stay exact ratios, and the accumulator rescale
// (one multiply per accumulator register) is skipped for almost every tile.
constexpr float kTau = 8.0f;

template <int D, int BR, int KRED, bool DISTR>
__global__ __launch_bounds__(BR * 2, DA_WAVES_PER_EU) void attn_bf16_kernel(
    const bf16* __restrict__ q, const bf16* __restrict__ k, const bf16* __restrict__ v,
    bf16* __restrict__ o, const uint8_t* __restrict__ perm, int H, int Hkv, int N, int Tq,
    int causal, float scale_log2e, int total_units) {
  using C = Cfg<D, BR, KRED, DISTR>;
  using kx8 = typename std::conditional<DISTR, f16x8, bf16x8>::type;
  // Kx and V tiles are double-buffered: while tile i multiplies, tile i+1 (V) / i+2 (K) lands.
  // Each buffer is a separate LDS object: the compiler can then tell that the operand reads of
  // one buffer do not depend on the direct loads still in flight into the other.
  __shared__ __attribute__((aligned(1024))) char kx_lds0[C::KX_BYTES];
  __shared__ __attribute__((aligned(1024))) char kx_lds1[C::KX_BYTES];
  __shared__ __attribute__((aligned(1024))) char v_lds0[C::TILEB];
  __shared__ __attribute__((aligned(1024))) char v_lds1[C::TILEB];
  auto kx_buf = [&](int par) -> char* { return par ? kx_lds1 : kx_lds0; };
  auto v_buf = [&](int par) -> char* { return par ? v_lds1 : v_lds0; };
  __shared__ __attribute__((aligned(16))) bf16 kraw_lds[DISTR ? kBc * C::KRS : 8];
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
  kx8 qop[C::KSTEPS];
  if constexpr (DISTR) {
    const bf16* qrow = qh + (size_t)q_ld * D;
#pragma unroll
    for (int s = 0; s < C::KSTEPS; ++s) {
#pragma unroll
      for (int j = 0; j < 8; ++j)
        qop[s][j] = to_half_sat((float)qrow[perm_lds[(16 * s + 8 * hh + j) * C::G]]);
    }
  } else {
#pragma unroll
    for (int s = 0; s < C::KSTEPS; ++s)
      qop[s] = *(const bf16x8*)(qh + (size_t)q_ld * D + 16 * s + 8 * hh);
  }
  // The Q operands must have landed before the loop starts: otherwise the compiler's wait-count
  // bookkeeping carries "Q loads pending" into the loop and the MFMAs also wait for the K/V
  // prefetch of later tiles.
#pragma unroll
  for (int s = 0; s < C::KSTEPS; ++s) asm volatile("" : "+v"(qop[s]));

  // ---- fusion gather offsets (bytes into kraw_lds), fixed for the Q block -------------------
  // Thread (row n = lane, part = wave) builds K_f[n][part*SP .. part*SP+SP-1].
  int goff[DISTR ? C::NGATHER : 1];
  if constexpr (DISTR) {
#pragma unroll
    for (int i = 0; i < C::NGATHER; ++i)
      goff[i] = (lane * C::KRS + perm_lds[wave * C::NGATHER + i]) * 2;
  }

  const int n_end = causal ? min(N, r0 + BR) : N;
  const int n_tiles = (n_end + kBc - 1) / kBc;
  // tiles [0, n_full) need no masking for any row of the block
  const int n_full = causal ? min(r0, N) / kBc : N / kBc;

  // ---- staging: global -> registers -> LDS ---------------------------------------------------
  // K and V rows are fetched through buffer descriptors: the per-lane byte offset inside a
  // tile is fixed, the tile advances through the scalar offset, and rows past the end of the
  // head read as zero (hardware range check), so a tile costs no address arithmetic.
  const unsigned head_bytes = (unsigned)N * D * 2;
  const __amdgpu_buffer_rsrc_t k_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)kh, 0, head_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t v_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)vh, 0, head_bytes, 0x00020000);

  // Direct global->LDS tile loads. Wave-level load j of this wave fills the 1 KB block
  // j*NW + wave of the tile; lane i owns the 16 bytes at offset 16*i of that block, i.e. LDS
  // row (slot / CH), chunk position (slot % CH) with slot = 64*block + i, and fetches the global
  // chunk the swizzle assigns to that position.
  int dma_k[DISTR ? 1 : C::CPT], dma_v[C::CPT];
#pragma unroll
  for (int j = 0; j < C::CPT; ++j) {
    const int slot = (j * C::NW + wave) * 64 + lane;
    const int row = slot / C::CH, pc = slot % C::CH;
    if constexpr (!DISTR) dma_k[j] = row * C::ROWB + (pc ^ (D == 128 ? (row & 15) : ((row >> 1) & 7))) * 16;
    const int lseg = (pc >> 1) ^ (D == 128 ? (row & 7) : ((row >> 1) & 3));
    dma_v[j] = row * C::ROWB + (lseg * 2 + (pc & 1)) * 16;
  }
  typedef __attribute__((address_space(3))) void lds_void;
  auto dma_tile = [&](__amdgpu_buffer_rsrc_t rsrc, int tile, const int* voff, char* dst) {
    const int soff = tile * C::TILEB;
#pragma unroll
    for (int j = 0; j < C::CPT; ++j)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void*)(dst + (j * C::NW + wave) * 1024), 16,
                                               voff[j], soff, 0, 0);
  };
  auto dma_wait = [&]() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); };

  // distr: the raw K tile goes through registers into the gather layout
  u32x4 kst[DISTR ? C::CPT : 1];
  const int st_voff = ((tid / C::CH) * D + (tid % C::CH) * 8) * 2;   // chunk j adds j * (T / CH) rows
  auto load_kraw = [&](int tile) {
    if constexpr (DISTR) {
      const int soff = tile * C::TILEB;
#pragma unroll
      for (int j = 0; j < C::CPT; ++j)
        kst[j] = __builtin_amdgcn_raw_buffer_load_b128(k_rsrc, st_voff + j * (C::T / C::CH) * C::ROWB, soff, 0);
    }
  };
  auto store_kraw = [&]() {
    if constexpr (DISTR) {
#pragma unroll
      for (int j = 0; j < C::CPT; ++j) {
        int id = tid + j * C::T;
        unsigned* dst = (unsigned*)(kraw_lds + (id / C::CH) * C::KRS + (id % C::CH) * 8);
        dst[0] = kst[j][0]; dst[1] = kst[j][1]; dst[2] = kst[j][2]; dst[3] = kst[j][3];
      }
    }
  };
  // ---- fusion (Sec. 3.2): K_f[n][j] = sum of the group's key channels, in float, rounded to
  // half once. Two members are gathered into one register and summed by a bf16 dot product
  // with (1, 1).
  auto fuse = [&](int buf) {
    if constexpr (DISTR) {
      const char* kraw = (const char*)kraw_lds;
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
      f16* dst = (f16*)kx_buf(buf) + lane * C::KXS + wave * C::SP;
      if constexpr (C::SP % 8 == 0) {
#pragma unroll
        for (int c8 = 0; c8 < C::SP / 8; ++c8) {
          f16x8 pk;
#pragma unroll
          for (int j = 0; j < 8; ++j) pk[j] = fused[c8 * 8 + j];
          *(f16x8*)(dst + c8 * 8) = pk;
        }
      } else {
        static_assert(!DISTR || C::SP % 8 == 0 || C::SP == 4, "fused slots per wave: 4 or a multiple of 8");
        f16x4 pk = {fused[0], fused[1], fused[2], fused[3]};
        *(f16x4*)dst = pk;
      }
    }
  };

  // ---- accumulators and softmax state ---------------------------------------------------------
  f32x16 oacc[D / 32];
#pragma unroll
  for (int mb = 0; mb < D / 32; ++mb)
#pragma unroll
    for (int i = 0; i < 16; ++i) oacc[mb][i] = 0.0f;
  float m_ref = -INFINITY;   // reference row max, log2 units (scaled); at most kTau below the true max
  float l_run = 0.0f;        // row sum over this lane's half of the keys, relative to m_ref

  // LDS byte offsets of this lane's operands inside a buffer.
  // Score product, A operand: row lq (+32 per key block), logical chunk 2*s + hh.
  int ka_off[C::KSTEPS];
#pragma unroll
  for (int s = 0; s < C::KSTEPS; ++s) {
    if constexpr (DISTR) ka_off[s] = (lq * C::KXS + 16 * s + 8 * hh) * 2;
    else ka_off[s] = lq * C::ROWB + ((2 * s + hh) ^ (D == 128 ? (lq & 15) : ((lq >> 1) & 7))) * 16;
  }
  // P.V, A operand via transposing reads: lane addresses row 4*hh + (lane%16)/4 (+8, +16*tt),
  // logical 32-byte segment 2*mb + (lane/16)%2, 8-byte piece lane%4 of it.
  int va_off[D / 32];
  {
    const int row_l = 4 * hh + ((lane & 15) >> 2);
    const int swz = D == 128 ? (row_l & 7) : ((row_l >> 1) & 3);
#pragma unroll
    for (int mb = 0; mb < D / 32; ++mb)
      va_off[mb] = row_l * C::ROWB + ((2 * mb + ((lane >> 4) & 1)) ^ swz) * 32 + 8 * (lane & 3);
  }

  // S^T = Kx . Qx^T for the Kx tile in buffer `buf`: register i of block mb holds key
  // 32*mb + 8*(i/4) + 4*hh + i%4 of the tile.
  auto qk = [&](int buf, f32x16 (&sacc)[2]) {
    const char* base = kx_buf(buf);
    constexpr int MB_STEP = 32 * (DISTR ? C::KXS * 2 : C::ROWB);
#pragma unroll
    for (int mb = 0; mb < 2; ++mb) {
#pragma unroll
      for (int i = 0; i < 16; ++i) sacc[mb][i] = 0.0f;
#pragma unroll
      for (int s = 0; s < C::KSTEPS; ++s) {
#ifdef DA_ABL_NOKREAD
        kx8 a = qop[(s + 1) % C::KSTEPS];
#else
        kx8 a = *(const kx8*)(base + ka_off[s] + mb * MB_STEP);
#endif
        sacc[mb] = mfma_32x32x16(a, qop[s], sacc[mb]);
      }
    }
  };

  // Softmax bookkeeping for the scores `sc` of tile `tile`, before they are exponentiated: mask,
  // row maximum, and -- only when some row's maximum ran more than kTau ahead of its reference --
  // a new reference with the matching rescale of the row sum and of the output accumulator.
  auto row_max = [&](auto mask_c, int tile, f32x16 (&sc)[2]) -> float {
    if constexpr (decltype(mask_c)::value) {
      const int lim = causal ? min(q_abs, N - 1) : N - 1;  // last visible key of this row
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          int kv = tile * kBc + 32 * mb + 8 * (i >> 2) + 4 * hh + (i & 3);
          if (kv > lim) sc[mb][i] = -INFINITY;
        }
    }
    float mt = sc[0][0];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int i = 0; i < 16; ++i) mt = fmaxf(mt, sc[mb][i]);
    return half_swap_max(mt) * scale_log2e;
  };
  auto move_reference = [&](float mt) {
    const bool moved = mt > m_ref + kTau;
    if (__builtin_amdgcn_ballot_w64(moved) != 0) {
      const float m_new = moved ? mt : m_ref;
      const float alpha = __builtin_amdgcn_exp2f(m_ref - m_new);   // exp2(-inf) = 0 on the first tile
      m_ref = m_new;
      l_run *= alpha;
#pragma unroll
      for (int mb = 0; mb < D / 32; ++mb)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[mb][i] *= alpha;
    }
  };

  // One tile `it`, whose scores `sc` already went through row_max / move_reference:
  //   phase X: scores of tile it+1 into `sn` (matrix pipe)  ||  exp, bf16 P, row sum of `sc` (vector ALUs)
  //   phase Y: O^T += V^T . P^T for tile it (matrix pipe)    ||  mask and row maximum of `sn` (vector ALUs)
  // then the rare reference move for tile it+1, the LDS stores of the prefetched tiles, one barrier.
  // The scheduling hints at the end ask the compiler to interleave the two instruction streams
  // instead of emitting them one after the other.
  auto body = [&](auto mask_next_c, auto next_c, int it, int par, f32x16 (&sc)[2], f32x16 (&sn)[2]) {
    constexpr bool HAS_NEXT = decltype(next_c)::value;
    // The buffers these loads fill were last read in the previous iteration, which every wave
    // has left (barrier): K(it+2) replaces K(it), V(it+1) replaces V(it-1).
    if constexpr (HAS_NEXT) {
      if constexpr (DISTR) load_kraw(it + 2);
      else dma_tile(k_rsrc, it + 2, dma_k, kx_buf(par));
      dma_tile(v_rsrc, it + 1, dma_v, v_buf(par ^ 1));
    }
    if constexpr (HAS_NEXT) qk(par ^ 1, sn);
    // The row sum is taken over the bf16-rounded P, the values P.V really uses (one bf16 dot
    // product with (1, 1) per register pair): numerator and denominator then carry the same
    // rounding, which cancels for rows dominated by few keys.
    bf16x8 pop[4];
    {
      const bf16x2 ones = {(bf16)1.0f, (bf16)1.0f};
      float rs0 = 0.0f, rs1 = 0.0f;
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int i = 0; i < 16; i += 2) {
#ifdef DA_ABL_NOEXP
          float p0 = __builtin_fmaf(sc[mb][i], scale_log2e, -m_ref);
          float p1 = __builtin_fmaf(sc[mb][i + 1], scale_log2e, -m_ref);
#else
          float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[mb][i], scale_log2e, -m_ref));
          float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[mb][i + 1], scale_log2e, -m_ref));
#endif
          bf16x2 pr = {(bf16)p0, (bf16)p1};
          pop[mb * 2 + (i >> 3)][i & 7] = pr[0];
          pop[mb * 2 + (i >> 3)][(i & 7) + 1] = pr[1];
          if (i & 2) rs1 = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, rs1, false);
          else rs0 = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, rs0, false);
        }
      l_run += rs0 + rs1;
    }
    // ---- O^T += V^T . P^T: step tt covers keys 16*tt + {8*(j/4) + 4*hh + j%4} of the tile,
    // i.e. V rows 16*tt + 4*hh + 0..3 and 16*tt + 8 + 4*hh + 0..3.
    const char* vb = v_buf(par);
#pragma unroll
    for (int tt = 0; tt < 4; ++tt) {
#pragma unroll
      for (int mb = 0; mb < D / 32; ++mb) {
        const char* p0 = vb + va_off[mb] + 16 * tt * C::ROWB;
#ifdef DA_ABL_NOVREAD
        bf16x8 a = pop[(tt + mb + 1) & 3];
        (void)p0;
#else
        bf16x8 a = lds_read_tr_pair((const bf16*)p0, (const bf16*)(p0 + 8 * C::ROWB));
#endif
        oacc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pop[tt], oacc[mb], 0, 0, 0);
      }
    }
    float mt_next = 0.0f;
    if constexpr (HAS_NEXT) mt_next = row_max(mask_next_c, it + 1, sn);
    // ---- scheduling hints (groups are filled in this order) -----------------------------------
    // One MFMA occupies the issue port for 8 cycles and the matrix pipe for 32: up to 6 vector
    // instructions fit beside it. Operands are fetched from LDS four MFMAs ahead.
#if DA_HINTS
    {
      constexpr int N_QK = HAS_NEXT ? 2 * C::KSTEPS : 0;
      constexpr int N_PV = D / 8;
      constexpr int VALU_PER_MFMA = (150 + N_QK + N_PV - 1) / (N_QK + N_PV);
      constexpr int PF = DA_KPF < N_QK ? DA_KPF : N_QK;
      __builtin_amdgcn_sched_group_barrier(0x100, HAS_NEXT ? PF : 2 * DA_KPF, 0);
#pragma unroll
      for (int i = 0; i < N_QK - PF; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);        // one score MFMA
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);        // a K operand, PF MFMAs ahead
        __builtin_amdgcn_sched_group_barrier(0x402, VALU_PER_MFMA, 0);
      }
#pragma unroll
      for (int i = 0; i < PF; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);        // one score MFMA
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);        // K operands are all in: first V operands
        __builtin_amdgcn_sched_group_barrier(0x402, VALU_PER_MFMA, 0);
      }
#pragma unroll
      for (int i = 0; i < N_PV; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);        // one P.V MFMA
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);        // next V operand
        __builtin_amdgcn_sched_group_barrier(0x402, VALU_PER_MFMA, 0);
      }
    }
#endif
    if constexpr (HAS_NEXT) {
      move_reference(mt_next);
      if constexpr (DISTR) {   // raw K(it+2) -> gather layout -> fused tile K_f(it+2)
        store_kraw();
        __syncthreads();
        fuse(par);
      }
      dma_wait();              // this wave's direct loads have landed
    }
#ifndef DA_ABL_NOBARRIER
    __syncthreads();
#endif
  };

  // ---- prologue: tiles 0 (K, V) and 1 (K) into LDS, scores of tile 0 ---------------------------
  dma_tile(v_rsrc, 0, dma_v, v_lds0);
  if constexpr (DISTR) {
    load_kraw(0);
    store_kraw();
    __syncthreads();
    fuse(0);
    if (n_tiles > 1) {
      load_kraw(1);
      __syncthreads();   // every wave is done gathering tile 0
      store_kraw();
      __syncthreads();
      fuse(1);
    }
  } else {
    dma_tile(k_rsrc, 0, dma_k, kx_lds0);
    if (n_tiles > 1) dma_tile(k_rsrc, 1, dma_k, kx_lds1);
  }
  dma_wait();
  __syncthreads();

  const std::true_type yes;
  const std::false_type no;
  f32x16 s0[2], s1[2];
  qk(0, s0);
  move_reference(row_max(yes, 0, s0));

  // Tile it+1 needs no mask while it+1 < n_full. The main loop is unrolled by two so that the
  // two score register sets swap roles without copies.
  int it = 0;
  for (; it + 2 < n_full; it += 2) {
    body(no, yes, it, 0, s0, s1);
    body(no, yes, it + 1, 1, s1, s0);
  }
  for (; it < n_tiles - 1; ++it) {   // at most two unmasked leftovers plus the masked tiles
    body(yes, yes, it, it & 1, s0, s1);
#pragma unroll
    for (int mb = 0; mb < 2; ++mb) s0[mb] = s1[mb];
  }
  body(no, no, it, it & 1, s0, s1);

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
