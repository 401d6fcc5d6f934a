// Tiled bf16 attention forward for gfx950 (CDNA4): exact attention (Sec. 2.1, tiled as in
// Sec. 2.2.2) and DistrAttention (Sec. 3.1 Eq. 2, Sec. 3.2 sampling and fusion, Sec. 3.3
// block-wise grouping) from one template.
//
// Work split. One workgroup owns one Q block of BR rows of one (batch, head); each of its
// BR/32 wavefronts owns 32 query rows for the whole inner loop over K/V tiles of BC rows
// (the paper's l and m: BR in {64, 128, 256}, BC in {32, 64, 128}).
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
//           (Q block, K tile) by all waves together: packed half adds in registers on pieces of
//           a transposed half-precision copy of K, result in LDS), Qx = Q_r (sampling: the
//           group's first channel in sorted order, gathered once per Q block), contraction over
//           n_groups = d / G*, on the f16 matrix path. The grouping itself (Sec. 3.2 LSH, sort,
//           groups) is either read from a table or computed by the workgroup in its prologue.
// Online softmax (reference max, row sum, rescaled accumulator) follows the block-wise scheme of
// Sec. 2.2.2 in the exp2 domain.
//
// Pipeline (one barrier per tile): K (exact) and V tiles reach LDS by direct global->LDS loads
// two tiles (K) / one tile (V) ahead, the K^T pieces of the fusion reach registers one tile
// ahead of their use; while the vector ALUs exponentiate tile i the matrix pipe computes the
// scores of tile i+1; P.V of tile i follows with its V operands read four ahead of their MFMAs.
// The reference of the online softmax moves only when a tile's row sum says it must (no row
// maximum per tile).
#pragma once
#include <type_traits>

#include "da_common.h"

namespace da {

namespace {

typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef _Float16 f16;
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

// Two transposing LDS reads (ds_read_b64_tr_b16): within each group of 16 lanes, lane i
// receives element (i % 4) of the 8-byte chunks addressed by lanes 4j + i/4, j = 0..3.
template <typename V8>
__device__ inline V8 lds_read_tr_pair(const void* p0, const void* p1) {
  s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p0);
  s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p1);
  s16x8 r = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
  return __builtin_bit_cast(V8, r);
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

// Swizzle of the 32-byte segments of a tile that is read with transposing accesses
// (ds_read_b64_tr_b16): the LDS serves 32 lanes of such a read per cycle, which address the rows
// r..r+3 (r a multiple of 4) at two adjacent 32-byte segments, 4 lanes x 8 bytes per row and
// segment. v_swizzle spreads those 4 rows x 2 segments over all 64 banks (no conflict cycles in
// the hardware counters): with 256-byte rows the row picks one of four segment pairs, with
// 128-byte rows two consecutive rows already sit in opposite bank halves and only rows of equal
// parity need separating.
template <int ROW_BYTES>
__device__ inline int v_swizzle(int row) {
  static_assert(ROW_BYTES == 256 || ROW_BYTES == 128, "row length");
  return ROW_BYTES == 256 ? ((row & 3) << 1) : (row & 2);
}
// The fused tile K_f^T (rows of 2*BC bytes, one per group) is read with the same transposing
// accesses and takes the same swizzle as a V tile with rows of that length; rows of 64 bytes
// (BC = 32) hold two segments, exchanged on every second pair of rows.
template <int BC>
__device__ inline int kf_swizzle(int row) {
  if constexpr (BC == 64) return v_swizzle<128>(row);
  else if constexpr (BC == 128) return v_swizzle<256>(row);
  else return (row >> 1) & 1;
}

// KRED: contraction length of the score product (a multiple of the MFMA step, 16). NG: number of
// channel groups; smaller than KRED only for n_groups 4 and 8, whose operands are zero-padded to 16.
template <int D, int BR, int BC, int KRED, bool DISTR, int NG = KRED>
struct Cfg {
  static constexpr int NW = BR / 32;              // wavefronts per workgroup
  static constexpr int T = NW * 64;               // threads
  static constexpr int G = D / NG;                // channels per group
  static constexpr int CH = D / 8;                // 16-byte chunks per row
  static constexpr int MB = BC / 32;              // 32-key blocks of the score product per tile
  static constexpr int TT = BC / 16;              // 16-key steps of P.V per tile
  static constexpr int NBLK = BC * CH / 64;       // 1 KB blocks (one wave-level direct load each) per tile
  static constexpr int CPT = (NBLK + NW - 1) / NW;  // direct loads each wave issues per tile
  // LDS layouts.
  //  * V tiles, and K tiles of the exact path, arrive by direct global->LDS loads (each
  //    wave-level load drops 64 x 16 bytes contiguously), so rows are unpadded (D*2 bytes) and
  //    bank conflicts are avoided by swizzling where a 16-byte chunk sits inside its row:
  //      K (read with 16-byte accesses, 16 lanes = 16 rows at one logical chunk):
  //          chunk' = chunk ^ (row & 15)            (D = 128: 16 chunks per row)
  //          chunk' = chunk ^ ((row >> 1) & 7)      (D = 64: 8 chunks per row, two rows per 256 B)
  //      V (read with transposing 8-byte accesses; the LDS serves 32 lanes per cycle, which
  //      address 4 rows x 2 adjacent 32-byte segments and must cover all 256 bytes of banks):
  //          32-byte segment' = segment ^ 2*(row & 3)       (D = 128: 8 segments per row)
  //          32-byte segment' = segment ^ (row & 2)         (D = 64: 4 segments per row, rows of
  //                                                          opposite parity sit in opposite bank halves)
  //    The loading lane fetches the global chunk that belongs at its LDS position.
  //  * distr path: the keys arrive transposed and in half precision (K^T in global memory, one
  //    row of BC keys = 2*BC bytes per channel and tile, written once per forward by the key
  //    pre-pass). Only the fused tile K_f^T (one such row per group) lives in LDS: written by
  //    the waves, read back with transposing accesses, segments swizzled by kf_swizzle.
  static constexpr int ROWB = D * 2;              // bytes of an unpadded K / V row
  static constexpr int TILEB = BC * ROWB;         // bytes of an unpadded tile
  static constexpr int KTROWB = BC * 2;           // bytes of a K^T / K_f^T row (BC keys)
  static constexpr int PPR = BC / 8;              // 16-byte pieces (8 keys) per K^T / K_f^T row
  static constexpr int KX_BYTES = DISTR ? KRED * KTROWB : TILEB;   // one Kx buffer: K_f^T or K
  static constexpr int FUSE_OUT = (NG * PPR + T - 1) / T;   // 16-byte fused outputs per thread and tile
  static constexpr int KSTEPS = KRED / 16;        // MFMA steps of the score product
  // Register budget: two waves per SIMD, except the widest tile at d = 128, whose two score sets
  // (128 registers) leave room for one.
  static constexpr int WAVES_PER_SIMD = (BC == 128 && D == 128) ? 1 : 2;
};

// Lazy reference maximum. A row keeps its reference until one of its scores runs more than kTau
// (log2 units) ahead of it: P is then at most 2^kTau, numerator and denominator share the
// reference, so the result is the same ratio, and the accumulator rescale (one multiply per
// accumulator register) almost never runs. The test needs no row maximum: a lane's row sum over
// the BC/2 keys it owns in a tile exceeds (BC/2) * 2^kTau only if one of them exceeds 2^kTau (an
// overflowed or NaN sum fails the comparison too), and the sum is needed anyway.
constexpr float kTau = 8.0f;

template <int D, int BR, int BC, int KRED, bool DISTR, int NG>
__global__ __launch_bounds__(BR * 2, (Cfg<D, BR, BC, KRED, DISTR, NG>::WAVES_PER_SIMD)) void attn_bf16_kernel(
    const bf16* __restrict__ q, const bf16* __restrict__ k, const bf16* __restrict__ v,
    bf16* __restrict__ o, const uint8_t* __restrict__ perm, const f16* __restrict__ kt, int Npad,
    int H, int Hkv, int N, int Nk, int Tq, int causal, float scale_log2e, int total_units, int n_planes,
    int gray_mode, uint64_t lsh_seed, float* __restrict__ lse, const char* __restrict__ rtab,
    uint8_t* __restrict__ perm_w) {
  using C = Cfg<D, BR, BC, KRED, DISTR, NG>;
  constexpr float kSumTrigger = (BC / 2) * 256.0f;   // BC/2 keys per lane and tile, each at most 2^kTau
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
  // The block's permutation is only needed while the prologue builds the sampled-query operands
  // and the fusion offsets: it borrows the head of the second V buffer, which receives its
  // first tile in the first loop iteration (after the prologue's barriers).
  uint8_t* perm_lds = (uint8_t*)v_lds1;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lq = lane & 31;   // query row of this lane inside the wave's 32 rows
  const int hh = lane >> 5;   // which half of each 8-wide contraction chunk this lane feeds

  // Workgroup -> (batch*head, Q block). Consecutive workgroup ids go round-robin over the 8 XCDs.
  int unit = blockIdx.x;
  int bh, t;
  if (causal == 2) {
    // Causal blocks differ up to Tq-fold in length. When (nearly) all of them are resident at
    // once, head after head would leave whole compute units with only long or only short
    // blocks: take them longest first over all heads, so that every round of the dispatcher
    // spreads one length class over the chip and the short blocks fill the slots that free up
    // last. With a head count that is a multiple of 8 a head still stays on one XCD.
    const int n_bh = total_units / Tq;
    t = Tq - 1 - unit / n_bh;
    bh = unit % n_bh;
  } else {
    // Each XCD walks a contiguous range of units, so the Q blocks of one head run together
    // and share that XCD's L2 for K and V; the causal blocks of a head longest first.
    if ((total_units & 7) == 0) unit = (blockIdx.x & 7) * (total_units >> 3) + (blockIdx.x >> 3);
    bh = unit / Tq;
    t = unit % Tq;
    if (causal) t = Tq - 1 - t;
  }
  const int b = bh / H, h = bh % H;
  const int hk = h / (H / Hkv);
  const int r0 = t * BR;

  const bf16* qh = q + (size_t)bh * N * D;
  const bf16* kh = k + (size_t)(b * Hkv + hk) * Nk * D;
  const bf16* vh = v + (size_t)(b * Hkv + hk) * Nk * D;
  // N queries against Nk keys; under the causal mask the last query is aligned with the last
  // key: key n is visible to query i iff n <= i + shift.
  const int shift = Nk - N;

  const int qw0 = r0 + wave * 32;              // first query row of this wave
  const int q_abs = qw0 + lq;                  // this lane's query row
  const int q_ld = min(q_abs, N - 1);          // ragged block: load a valid row, never store it

  // distr at d = 64: the Q block first lands in LDS by direct loads, all in flight at once
  // (16-byte chunks, rows past N zero-filled by the range check); the LSH stage and the sampling
  // then read its columns from there. Walking the columns in global memory instead costs the
  // workgroup one memory round trip per 16 rows and another for the sampled columns, which at
  // d = 64, where a block only has a few short tiles of work, is a large part of its lifetime.
  // (At d = 128 the stage is a percent of the block's time and the 32 KB are not spent.)
  constexpr bool QSTAGE = DISTR && D == 64;
  __shared__ __attribute__((aligned(1024))) char q_stage[QSTAGE ? BR * C::ROWB : 16];
  // The 16-byte chunks of a staged row are exchanged by the row index (chunk ^ ((row >> 1) & 7);
  // two rows of 128 bytes share a line of banks): the sampling reads one column of 32 different
  // rows at once and the LSH stage's transposing reads four rows per 16 lanes, which would
  // otherwise fall into one or two banks; reading along a row is conflict-free either way.
  auto q_swz = [](int row) { return (row >> 1) & 7; };
  auto q_staged = [&](int row, int ch) -> bf16 {
    return *(const bf16*)(q_stage + row * C::ROWB + (((ch >> 3) ^ q_swz(row)) << 4) + (ch & 7) * 2);
  };
  // (a generic lambda, like the other direct loads below: the builtins exist for the device only,
  // and a template is not checked against the host's builtin set)
  auto stage_q_block = [&](auto n_c, char* dst) {
    typedef __attribute__((address_space(3))) void lds_void_q;
    const __amdgpu_buffer_rsrc_t q_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)qh, 0, (unsigned)N * D * 2, 0x00020000);
#pragma unroll
    for (int j = 0; j < decltype(n_c)::value; ++j) {
      const int blk = j * C::NW + wave;
      const int slot = blk * 64 + lane;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(q_rsrc, (lds_void_q*)(dst + blk * 1024), 16,
                                               (slot / (D / 8)) * (D * 2) + ((slot % (D / 8)) ^ (((slot / (D / 8)) >> 1) & 7)) * 16,
                                               r0 * (D * 2), 0, 0);
    }
  };
  // The two pieces of the projection table (each a whole number of 1 KB blocks) from the table in
  // global memory into d1 and d2: block j of the 2 * PB blocks goes to wave j % NW.
  auto load_rtab = [&](auto n_c, char* d1, char* d2) {
    typedef __attribute__((address_space(3))) void lds_void_r;
    constexpr int PB = ((16 * (BR + 8) * 2 + 1023) / 1024);
    const __amdgpu_buffer_rsrc_t r_rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void*)(rtab + 1024), 0, 2 * PB * 1024, 0x00020000);
#pragma unroll
    for (int j = 0; j < decltype(n_c)::value; ++j) {
      const int blk = j * (BR / 32) + wave;
      if (blk < 2 * PB) {
        char* dst = blk < PB ? d1 + blk * 1024 : d2 + (blk - PB) * 1024;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(r_rsrc, (lds_void_r*)dst, 16, lane * 16, blk * 1024, 0, 0);
      }
    }
  };
  if constexpr (QSTAGE) {
    constexpr int QBLK = BR * C::ROWB / 1024;      // 1 KB blocks of the Q block
    static_assert(QBLK % C::NW == 0, "whole blocks per wave");
    stage_q_block(std::integral_constant<int, QBLK / C::NW>(), q_stage);
  }
  if constexpr (DISTR) {
    if (perm != nullptr) {
      const size_t pbase = ((size_t)bh * Tq + t) * D;
      // D is a power of two: an out-of-range entry of a caller's table cannot index past a row
      for (int i = tid; i < D; i += C::T) perm_lds[i] = perm[pbase + i] & (D - 1);
    } else {
      // ---- LSH hash-and-group of this Q block inside the workgroup (Sec. 3.2, 3.3) -------------
      // The table equals the stand-alone LSH kernel's bit for bit: a projection's sign is that of
      // the float sum with one fused multiply-add per row, rows ascending, from +0. At d = 128 the
      // sums are taken exactly that way; at d = 64 the matrix pipe takes them first and the defining
      // sum is only redone where the pipe's result is too close to zero to decide (below). Here the
      // stage costs no launch and no table in HBM, and runs while the CU's other workgroups keep
      // the matrix pipes busy. Up to 16 projections: R[row][16] (d = 128) or its two bf16 pieces
      // (d = 64) borrow the V buffers, the codes and hashes the first Kx buffer; all are filled
      // only after the barriers below.
      constexpr int NPG = C::T / D;             // threads per channel
      constexpr int PPT = 16 / NPG;             // projections per thread: pg*PPT .. pg*PPT+PPT-1
      static_assert(C::T % D == 0, "whole threads per channel");
      // (small tiles: the borrowed buffers are too short and the stage gets arrays of its own)
      constexpr bool R_BORROWS = BR * 16 * 4 <= C::TILEB, CODE_BORROWS = 2 * D * 4 <= C::KX_BYTES;
      __shared__ float R_own[(R_BORROWS || QSTAGE) ? 1 : BR * 16];
      __shared__ uint32_t code_own[CODE_BORROWS ? 1 : 2 * D];
      float* R_lds = R_BORROWS ? (float*)v_lds0 : R_own;
      uint32_t* code_lds = CODE_BORROWS ? (uint32_t*)kx_lds0 : code_own;
      uint32_t* hash_lds = code_lds + D;
      // Staged block: the projections are first taken on the matrix pipe, from R split into two
      // bf16 pieces (an entry is an integer of 17 bits times 2^-16: r1 = R rounded to bf16 and
      // r2 = R - r1 hold it exactly, and r1 + r2 gives it back exactly in float), next to
      // sum |q| |r1|, which bounds how far that sum can be from the float sum that defines the
      // sign. Only sums inside the bound are taken again the defining way (below). The pieces,
      // [projection][row] with rows padded by 16 bytes (16 lanes read 16 rows at once), borrow
      // the two V buffers where they fit.
      // The pieces come from the table the key pre-pass left behind the K^T copy when its header
      // names this call's seed, projection count and block rows (direct loads into LDS, no vector
      // work); otherwise the workgroup generates them.
      constexpr int RPAD = BR + 8;
      constexpr int RP_BYTES = rtab_piece_bytes(BR);
      constexpr bool RP_BORROWS = RP_BYTES <= C::TILEB;
      __shared__ __attribute__((aligned(1024))) char rp_own[(QSTAGE && !RP_BORROWS) ? 2 : 1][(QSTAGE && !RP_BORROWS) ? RP_BYTES : 16];
      bf16* rp1 = RP_BORROWS ? (bf16*)v_lds0 : (bf16*)rp_own[0];
      bf16* rp2 = RP_BORROWS ? (bf16*)v_lds1 : (bf16*)rp_own[(QSTAGE && !RP_BORROWS) ? 1 : 0];
      if constexpr (QSTAGE) {
        bool have_table = false;
        if (rtab != nullptr) {
          const RtabHeader hd = *(const RtabHeader*)rtab;
          have_table = hd.seed == lsh_seed && hd.n_planes == n_planes && hd.Br == BR;
        }
        if (have_table) {
          load_rtab(std::integral_constant<int, (2 * (RP_BYTES / 1024) + C::NW - 1) / C::NW>(), (char*)rp1, (char*)rp2);
        } else {
          for (int i = tid; i < BR * 16; i += C::T) {
            const int r = i % BR, pl = i / BR;
            const float rv = pl < n_planes ? hyperplane_entry(lsh_seed, (uint32_t)pl, (uint32_t)r) : 0.0f;
            const bf16 r1 = (bf16)rv;
            rp1[pl * RPAD + r] = r1;
            rp2[pl * RPAD + r] = (bf16)(rv - (float)r1);
          }
        }
      } else {
        for (int i = tid; i < BR * 16; i += C::T)
          R_lds[i] = (i & 15) < n_planes ? hyperplane_entry(lsh_seed, (uint32_t)(i & 15), (uint32_t)(i >> 4)) : 0.0f;
      }
      if (tid < D) code_lds[tid] = 0;
      if constexpr (QSTAGE) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wave's part of the Q block has landed
      __syncthreads();
      const int c = tid % D, pg = tid / D;
      const int rows = min(BR, N - r0);
      const bf16* qcol = qh + (size_t)r0 * D + c;
      if constexpr (QSTAGE) {
        // v_mfma_f32_16x16x32_bf16: 16 channels x 16 projections per product, 32 rows of the block
        // per step; lane = (projection pl16 = lane % 16, row group kg = lane / 16) on the R side
        // and (channel, row group) on the Q side, whose operand comes out of the staged block by
        // transposing reads (rows past N are zeros there). Register i of the result belongs to
        // channel 16*ct + 4*kg + i and projection pl16.
        const int pl16 = lane & 15, kg = lane >> 4;
        // The sign of a sum is taken from the matrix pipe only if the sum is further from zero
        // than both roundings can reach, each relative to sum |q| |R| <= (1 + 2^-8) sum |q| |r1|:
        // the pipe's, at most 2*BR products and BR/16 chained accumulators added in any order with
        // any rounding direction (2 * (2*BR + BR/16) * 2^-24), and the defining float chain's,
        // BR fused multiply-adds (BR * 2^-24). The absolute term covers products flushed to zero.
        constexpr float kDoubt = 3.1e-7f * BR, kTiny = 1e-30f;
        for (int ct = wave; ct < D / 16; ct += C::NW) {
          f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f}, bnd = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
          for (int ks = 0; ks < BR / 32; ++ks) {
            const int row0 = 32 * ks + 8 * kg + (pl16 >> 2), row1 = row0 + 4;
            const int chunk = 2 * ct + ((pl16 & 3) >> 1), inch = 8 * (pl16 & 1);
            const s16x8 a = lds_read_tr_pair<s16x8>(q_stage + row0 * C::ROWB + ((chunk ^ q_swz(row0)) << 4) + inch,
                                                    q_stage + row1 * C::ROWB + ((chunk ^ q_swz(row1)) << 4) + inch);
            const int roff = 32 * ks + 8 * kg;
            const s16x8 b1 = *(const s16x8*)&rp1[pl16 * RPAD + roff];
            const s16x8 b2 = *(const s16x8*)&rp2[pl16 * RPAD + roff];
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b1), acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b2), acc, 0, 0, 0);
            bnd = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a & (short)0x7fff),
                                                          __builtin_bit_cast(bf16x8, b1 & (short)0x7fff), bnd, 0, 0, 0);
          }
          bool positive[4], doubt[4], any_doubt = false;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            positive[i] = acc[i] > 0.0f;
            doubt[i] = pl16 < n_planes && !(__builtin_fabsf(acc[i]) > kDoubt * bnd[i] + kTiny);
            any_doubt |= doubt[i];
          }
          if (__builtin_amdgcn_ballot_w64(any_doubt) != 0) {
            // The defining sums of this lane's four channels (float, one fused multiply-add per
            // row, rows ascending): the channels 16*ct + 4*kg + 0..3 sit in one 8-byte piece of
            // every staged row.
            float sum[4] = {0.0f, 0.0f, 0.0f, 0.0f};
            const int ch0 = 16 * ct + 4 * kg;
            const char* col = q_stage + (ch0 & 7) * 2;
            for (int r8 = 0; r8 < BR; r8 += 8) {
#pragma unroll
              for (int j8 = 0; j8 < 8; ++j8) {
                const s16x4 x4 = *(const s16x4*)(col + (r8 + j8) * C::ROWB + (((ch0 >> 3) ^ q_swz(r8 + j8)) << 4));
                const float rv = (float)rp1[pl16 * RPAD + r8 + j8] + (float)rp2[pl16 * RPAD + r8 + j8];   // exact
#pragma unroll
                for (int i = 0; i < 4; ++i)
                  sum[i] = __builtin_fmaf(__builtin_bit_cast(float, (uint32_t)(uint16_t)x4[i] << 16), rv, sum[i]);
              }
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
              if (doubt[i]) positive[i] = sum[i] > 0.0f;
          }
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            // lanes 16*kg .. 16*kg + 15 of the ballot are projections 0..15 of channel 16*ct + 4*kg + i;
            // projection 0 is the top bit of the n_planes-bit code
            const uint64_t signs = __builtin_amdgcn_ballot_w64(positive[i]);
            if (pl16 == 0)
              code_lds[16 * ct + 4 * kg + i] = __builtin_bitreverse32((uint32_t)(signs >> (16 * kg)) & 0xffffu) >> (32 - n_planes);
          }
        }
      } else {
        // (not staged: 16 column loads in flight per thread, because with two workgroups per CU
        // nothing else hides their latency here)
        float acc[PPT];
#pragma unroll
        for (int j = 0; j < PPT; ++j) acc[j] = 0.0f;
#pragma unroll 16
        for (int r = 0; r < rows; ++r) {
          const float x = (float)qcol[(size_t)r * D];
#pragma unroll
          for (int j = 0; j < PPT; ++j) acc[j] = __builtin_fmaf(x, R_lds[r * 16 + pg * PPT + j], acc[j]);
        }
        uint32_t bits = 0;
#pragma unroll
        for (int j = 0; j < PPT; ++j) {
          const int pl = pg * PPT + j;
          if (pl < n_planes && acc[j] > 0.0f) bits |= 1u << (n_planes - 1 - pl);   // projection 0 = top bit
        }
        if (NPG == 1) code_lds[c] = bits;
        else if (bits) atomicOr(&code_lds[c], bits);
      }
      __syncthreads();
      if (tid < D) {
        hash_lds[tid] = lsh_hash_of_code(code_lds[tid], gray_mode);
        code_lds[tid] = 0;   // from here on the channel's rank is counted in this word
      }
      __syncthreads();
      {
        // Rank by counting = stable ascending sort; perm = inverse of the rank. Every thread
        // counts a slice of the other channels for its own (NPG threads per channel, the hashes
        // read four at a time), the slices meet in an integer LDS add.
        constexpr int SL = D / NPG;
        static_assert(SL % 4 == 0, "whole 16-byte reads per slice");
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
        if (NPG == 1) rank_lds[c] = cnt;
        else if (cnt) atomicAdd(&rank_lds[c], cnt);
        __syncthreads();
        if (tid < D) perm_lds[rank_lds[tid]] = (uint8_t)tid;
      }
    }
    if constexpr (QSTAGE) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    // the table of the workgroup's own LSH stage, for a caller that wants it (e.g. to hand it to
    // the backward pass)
    if (perm == nullptr && perm_w != nullptr)
      for (int i = tid; i < D; i += C::T) perm_w[((size_t)bh * Tq + t) * D + i] = perm_lds[i];
    if constexpr (NG < KRED) {
      // Rows NG..KRED-1 of K_f^T pad the contraction: zeroed once (after the LSH stage, which may
      // have borrowed them), the fusion never writes them; visible to every wave after the
      // barrier that ends the prologue.
      const f16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
      for (int i = NG * C::KTROWB / 16 + tid; i < C::KX_BYTES / 16; i += C::T) {
        ((f16x8*)kx_lds0)[i] = zero;
        ((f16x8*)kx_lds1)[i] = zero;
      }
    }
  }

  // ---- Q operands, held for the whole inner loop ------------------------------------------
  // distr: the reduced product runs on the f16 matrix path. A bf16 value converts to half
  // exactly (8 vs 11 significand bits) inside half's exponent range, and the fused keys, rounded
  // to half from the sum of such values, keep 3 more bits than bf16 would: with bf16 K_f the logit error
  // on inputs with heavy-tailed channel scales exceeds what the output tolerance allows.
  // distr: Q_r carries the factor softmax_scale * log2(e), rounded once more to half (11 bits:
  // the rounding is 8 times finer than the bf16 grid the inputs come from). The score
  // accumulators then hold the exponent of 2 directly. The exact path keeps Q as it is: scaling
  // and re-rounding to bf16 would cost accuracy on rows with close top scores, so there the
  // factor is applied to the float scores, one fused multiply-add per score.
  kx8 qop[C::KSTEPS];
  if constexpr (DISTR) {
    // (staged block: a row past N reads as zeros and is never stored)
    const bf16* qrow = qh + (size_t)q_ld * D;
#pragma unroll
    for (int s = 0; s < C::KSTEPS; ++s) {
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if (NG == KRED || 16 * s + 8 * hh + j < NG)
          qop[s][j] = to_half_sat((QSTAGE ? (float)q_staged(wave * 32 + lq, perm_lds[(16 * s + 8 * hh + j) * C::G])
                                          : (float)qrow[perm_lds[(16 * s + 8 * hh + j) * C::G]]) * scale_log2e);
        else
          qop[s][j] = (f16)0.0f;   // padding of the contraction: no group there
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

  // ---- fusion bookkeeping, fixed for the Q block ------------------------------------------------
  // Fused output u of this thread is the 16-byte piece (8 keys) number idx % 8 of group
  // idx / PPR, idx = tid + u*T: it sums the same piece of the group's G channel rows of K^T
  // (f_src: byte offset of the piece inside the head's K^T, tile 0) and lands in row idx / 8 of
  // K_f^T at the swizzled position (f_dst).
  int f_src[DISTR ? C::FUSE_OUT : 1][DISTR ? C::G : 1];
  int f_dst[DISTR ? C::FUSE_OUT : 1];
  if constexpr (DISTR) {
#pragma unroll
    for (int u = 0; u < C::FUSE_OUT; ++u) {
      const int idx = min(tid + u * C::T, NG * C::PPR - 1);
      const int j = idx / C::PPR, c8 = idx % C::PPR;
#pragma unroll
      for (int g = 0; g < C::G; ++g)
        f_src[u][g] = perm_lds[j * C::G + g] * Npad * 2 + c8 * 16;
      f_dst[u] = j * C::KTROWB + ((((c8 >> 1) ^ kf_swizzle<BC>(j)) << 1) | (c8 & 1)) * 16;
    }
  }

  const int n_end = causal ? min(Nk, r0 + BR + shift) : Nk;
  const int n_tiles = (n_end + BC - 1) / BC;
  // tiles [0, n_full) need no masking for any row of the block
  const int n_full = causal ? min(r0 + shift, Nk) / BC : Nk / BC;

  // ---- tile loads: global -> LDS ---------------------------------------------------------------
  // K and V rows are fetched through buffer descriptors: the per-lane byte offset inside a
  // tile is fixed, the tile advances through the scalar offset, and rows past the end of the
  // head read as zero (hardware range check), so a tile costs no address arithmetic.
  const unsigned head_bytes = (unsigned)Nk * D * 2;
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
    const int lseg = (pc >> 1) ^ v_swizzle<C::ROWB>(row);
    dma_v[j] = row * C::ROWB + (lseg * 2 + (pc & 1)) * 16;
  }
  typedef __attribute__((address_space(3))) void lds_void;
  auto dma_blocks = [&](auto n_c, __amdgpu_buffer_rsrc_t rsrc, int soff, const int* voff, char* dst) {
#pragma unroll
    for (int j = 0; j < decltype(n_c)::value; ++j)
      if (C::NBLK % C::NW == 0 || j * C::NW + wave < C::NBLK)   // (more waves than 1 KB blocks: the rest sit out)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void*)(dst + (j * C::NW + wave) * 1024), 16,
                                                 voff[j], soff, 0, 0);
  };
  auto dma_tile = [&](__amdgpu_buffer_rsrc_t rsrc, int tile, const int* voff, char* dst) {
    dma_blocks(std::integral_constant<int, C::CPT>(), rsrc, tile * C::TILEB, voff, dst);
  };
  auto dma_wait = [&]() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); };

  // distr: K^T of this kv head, [D channel rows][Npad keys] half.
  const __amdgpu_buffer_rsrc_t kt_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      (void*)(DISTR ? kt + (size_t)(b * Hkv + hk) * D * Npad : nullptr), 0, (unsigned)D * Npad * 2, 0x00020000);
  // ---- fusion (Sec. 3.2): K_f^T[j][n] = sum over the group's channels c of K^T[c][n], eight keys
  // at a time with packed half adds (for G* = 2 the sum of two bf16-valued halves is rounded to
  // half once; larger groups add one channel after the other). Every thread loads the 16-byte
  // pieces it sums straight from K^T in global memory (8 lanes cover one 128-byte channel row)
  // one tile iteration before it adds them, so the LDS only sees K_f^T (8-16 KB per tile): with
  // the raw tile staged in LDS and summed from there (direct load, 16 KB read, K_f^T written)
  // the kernel was bound by LDS traffic and 2-12 % slower.
    typedef f16x8 Pieces[DISTR ? C::FUSE_OUT : 1][DISTR ? C::G : 1];
  Pieces piece;   // the set the main loop carries from one iteration to the next
  auto load_pieces = [&](int tile, Pieces& pc) {
    if constexpr (DISTR) {
#pragma unroll
      for (int u = 0; u < C::FUSE_OUT; ++u)
#pragma unroll
        for (int g = 0; g < C::G; ++g)
          pc[u][g] = __builtin_bit_cast(f16x8, __builtin_amdgcn_raw_buffer_load_b128(kt_rsrc, f_src[u][g], tile * C::KTROWB, 0));
    }
  };
  auto fuse_pieces = [&](int buf, const Pieces& pc) {   // loaded pieces -> K_f^T in kx_buf(buf)
    if constexpr (DISTR) {
      char* dst = kx_buf(buf);
#pragma unroll
      for (int u = 0; u < C::FUSE_OUT; ++u) {
        f16x8 acc = pc[u][0];
#pragma unroll
        for (int g = 1; g < C::G; ++g) acc += pc[u][g];
        if (NG * C::PPR % C::T == 0 || tid + u * C::T < NG * C::PPR) *(f16x8*)(dst + f_dst[u]) = acc;
      }
    }
  };

  // ---- accumulators and softmax state ---------------------------------------------------------
  f32x16 oacc[D / 32];
#pragma unroll
  for (int mb = 0; mb < D / 32; ++mb)
#pragma unroll
    for (int i = 0; i < 16; ++i) oacc[mb][i] = 0.0f;
  // Softmax state of this lane's query row, in the exp2 domain: the negated reference maximum
  // and the row sum relative to it. distr: the negated reference also sits in all 16 registers
  // of neg_ref, which the first MFMA of every score chain takes as its addend, so the
  // accumulators come out as (scaled score - m_ref) and go straight into exp2.
  constexpr bool PRESCALED = DISTR;
  float nref = 0.0f;
  f32x16 neg_ref;
#pragma unroll
  for (int i = 0; i < 16; ++i) neg_ref[i] = 0.0f;
  float l_run = 0.0f;        // over this lane's half of the keys

  // LDS byte offsets of this lane's operands inside a buffer.
  // Score product, A operand (exact): row lq (+32 per key block), logical chunk 2*s + hh.
  int ka_off[DISTR ? 2 * C::MB : C::KSTEPS];
  if constexpr (DISTR) {
    // K_f^T is read like V: lane addresses group row 8*hh + 4*half + (lane%16)/4 (+16*s), 32-byte
    // segment 2*mb + (lane/16)%2 (keys 32*mb + 16*((lane/16)%2) ..), 8-byte piece lane%4.
    const int r4 = (lane & 15) >> 2;
#pragma unroll
    for (int mb = 0; mb < C::MB; ++mb)
#pragma unroll
      for (int hf = 0; hf < 2; ++hf)
        ka_off[mb * 2 + hf] = (8 * hh + 4 * hf + r4) * C::KTROWB +
                              ((2 * mb + ((lane >> 4) & 1)) ^ kf_swizzle<BC>(4 * hf + r4)) * 32 + 8 * (lane & 3);
  } else {
#pragma unroll
    for (int s = 0; s < C::KSTEPS; ++s)
      ka_off[s] = lq * C::ROWB + ((2 * s + hh) ^ (D == 128 ? (lq & 15) : ((lq >> 1) & 7))) * 16;
  }
  // P.V, A operand via transposing reads: lane addresses row 4*hh + (lane%16)/4 (+8, +16*tt),
  // logical 32-byte segment 2*mb + (lane/16)%2, 8-byte piece lane%4 of it.
  int va_off[D / 32];
  {
    const int row_l = 4 * hh + ((lane & 15) >> 2);
    const int swz = v_swizzle<C::ROWB>(row_l);
#pragma unroll
    for (int mb = 0; mb < D / 32; ++mb)
      va_off[mb] = row_l * C::ROWB + ((2 * mb + ((lane >> 4) & 1)) ^ swz) * 32 + 8 * (lane & 3);
  }

  // S^T = Kx . Qx^T for the Kx tile in buffer `buf`: register i of block mb holds key
  // 32*mb + 8*(i/4) + 4*hh + i%4 of the tile.
  auto qk = [&](int buf, f32x16 (&sacc)[C::MB]) {
    const char* base = kx_buf(buf);
#pragma unroll
    for (int mb = 0; mb < C::MB; ++mb) {
#pragma unroll
      for (int s = 0; s < C::KSTEPS; ++s) {
        kx8 a;
        if constexpr (DISTR)
          a = lds_read_tr_pair<kx8>(base + ka_off[mb * 2] + s * 16 * C::KTROWB,
                                    base + ka_off[mb * 2 + 1] + s * 16 * C::KTROWB);
        else
          a = *(const kx8*)(base + ka_off[s] + mb * 32 * C::ROWB);
        if (s == 0) {
          if constexpr (PRESCALED) sacc[mb] = neg_ref;
          else
#pragma unroll
            for (int i = 0; i < 16; ++i) sacc[mb][i] = 0.0f;
        }
        sacc[mb] = mfma_32x32x16(a, qop[s], sacc[mb]);
      }
    }
  };

  // Causal / ragged-tail mask of the scores of tile `tile`.
  auto apply_mask = [&](int tile, f32x16 (&sc)[C::MB]) {
    const int lim = causal ? min(q_abs + shift, Nk - 1) : Nk - 1;  // last visible key of this row
#pragma unroll
    for (int mb = 0; mb < C::MB; ++mb)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        int kv = tile * BC + 32 * mb + 8 * (i >> 2) + 4 * hh + (i & 3);
        if (kv > lim) sc[mb][i] = -INFINITY;
      }
  };
  // Row maximum of a tile's scores (relative to the current reference), the same in both lanes
  // of a row.
  auto tile_max = [&](const f32x16 (&sc)[C::MB]) -> float {
    float mt = sc[0][0];
#pragma unroll
    for (int mb = 0; mb < C::MB; ++mb)
#pragma unroll
      for (int i = 0; i < 16; ++i) mt = fmaxf(mt, sc[mb][i]);
    mt = half_swap_max(mt);
    return PRESCALED ? mt : __builtin_fmaf(mt, scale_log2e, nref);
  };
  // P = exp2(scores) rounded to bf16, as the B operands of P.V; returns this lane's row sum. The
  // sum is taken over the rounded P, the values P.V really uses (one bf16 dot product with (1, 1)
  // per register pair): numerator and denominator then carry the same rounding, which cancels
  // for rows dominated by few keys.
  auto exp_tile = [&](const f32x16 (&sc)[C::MB], bf16x8 (&pop)[C::TT]) -> float {
    const bf16x2 ones = {(bf16)1.0f, (bf16)1.0f};
    float rs0 = 0.0f, rs1 = 0.0f;
#pragma unroll
    for (int mb = 0; mb < C::MB; ++mb)
#pragma unroll
      for (int i = 0; i < 16; i += 2) {
        float x0 = sc[mb][i], x1 = sc[mb][i + 1];
        if constexpr (!PRESCALED) {
          x0 = __builtin_fmaf(x0, scale_log2e, nref);
          x1 = __builtin_fmaf(x1, scale_log2e, nref);
        }
        bf16x2 pr = {(bf16)__builtin_amdgcn_exp2f(x0), (bf16)__builtin_amdgcn_exp2f(x1)};
        pop[mb * 2 + (i >> 3)][i & 7] = pr[0];
        pop[mb * 2 + (i >> 3)][(i & 7) + 1] = pr[1];
        if (i & 2) rs1 = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, rs1, false);
        else rs0 = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, rs0, false);
      }
    return rs0 + rs1;
  };
  // The reference of this lane's row moves up by `delta`: everything that is relative to it
  // follows (row sum, output accumulator, the scores already computed against the old one).
  auto shift_reference = [&](float delta, auto rescale_c, f32x16 (&sc)[C::MB], auto next_c, f32x16 (&sn)[C::MB]) {
    nref -= delta;
    if constexpr (PRESCALED) {
#pragma unroll
      for (int i = 0; i < 16; ++i) neg_ref[i] -= delta;
#pragma unroll
      for (int mb = 0; mb < C::MB; ++mb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          sc[mb][i] -= delta;
          if constexpr (decltype(next_c)::value) sn[mb][i] -= delta;
        }
    }
    if constexpr (decltype(rescale_c)::value) {
      const float alpha = __builtin_amdgcn_exp2f(-delta);
      l_run *= alpha;
#pragma unroll
      for (int mb = 0; mb < D / 32; ++mb)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[mb][i] *= alpha;
    }
  };

  // One tile `it`, whose scores `sc` are masked and relative to the row's reference:
  //   scores of tile it+1 into `sn` (matrix pipe)  ||  exp2, bf16 P, row sum of `sc` (vector ALUs)
  //   the rare reference move, then O^T += V^T . P^T for tile it (matrix pipe), the mask of
  //   tile it+1 where it needs one, one barrier.
  auto body = [&](auto mask_next_c, auto next_c, int it, int par, f32x16 (&sc)[C::MB], f32x16 (&sn)[C::MB]) {
    constexpr bool HAS_NEXT = decltype(next_c)::value;
    // The buffers these loads fill were last read in the previous iteration, which every wave
    // has left (barrier): K(it+2) replaces K(it), V(it+1) replaces V(it-1).
    if constexpr (HAS_NEXT) {
      // distr: the pieces of K^T(it+2), loaded during the previous iteration, are summed now
      // into the buffer K_f^T(it) has left, and the loads of K^T(it+3) take their registers.
      // Nothing in this iteration depends on the fusion: it runs beside the MFMAs.
      if constexpr (DISTR) {
        fuse_pieces(par, piece);       // K^T(it+2), loaded during the previous iteration
        load_pieces(it + 3, piece);
      }
      if constexpr (!DISTR) dma_tile(k_rsrc, it + 2, dma_k, kx_buf(par));
      dma_tile(v_rsrc, it + 1, dma_v, v_buf(par ^ 1));
    }
    if constexpr (HAS_NEXT) qk(par ^ 1, sn);
    bf16x8 pop[C::TT];
    float rs = exp_tile(sc, pop);
    if (__builtin_amdgcn_ballot_w64(!(rs <= kSumTrigger)) != 0) {
      // Some row of this wave met a score more than kTau above its reference: such rows take the
      // tile's maximum as their new reference and the tile's P is computed again.
      const float mt = tile_max(sc);
      shift_reference(mt > kTau ? mt : 0.0f, std::true_type(), sc, next_c, sn);
      rs = exp_tile(sc, pop);
    }
    l_run += rs;
    // ---- O^T += V^T . P^T: step tt covers keys 16*tt + {8*(j/4) + 4*hh + j%4} of the tile,
    // i.e. V rows 16*tt + 4*hh + 0..3 and 16*tt + 8 + 4*hh + 0..3.
    const char* vb = v_buf(par);
    // The V operands are read PF steps (four operands) ahead of the MFMA that takes them, and the
    // scheduler is told to keep that order: left alone it issues an operand's reads right in
    // front of its MFMA, which then waits out the LDS latency 4 * TT times per tile.
    constexpr int NMB = D / 32;
    constexpr int PF = (4 / NMB < C::TT) ? 4 / NMB : C::TT - 1;
    auto v_operand = [&](int tt, int mb) {
      const char* p0 = vb + va_off[mb] + 16 * tt * C::ROWB;
      return lds_read_tr_pair<bf16x8>(p0, p0 + 8 * C::ROWB);
    };
    bf16x8 va[PF + 1][NMB];
#pragma unroll
    for (int t0 = 0; t0 < PF; ++t0)
#pragma unroll
      for (int mb = 0; mb < NMB; ++mb) va[t0][mb] = v_operand(t0, mb);
#pragma unroll
    for (int tt = 0; tt < C::TT; ++tt) {
      if (tt + PF < C::TT) {
#pragma unroll
        for (int mb = 0; mb < NMB; ++mb) va[(tt + PF) % (PF + 1)][mb] = v_operand(tt + PF, mb);
      }
#pragma unroll
      for (int mb = 0; mb < NMB; ++mb)
        oacc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[tt % (PF + 1)][mb], pop[tt], oacc[mb], 0, 0, 0);
    }
    // instruction order: the reads of the first PF steps, then every MFMA followed by the two
    // reads of one operand PF steps ahead (0x100 = LDS reads, 0x008 = MFMA)
    __builtin_amdgcn_sched_group_barrier(0x100, 2 * NMB * PF, 0);
#pragma unroll
    for (int i = 0; i < (C::TT - PF) * NMB; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, PF * NMB, 0);
    if constexpr (HAS_NEXT) {
      if constexpr (decltype(mask_next_c)::value) apply_mask(it + 1, sn);
      dma_wait();              // this wave's direct loads have landed
    }
    __syncthreads();
  };

  // ---- prologue: tiles 0 (K, V) and 1 (K) into LDS, scores of tile 0 ---------------------------
  dma_tile(v_rsrc, 0, dma_v, v_lds0);
  if constexpr (DISTR) {
    Pieces first;        // tiles 0 and 1 travel together (registers are plentiful before the loop)
    load_pieces(0, first);
    load_pieces(1, piece);
    fuse_pieces(0, first);
    fuse_pieces(1, piece);
    load_pieces(2, piece);
    dma_wait();          // V(0) has landed (and, with it, the pieces of tile 2)
    __syncthreads();     // K_f^T(0), K_f^T(1) and V(0) are visible
  } else {
    dma_tile(k_rsrc, 0, dma_k, kx_lds0);
    if (n_tiles > 1) dma_tile(k_rsrc, 1, dma_k, kx_lds1);
    dma_wait();
    __syncthreads();
  }

  const std::true_type yes;
  const std::false_type no;
  f32x16 s0[C::MB], s1[C::MB];
  qk(0, s0);             // against the initial reference 0
  apply_mask(0, s0);
  // The first tile sets the reference to its row maximum (key 0 is visible to every row, so the
  // maximum is finite); nothing has been accumulated yet, so nothing is rescaled.
  shift_reference(tile_max(s0), no, s0, no, s1);
  // The first iteration refills the buffer of tile 0 (direct load of K(2), or the fusion of
  // K_f^T(2)): every wave must have read its scores of tile 0 out of it first.
  __syncthreads();

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
    for (int mb = 0; mb < C::MB; ++mb) s0[mb] = s1[mb];
  }
  body(no, no, it, it & 1, s0, s1);

  // ---- epilogue: O = O_acc / l, bf16, 8-byte stores ---------------------------------------------
  const float l_tot = half_swap_sum(l_run);
  const float inv = 1.0f / l_tot;
  // row statistics for a backward pass: ln(sum of exp(score)) = ln 2 * (reference + log2(l))
  if (lse && q_abs < N && hh == 0) lse[(size_t)bh * N + q_abs] = 0.6931471805599453f * (__builtin_log2f(l_tot) - nref);
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

template <int D, int BR, int BC, int KRED, bool DISTR, int NG = KRED>
hipError_t launch_one(const void* q, const void* k, const void* v, void* o, const uint8_t* perm,
                      const void* kt, const Problem& pb, hipStream_t stream) {
  const int Tq = (pb.N + BR - 1) / BR;
  const long long units = (long long)pb.B * pb.H * Tq;
  const float scale_log2e = pb.scale * 1.4426950408889634f;
  // causal_mode 2 = blocks issued longest first over all heads (see the kernel): for problems
  // of up to 8 workgroups per compute unit, where load balance matters more than L2 locality
  // (with more blocks the dispatcher balances by itself and the head-major order fetches half
  // as many bytes from HBM).
  const int causal_mode = pb.causal ? (units <= 8 * 256 ? 2 : 1) : 0;
  hipLaunchKernelGGL((attn_bf16_kernel<D, BR, BC, KRED, DISTR, NG>), dim3((unsigned)units), dim3(BR * 2), 0,
                     stream, (const bf16*)q, (const bf16*)k, (const bf16*)v, (bf16*)o, perm, (const f16*)kt,
                     (pb.Nk + kKtPad - 1) / kKtPad * kKtPad, pb.H, pb.Hkv, pb.N, pb.Nk, Tq, causal_mode,
                     scale_log2e, (int)units, pb.n_planes, pb.gray_mode, pb.seed, pb.lse,
                     (DISTR && kt) ? (const char*)kt + kt_copy_bytes(pb.B, pb.Hkv, pb.d, pb.Nk) : nullptr,
                     DISTR ? pb.perm_w : nullptr);
  return hipGetLastError();
}

// Group counts built for a K/V tile of BC rows: every supported one for the default tile of
// 64 rows, the common ones (16, 32, 64 groups) for the tiles of the block-size study.
constexpr bool attn_bf16_groups_built(int BC, int d, int n_groups) {
  if (n_groups > d || d % n_groups != 0 || d / n_groups > 16) return false;
  if (n_groups == d) return true;   // exact product
  if (BC == 64) return n_groups == 4 || n_groups == 8 || n_groups == 16 || n_groups == 32 || n_groups == 64;
  return n_groups == 16 || n_groups == 32 || n_groups == 64;
}

template <int D, int BR, int BC>
hipError_t dispatch_kred(const void* q, const void* k, const void* v, void* o, const uint8_t* perm,
                         const void* kt, const Problem& pb, int distr, hipStream_t stream) {
  if (!distr) return launch_one<D, BR, BC, D, false>(q, k, v, o, perm, kt, pb, stream);
  switch (pb.n_groups) {   // n_groups = d (groups of one channel) is the exact product: dispatched by the caller
    case 4:                // fewer groups than one MFMA step: contraction zero-padded to 16
      if constexpr (D == 64 && BC == 64) return launch_one<D, BR, BC, 16, true, 4>(q, k, v, o, perm, kt, pb, stream);
      return hipErrorInvalidValue;
    case 8:
      if constexpr (BC == 64) return launch_one<D, BR, BC, 16, true, 8>(q, k, v, o, perm, kt, pb, stream);
      return hipErrorInvalidValue;
    case 16: return launch_one<D, BR, BC, 16, true>(q, k, v, o, perm, kt, pb, stream);
    case 32: return launch_one<D, BR, BC, 32, true>(q, k, v, o, perm, kt, pb, stream);
    case 64:
      if constexpr (D == 128) return launch_one<D, BR, BC, 64, true>(q, k, v, o, perm, kt, pb, stream);
      [[fallthrough]];
    default: return hipErrorInvalidValue;
  }
}

// Every (head dim, Q block rows) pair for one K/V tile size; one translation unit per tile size.
template <int BC>
hipError_t dispatch_shape(const void* q, const void* k, const void* v, void* o, const uint8_t* perm,
                          const void* kt, const Problem& pb, int distr, hipStream_t stream) {
  if (pb.d == 64 && pb.Br == 64) return dispatch_kred<64, 64, BC>(q, k, v, o, perm, kt, pb, distr, stream);
  if (pb.d == 64 && pb.Br == 128) return dispatch_kred<64, 128, BC>(q, k, v, o, perm, kt, pb, distr, stream);
  if (pb.d == 64 && pb.Br == 256) return dispatch_kred<64, 256, BC>(q, k, v, o, perm, kt, pb, distr, stream);
  if (pb.d == 128 && pb.Br == 64) return dispatch_kred<128, 64, BC>(q, k, v, o, perm, kt, pb, distr, stream);
  if (pb.d == 128 && pb.Br == 128) return dispatch_kred<128, 128, BC>(q, k, v, o, perm, kt, pb, distr, stream);
  if (pb.d == 128 && pb.Br == 256) return dispatch_kred<128, 256, BC>(q, k, v, o, perm, kt, pb, distr, stream);
  return hipErrorInvalidValue;
}

}  // namespace

}  // namespace da
