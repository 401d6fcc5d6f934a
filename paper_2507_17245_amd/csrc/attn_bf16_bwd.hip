// Backward of the attention forward (exact and DistrAttention) for bf16 tensors on the gfx950
// matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulate). Three kernels (and a reduction when the
// dK/dV launch is split over query heads), no atomics (results do not depend on the run).
//
// The paper trains through the approximation (Sec. 4.3, 4.4) and gives no gradient; computed here
// is the derivative of the forward with every Q block's grouping held fixed. With Q_r the sampled
// and K_f the fused columns of Sec. 3.2 (Eq. 2: S^ = Q_r K_f^T, one grouping per Q block,
// Sec. 3.3), write Q~ for Q with every channel replaced by its group's sampled channel:
//   S^ = Q_r K_f^T = Q~ K^T                       (a sum over groups of sums over members)
//   dK = scale * dS^T Q~                          (every member of a group receives dK_f's column)
//   dQ[:, sampled channel of group j] = scale * sum over the group's members c of (dS K)[:, c]
// so the backward of DistrAttention is the backward of exact attention taken on Q~, followed by a
// sum over each group's members for dQ. P = exp(S^ - lse) is rebuilt from the forward's row
// statistics, dP = dO V^T, D_i = sum_c dO_ic O_ic, dS = P o (dP - D), dV = P^T dO.
//
//   bwd_prepare_kernel  D_i and lse * log2(e) for every row; Q~ (DistrAttention only) into scratch
//   bwd_dq_kernel       one workgroup per 128 query rows, lane = query row; K and V tiles of 64
//                       rows stream through LDS:  S^T = K Q~^T, dP^T = V dO^T, dQ~^T += K^T dS^T
//   bwd_dkv_kernel      one workgroup per 128 keys of a kv head, lane = key; Q~ and dO tiles of 64
//                       rows of every query head of the group stream through LDS:
//                       S = Q~ K^T, dP = dO V^T, dV^T += dO^T P, dK^T += Q~^T dS
//   bwd_reduce_kernel   sums the float partial dK, dV of a head-split dK/dV launch
// In both, the accumulator layout of the first products (registers = streamed rows, lanes =
// resident rows) is the B-operand layout of the last ones, so P and dS never leave registers; the
// streamed tiles are read once row-wise (16-byte reads) and once with transposing reads. Tiles are
// double-buffered in LDS and loaded one iteration ahead (one barrier per tile).
#include <type_traits>

#include "da_common.h"

namespace da {

namespace {

typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

constexpr int kBwdRows = 128;      // resident rows per workgroup (4 waves x 32)
constexpr int kBwdStream = 64;     // streamed rows per LDS tile
constexpr int kBwdThreads = 256;
constexpr float kLog2e = 1.4426950408889634f;

__device__ inline f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Position of a 16-byte chunk inside its row of a streamed tile (rows of D bf16, unpadded). A
// tile is read two ways: 16 lanes take the same chunk of 16 consecutive rows (16-byte reads), and
// the transposing reads take, per 32 lanes, 64 consecutive bytes of 4 consecutive rows. Both are
// free of bank conflicts when the chunk index is XORed with these bits of the row.
template <int D>
__device__ inline int chunk_swz(int row) {
  if constexpr (D == 128) return ((row & 3) << 2) | ((row >> 2) & 3);
  else return (((row >> 1) & 1) << 2) | ((row >> 2) & 3);
}

template <int D>
__device__ inline char* chunk_addr(char* tile, int row, int chunk) {
  return tile + row * (D * 2) + ((chunk ^ chunk_swz<D>(row)) << 4);
}

// Streamed tiles reach LDS by direct global->LDS loads (buffer_load ... lds: each wave-level load
// drops 64 x 16 bytes contiguously): wave-level load j of wave w fills the 1 KB block 4*j + w of
// the tile; the lane that owns a 16-byte position fetches the global chunk the swizzle assigns to
// it. The source is a buffer descriptor over one head, whose range check makes rows past the end
// read as zeros.
typedef __attribute__((address_space(3))) void lds_void;
template <int D>
struct TileLoader {
  static constexpr int CH = D / 8, ROWB = D * 2, TILE = kBwdStream * ROWB;
  static constexpr int CPT = TILE / 1024 / (kBwdThreads / 64);
  int voff[CPT];
  int wave;
  __device__ TileLoader(int wave_, int lane) : wave(wave_) {
#pragma unroll
    for (int j = 0; j < CPT; ++j) {
      const int slot = (j * (kBwdThreads / 64) + wave) * 64 + lane;
      const int row = slot / CH, pc = slot % CH;
      voff[j] = row * ROWB + ((pc ^ chunk_swz<D>(row)) << 4);
    }
  }
  __device__ void load(__amdgpu_buffer_rsrc_t rsrc, int row0, char* dst) const {
#pragma unroll
    for (int j = 0; j < CPT; ++j)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void*)(dst + (j * (kBwdThreads / 64) + wave) * 1024), 16,
                                               voff[j], row0 * ROWB, 0, 0);
  }
};
__device__ inline __amdgpu_buffer_rsrc_t head_rsrc(const void* base, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, bytes, 0x00020000);
}
__device__ inline void wait_loads() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Per-lane byte offsets of the MFMA A operands inside a streamed tile (the swizzle depends on the
// low four bits of the row only, so a 32-row block or a 16-row step adds a multiple of the row
// length).
//  rows[s]:   row-wise operand of contraction step s: the 16-byte chunk 2*s + hh of tile row
//             lane%32 (contraction slots 8*hh .. 8*hh+7 of the step).
//  tr[cb][.]: operand of a product that contracts over the tile's rows (the tile transposed):
//             output rows are the channels 32*cb + lane%32, the contraction runs over 16 tile rows
//             in the order an accumulator enumerates them (slot j of lane half hh = row
//             8*(j/4) + 4*hh + j%4), read by two ds_read_b64_tr_b16 (within 16 lanes, lane i
//             receives element i%4 of the 8-byte pieces addressed by lanes 4j + i/4, j = 0..3):
//             this lane addresses rows 4*hh + (lane%16)/4 and that + 8.
template <int D>
struct OperandOffsets {
  int rows[D / 16];
  int tr[D / 32][2];
  __device__ OperandOffsets(int lane) {
    const int lq = lane & 31, hh = lane >> 5;
#pragma unroll
    for (int s = 0; s < D / 16; ++s) rows[s] = (int)(chunk_addr<D>(nullptr, lq, 2 * s + hh) - (char*)nullptr);
    const int row = 4 * hh + ((lane & 15) >> 2);
    const int inb = 8 * (lane & 1);
#pragma unroll
    for (int cb = 0; cb < D / 32; ++cb) {
      const int chunk = 4 * cb + 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1);
      tr[cb][0] = (int)(chunk_addr<D>(nullptr, row, chunk) - (char*)nullptr) + inb;
      tr[cb][1] = (int)(chunk_addr<D>(nullptr, row + 8, chunk) - (char*)nullptr) + inb;
    }
  }
};

// all row-wise operands of the 32-row block `blk` of a tile
template <int D>
__device__ inline void read_rows(const char* tile, int blk, const OperandOffsets<D>& off, bf16x8 (&a)[D / 16]) {
#pragma unroll
  for (int s = 0; s < D / 16; ++s) a[s] = *(const bf16x8*)(tile + blk * 32 * (D * 2) + off.rows[s]);
}

// all transposed operands of the 32-row block `blk`: [channel block][16-row step]
template <int D>
__device__ inline void read_transposed(const char* tile, int blk, const OperandOffsets<D>& off,
                                       bf16x8 (&a)[D / 32][2]) {
#pragma unroll
  for (int cb = 0; cb < D / 32; ++cb)
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
      const char* base = tile + (blk * 32 + tt * 16) * (D * 2);
      s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(base + off.tr[cb][0]));
      s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(base + off.tr[cb][1]));
      s16x8 r = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
      a[cb][tt] = __builtin_bit_cast(bf16x8, r);
    }
}

// nothing moves across: operand reads issued before it stay ahead of the MFMAs behind it
__device__ inline void fence() { __builtin_amdgcn_sched_barrier(0); }

// tile row that register i of a 32 x 32 accumulator block holds, for lane half hh
__device__ inline int acc_row(int i, int hh) { return 8 * (i >> 2) + 4 * hh + (i & 3); }

__device__ inline void zero(f32x16& x) {
#pragma unroll
  for (int i = 0; i < 16; ++i) x[i] = 0.0f;
}

}  // namespace

// ------------------------------------------------------------------------------------------------
// D_i = sum_c dO_ic O_ic and lse_i * log2(e) for every query row; for DistrAttention also Q~:
// channel c of a row takes the value of the first channel (sorted order) of c's group in the
// row's Q block.
template <int D>
__global__ __launch_bounds__(kBwdThreads) void bwd_prepare_kernel(
    const bf16* __restrict__ q, const bf16* __restrict__ o, const bf16* __restrict__ dout,
    const float* __restrict__ lse, const uint8_t* __restrict__ perm, bf16* __restrict__ qrep,
    float* __restrict__ delta, float* __restrict__ lse2, int N, int Br, int Tq, int n_groups) {
  constexpr int CH = D / 8;
  constexpr int RPP = kBwdThreads / CH;   // rows per pass
  __shared__ uint8_t rep_lds[D];
  __shared__ __attribute__((aligned(16))) bf16 row_lds[RPP][D];
  const int tid = threadIdx.x;
  const int t = blockIdx.x % Tq;
  const size_t bh = blockIdx.x / Tq;
  const int r0 = t * Br;
  const int rows = min(Br, N - r0);
  if (perm) {
    const int G = D / n_groups;
    for (int i = tid; i < D; i += kBwdThreads) {
      const uint8_t* pr = perm + (size_t)blockIdx.x * D;
      rep_lds[pr[i] & (D - 1)] = pr[i / G * G] & (D - 1);
    }
  }
  const int rr = tid / CH, chunk = tid % CH;
  for (int p0 = 0; p0 < rows; p0 += RPP) {
    const int row = p0 + rr;
    const bool on = row < rows;
    const size_t off = ((bh * N) + r0 + (on ? row : 0)) * D + chunk * 8;
    float acc = 0.0f;
    if (on) {
      const bf16x8 a = *(const bf16x8*)(dout + off), b = *(const bf16x8*)(o + off);
#pragma unroll
      for (int j = 0; j < 8; ++j) acc = __builtin_fmaf((float)a[j], (float)b[j], acc);
    }
#pragma unroll
    for (int m = 1; m < CH; m <<= 1) acc += __shfl_xor(acc, m);
    if (on && chunk == 0) {
      delta[bh * N + r0 + row] = acc;
      lse2[bh * N + r0 + row] = lse[bh * N + r0 + row] * kLog2e;
    }
    if (perm) {
      __syncthreads();   // rep_lds written; the previous pass's reads of row_lds done
      if (on) *(bf16x8*)&row_lds[rr][chunk * 8] = *(const bf16x8*)(q + off);
      __syncthreads();
      if (on) {
        bf16x8 y;
#pragma unroll
        for (int j = 0; j < 8; ++j) y[j] = row_lds[rr][rep_lds[chunk * 8 + j] & (D - 1)];
        *(bf16x8*)(qrep + off) = y;
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(kBwdThreads, 2) void bwd_dq_kernel(
    const bf16* __restrict__ qrep, const bf16* __restrict__ k, const bf16* __restrict__ v,
    const bf16* __restrict__ dout, const float* __restrict__ lse2p, const float* __restrict__ delta,
    bf16* __restrict__ dq, const uint8_t* __restrict__ perm, int H, int Hkv, int N, int Nk, int Br, int Tq,
    int Tw, int n_groups, int causal, float scale) {
  constexpr int CH = D / 8;
  constexpr int KS = D / 16;    // MFMA steps over the channels
  constexpr int CB = D / 32;    // 32-channel blocks of the dQ~ accumulator
  constexpr int TILE = kBwdStream * D * 2;
  // separate objects: the compiler then does not make reads of one buffer wait for loads in
  // flight into another
  __shared__ __attribute__((aligned(1024))) char k_lds0[TILE];
  __shared__ __attribute__((aligned(1024))) char k_lds1[TILE];
  __shared__ __attribute__((aligned(1024))) char v_lds0[TILE];
  __shared__ __attribute__((aligned(1024))) char v_lds1[TILE];
  __shared__ uint8_t perm_lds[kBwdRows / 32][D];
  __shared__ uint8_t group_lds[kBwdRows / 32][D];   // group whose sampled channel c is, else 255

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int lq = lane & 31, hh = lane >> 5;
  // causal: the blocks with the most keys first
  const int t = causal ? Tw - 1 - (int)(blockIdx.x % Tw) : (int)(blockIdx.x % Tw);
  const size_t bh = blockIdx.x / Tw;
  const int b = (int)(bh / H), h = (int)(bh % H);
  const int hk = h / (H / Hkv);
  const int r0 = t * kBwdRows;
  const int rows = min(kBwdRows, N - r0);
  const int q_abs = r0 + 32 * w + lq;
  const bool active = q_abs < N;
  const int shift = Nk - N;
  const float sl2e = scale * kLog2e;

  const unsigned head_bytes = (unsigned)Nk * D * 2;
  const __amdgpu_buffer_rsrc_t k_rsrc = head_rsrc(k + (size_t)(b * Hkv + hk) * Nk * D, head_bytes);
  const __amdgpu_buffer_rsrc_t v_rsrc = head_rsrc(v + (size_t)(b * Hkv + hk) * Nk * D, head_bytes);
  const TileLoader<D> loader(w, lane);
  const int n_end = causal ? min(Nk, r0 + rows + shift) : Nk;
  const int n_tiles = ((n_end + kBwdStream - 1) / kBwdStream + 1) & ~1;   // even
  // tiles that end at or before n_free need no mask for any row of the workgroup
  const int n_free = causal ? min(r0 + shift + 1, Nk) : Nk;
  loader.load(k_rsrc, 0, k_lds0);
  loader.load(v_rsrc, 0, v_lds0);

  const size_t row_off = (bh * N + (active ? q_abs : r0)) * D;
  bf16x8 qop[KS], doop[KS];
#pragma unroll
  for (int s = 0; s < KS; ++s) {
    u32x4 x = {0u, 0u, 0u, 0u}, y = {0u, 0u, 0u, 0u};
    if (active) {
      x = *(const u32x4*)(qrep + row_off + (2 * s + hh) * 8);
      y = *(const u32x4*)(dout + row_off + (2 * s + hh) * 8);
    }
    qop[s] = __builtin_bit_cast(bf16x8, x);
    doop[s] = __builtin_bit_cast(bf16x8, y);
  }
  const float lse2 = active ? lse2p[bh * N + q_abs] : 0.0f;
  const float dl = active ? delta[bh * N + q_abs] : 0.0f;
  const int lim = causal ? min(q_abs + shift, Nk - 1) : Nk - 1;   // last key this row sees

  f32x16 dqacc[CB];
#pragma unroll
  for (int cb = 0; cb < CB; ++cb) zero(dqacc[cb]);

  const OperandOffsets<D> off(lane);
  // dS^T of one 32-key block as B operands
  auto ds_operands = [&](const f32x16& sacc, const f32x16& dpacc, int kv0, auto masked_c, bf16x8 (&dsop)[2]) {
    float pv[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) pv[i] = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[i], sl2e, -lse2));
    if constexpr (decltype(masked_c)::value) {
#pragma unroll
      for (int i = 0; i < 16; ++i) pv[i] = kv0 + acc_row(i, hh) <= lim ? pv[i] : 0.0f;
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) dsop[i >> 3][i & 7] = (bf16)(pv[i] * (dpacc[i] - dl));
  };
  auto dq_update = [&](const bf16x8 (&at)[CB][2], const bf16x8 (&dsop)[2]) {
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) dqacc[cb] = mfma(at[cb][tt], dsop[tt], dqacc[cb]);
  };

  // One tile; the loop is unrolled by two so that every buffer is a fixed object in each copy
  // (the compiler then knows that the loads in flight do not touch the tile being read). Tiles
  // that need the mask take a copy of the body of their own.
  auto tile_step = [&](auto par_c, auto masked, int n0) __attribute__((always_inline)) {
    constexpr int par = decltype(par_c)::value;
    const char* k_lds = par ? k_lds1 : k_lds0;
    const char* v_lds = par ? v_lds1 : v_lds0;
    wait_loads();
    __syncthreads();   // this tile has landed; the other buffers' readers are done
    if (n0 + kBwdStream < n_tiles * kBwdStream) {
      loader.load(k_rsrc, n0 + kBwdStream, par ? k_lds0 : k_lds1);
      loader.load(v_rsrc, n0 + kBwdStream, par ? v_lds0 : v_lds1);
    }
    // Two waves share a SIMD (a single wave cannot fill it: its LDS reads alone take as many
    // issue cycles as its MFMAs take pipe cycles), so the blocks follow one another and operands
    // are read in batches of HB contraction steps in front of their MFMAs (all of them at d = 64;
    // at d = 128 two batches: with the 96 accumulator registers the whole set does not fit beside
    // the resident operands).
    constexpr int HB = D == 128 ? KS / 2 : KS;
#pragma unroll
    for (int mb = 0; mb < kBwdStream / 32; ++mb) {
      bf16x8 ak[HB], av[HB], at[CB][2], ds[2];
      f32x16 sacc, dpacc;
      zero(sacc);
      zero(dpacc);
#pragma unroll
      for (int h0 = 0; h0 < KS; h0 += HB) {
#pragma unroll
        for (int s = 0; s < HB; ++s) {
          ak[s] = *(const bf16x8*)(k_lds + mb * 32 * (D * 2) + off.rows[h0 + s]);
          av[s] = *(const bf16x8*)(v_lds + mb * 32 * (D * 2) + off.rows[h0 + s]);
        }
        fence();
#pragma unroll
        for (int s = 0; s < HB; ++s) {
          sacc = mfma(ak[s], qop[h0 + s], sacc);
          dpacc = mfma(av[s], doop[h0 + s], dpacc);
        }
        fence();
      }
      ds_operands(sacc, dpacc, n0 + 32 * mb, masked, ds);
      read_transposed<D>(k_lds, mb, off, at);
      fence();
      dq_update(at, ds);
      fence();
    }
  };
  // Tiles [a, b), b - a even, with or without the mask; buffer parity = tile parity. The loop is
  // unrolled by two over fixed buffers; masked and unmasked tiles run in loops of their own (both
  // copies under a branch inside one loop cost 200 spilled registers). The tile count is rounded
  // up to an even number: a tile past the last visible key is masked out entirely.
  auto run = [&](int a, int b, auto masked_c) {
    for (int t = a; t < b; t += 2) {
      tile_step(std::integral_constant<int, 0>(), masked_c, t * kBwdStream);
      tile_step(std::integral_constant<int, 1>(), masked_c, (t + 1) * kBwdStream);
    }
  };
  const int free_tiles = min(n_free / kBwdStream, n_tiles) & ~1;
  run(0, free_tiles, std::false_type());
  run(free_tiles, n_tiles, std::true_type());

  // Epilogue: every wave puts the dQ~ of its 32 rows into LDS (float; the column index XORed
  // with the row so that a register's 32 rows fall into different banks) and sums, for every
  // group of its rows' Q block, the members' columns into the sampled channel; the other channels
  // get 0.
  __syncthreads();   // all waves are done with the tiles
  float* stage = (float*)(w == 0 ? k_lds0 : w == 1 ? k_lds1 : w == 2 ? v_lds0 : v_lds1);
  static_assert(32 * D * 4 <= TILE, "a wave's staging fits one tile buffer");
#pragma unroll
  for (int cb = 0; cb < CB; ++cb)
#pragma unroll
    for (int i = 0; i < 16; ++i) stage[lq * D + ((32 * cb + acc_row(i, hh)) ^ lq)] = dqacc[cb][i];
  const int G = D / n_groups;
  {
    const int blk = (r0 + 32 * w) / Br;   // a wave's 32 rows lie in one Q block (Br is a multiple of 32)
    const uint8_t* pr = perm ? perm + (bh * Tq + min(blk, Tq - 1)) * D : nullptr;
    for (int i = lane; i < D; i += 64) {
      perm_lds[w][i] = pr ? (pr[i] & (D - 1)) : (uint8_t)i;
      group_lds[w][i] = 255;
    }
  }
  __syncthreads();
  for (int j = lane; j < n_groups; j += 64) group_lds[w][perm_lds[w][j * G]] = (uint8_t)j;
  __syncthreads();
  for (int id = lane; id < 32 * CH; id += 64) {
    const int lr = id / CH, chunk = id % CH;
    const int row = r0 + 32 * w + lr;
    if (row >= N) continue;
    bf16x8 y;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int j = group_lds[w][chunk * 8 + e];
      float s = 0.0f;
      if (j != 255)
        for (int m = 0; m < G; ++m) s += stage[lr * D + (perm_lds[w][j * G + m] ^ lr)];
      y[e] = (bf16)(scale * s);
    }
    *(bf16x8*)(dq + (bh * N + row) * D + chunk * 8) = y;
  }
}

// What the dK/dV kernel streams: iteration `it` brings rows i_start + 64 * (it % tiles) .. of
// query head bh0 + it / tiles (Q~, dO, and the rows' statistics) into the given buffers.
template <int D>
struct QueryStream {
  const bf16 *qrep, *dout;
  const float *lse2, *delta;
  size_t bh0;   // b * H + first query head of the kv head
  int N, i_start, tiles, wave, lane;
  TileLoader<D> loader;
  __device__ void issue(int it, char* q_dst, char* do_dst, float* lse_dst, float* dl_dst) const {
    const size_t bh = bh0 + it / tiles;
    const int i0 = i_start + kBwdStream * (it % tiles);
    const unsigned head_bytes = (unsigned)N * D * 2;
    loader.load(head_rsrc(qrep + bh * N * D, head_bytes), i0, q_dst);
    loader.load(head_rsrc(dout + bh * N * D, head_bytes), i0, do_dst);
    if (wave == 0)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(head_rsrc(lse2 + bh * N, (unsigned)N * 4), (lds_void*)lse_dst, 4,
                                               lane * 4, i0 * 4, 0, 0);
    if (wave == 1)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(head_rsrc(delta + bh * N, (unsigned)N * 4), (lds_void*)dl_dst, 4,
                                               lane * 4, i0 * 4, 0, 0);
  }
};

// ------------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(kBwdThreads, (D == 64 ? 2 : 1)) void bwd_dkv_kernel(
    const bf16* __restrict__ qrep, const bf16* __restrict__ k, const bf16* __restrict__ v,
    const bf16* __restrict__ dout, const float* __restrict__ lse2p, const float* __restrict__ delta,
    bf16* __restrict__ dk, bf16* __restrict__ dv, float* __restrict__ part, int hsplit, int H, int Hkv, int N,
    int Nk, int Tw, int causal, float scale) {
  constexpr int KS = D / 16;
  constexpr int CB = D / 32;
  constexpr int TILE = kBwdStream * D * 2;
  __shared__ __attribute__((aligned(1024))) char q_lds0[TILE];
  __shared__ __attribute__((aligned(1024))) char q_lds1[TILE];
  __shared__ __attribute__((aligned(1024))) char do_lds0[TILE];
  __shared__ __attribute__((aligned(1024))) char do_lds1[TILE];
  __shared__ __attribute__((aligned(256))) float lse_lds0[kBwdStream];   // lse * log2(e)
  __shared__ __attribute__((aligned(256))) float lse_lds1[kBwdStream];
  __shared__ __attribute__((aligned(256))) float dl_lds0[kBwdStream];
  __shared__ __attribute__((aligned(256))) float dl_lds1[kBwdStream];

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int lq = lane & 31, hh = lane >> 5;
  // hsplit > 1: the query heads of the kv head are dealt out to hsplit workgroups, which leave
  // float partial sums in `part` for the reduction kernel
  const int hs = blockIdx.x % hsplit;
  const int t = (blockIdx.x / hsplit) % Tw;
  const size_t bk = blockIdx.x / hsplit / Tw;   // b * Hkv + hk
  const int b = (int)(bk / Hkv), hk = (int)(bk % Hkv);
  const int rep = H / Hkv / hsplit;             // query heads of this workgroup
  const int n0 = t * kBwdRows;
  const int key = n0 + 32 * w + lq;
  const bool valid = key < Nk;
  const int shift = Nk - N;
  const float sl2e = scale * kLog2e;

  // causal: query i sees key n iff n <= i + shift; the first tile with a row that sees key n0
  const int i_start = causal ? max(0, n0 - shift) / kBwdStream * kBwdStream : 0;
  const int tiles = ((N - i_start + kBwdStream - 1) / kBwdStream + 1) & ~1;   // per query head, even
  const int n_it = rep * tiles;
  const TileLoader<D> loader(w, lane);
  const QueryStream<D> ctx = {qrep, dout, lse2p, delta, (size_t)b * H + (hk * hsplit + hs) * rep, N, i_start, tiles, w, lane, loader};
  ctx.issue(0, q_lds0, do_lds0, lse_lds0, dl_lds0);

  bf16x8 kop[KS], vop[KS];
  {
    const size_t row_off = (bk * Nk + (valid ? key : n0)) * D;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      u32x4 x = {0u, 0u, 0u, 0u}, y = {0u, 0u, 0u, 0u};
      if (valid) {
        x = *(const u32x4*)(k + row_off + (2 * s + hh) * 8);
        y = *(const u32x4*)(v + row_off + (2 * s + hh) * 8);
      }
      kop[s] = __builtin_bit_cast(bf16x8, x);
      vop[s] = __builtin_bit_cast(bf16x8, y);
    }
  }
  f32x16 dkacc[CB], dvacc[CB];
#pragma unroll
  for (int cb = 0; cb < CB; ++cb) {
    zero(dkacc[cb]);
    zero(dvacc[cb]);
  }

  const OperandOffsets<D> off(lane);
  // One tile; the loop is unrolled by two so that every buffer is a fixed object in each copy
  // (the compiler then knows that the loads in flight do not touch the tile being read).
  auto tile_step = [&](auto par_c, auto masked_c, int it) __attribute__((always_inline)) {
    constexpr int par = decltype(par_c)::value;
    const char* q_lds = par ? q_lds1 : q_lds0;
    const char* do_lds = par ? do_lds1 : do_lds0;
    const float* lse_lds = par ? lse_lds1 : lse_lds0;
    const float* dl_lds = par ? dl_lds1 : dl_lds0;
    const int i0 = i_start + kBwdStream * (it % tiles);
    // Register classes, stated once per tile: the accumulators of dK and dV live in the
    // accumulator half of the register file, the resident K and V operands in the vector half
    // (left to itself the allocator moved 128 accumulator registers back and forth per tile).
    if constexpr (D == 128) {
#pragma unroll
      for (int cb = 0; cb < CB; ++cb) asm volatile("" : "+a"(dkacc[cb]), "+a"(dvacc[cb]));
#pragma unroll
      for (int s = 0; s < KS; ++s) asm volatile("" : "+v"(kop[s]), "+v"(vop[s]));
    }
    wait_loads();
    __syncthreads();   // this tile has landed; the other buffers' readers are done
    if (it + 1 < n_it) {
      if constexpr (par) ctx.issue(it + 1, q_lds0, do_lds0, lse_lds0, dl_lds0);
      else ctx.issue(it + 1, q_lds1, do_lds1, lse_lds1, dl_lds1);
    }
    // Operands are read a phase ahead of the MFMAs that take them; the vector work of a 32-row
    // block sits next to the matrix work of the other one.
    bf16x8 ar[KS], at[CB][2], pop0[2], ds0[2], pop1[2], ds1[2];
    f32x16 s0, p0, s1, p1;
    f32x4 l4[4], d4[4];
    auto product = [&](const bf16x8 (&b)[KS], f32x16& acc) {
      zero(acc);
#pragma unroll
      for (int s = 0; s < KS; ++s) acc = mfma(ar[s], b[s], acc);
    };
    auto read_stats = [&](int qb) {
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        l4[i4] = *(const f32x4*)&lse_lds[32 * qb + 8 * i4 + 4 * hh];
        d4[i4] = *(const f32x4*)&dl_lds[32 * qb + 8 * i4 + 4 * hh];
      }
    };
    auto p_ds_operands = [&](const f32x16& sacc, const f32x16& dpacc, int qb, bf16x8 (&pop)[2], bf16x8 (&dsop)[2]) {
      float pv[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) pv[i] = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[i], sl2e, -l4[i >> 2][i & 3]));
      if constexpr (decltype(masked_c)::value) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int qi = i0 + 32 * qb + acc_row(i, hh);
          const bool vis = valid && qi < N && !(causal && key > qi + shift);
          pv[i] = vis ? pv[i] : 0.0f;
        }
      }
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        pop[i >> 3][i & 7] = (bf16)pv[i];
        dsop[i >> 3][i & 7] = (bf16)(pv[i] * (dpacc[i] - d4[i >> 2][i & 3]));
      }
    };
    auto update = [&](const bf16x8 (&b)[2], f32x16 (&acc)[CB]) {
#pragma unroll
      for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) acc[cb] = mfma(at[cb][tt], b[tt], acc[cb]);
    };
    read_rows<D>(q_lds, 0, off, ar);
    fence();
    product(kop, s0);
    read_rows<D>(do_lds, 0, off, ar);
    fence();
    product(vop, p0);
    read_rows<D>(q_lds, 1, off, ar);
    read_stats(0);
    fence();
    product(kop, s1);
    read_rows<D>(do_lds, 1, off, ar);
    fence();
    product(vop, p1);
    p_ds_operands(s0, p0, 0, pop0, ds0);
    read_transposed<D>(do_lds, 0, off, at);
    fence();
    update(pop0, dvacc);
    read_transposed<D>(q_lds, 0, off, at);
    read_stats(1);
    fence();
    update(ds0, dkacc);
    p_ds_operands(s1, p1, 1, pop1, ds1);
    read_transposed<D>(do_lds, 1, off, at);
    fence();
    update(pop1, dvacc);
    read_transposed<D>(q_lds, 1, off, at);
    fence();
    update(ds1, dkacc);
  };
  // Iterations [a, b), b - a even, with or without the mask; buffer parity = iteration parity.
  // The loop is unrolled by two over fixed buffers, masked and unmasked tiles run in loops of
  // their own.
  auto run = [&](int a, int b, auto masked_c) {
    for (int it = a; it < b; it += 2) {
      tile_step(std::integral_constant<int, 0>(), masked_c, it);
      tile_step(std::integral_constant<int, 1>(), masked_c, it + 1);
    }
  };
  // Per query head (an even number of tiles; a tile past the last query row is masked out
  // entirely): the first m1 tiles touch the causal diagonal (all tiles, when some key of the
  // workgroup does not exist), the last two may hold rows past N; the tiles between need no
  // mask: every row is a query, every key exists and is visible to all rows.
  int m1 = 0;
  if (n0 + kBwdRows > Nk) m1 = tiles;
  else if (causal) m1 = min(tiles, (max(0, (n0 + kBwdRows - 1 - shift - i_start + kBwdStream - 1) / kBwdStream) + 1) & ~1);
  const int m2 = (i_start + tiles * kBwdStream > N && m1 < tiles) ? 2 : 0;
  for (int hh_ = 0; hh_ < rep; ++hh_) {
    const int base = hh_ * tiles;
    run(base, base + m1, std::true_type());
    run(base + m1, base + tiles - m2, std::false_type());
    run(base + tiles - m2, base + tiles, std::true_type());
  }
  if (valid && hsplit > 1) {
    // partial sums: [dK | dV][hsplit][B * Hkv * Nk][D] float
    const size_t elems = (size_t)gridDim.x / hsplit / Tw * Nk * D;
    float* dkrow = part + (size_t)hs * elems + (bk * Nk + key) * D;
    float* dvrow = dkrow + (size_t)hsplit * elems;
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        const int c = 32 * cb + 8 * i4 + 4 * hh;
        f32x4 a, bq;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          a[e] = scale * dkacc[cb][4 * i4 + e];
          bq[e] = dvacc[cb][4 * i4 + e];
        }
        *(f32x4*)(dkrow + c) = a;
        *(f32x4*)(dvrow + c) = bq;
      }
  } else if (valid) {
    bf16* dkrow = dk + (bk * Nk + key) * D;
    bf16* dvrow = dv + (bk * Nk + key) * D;
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        const int c = 32 * cb + 8 * i4 + 4 * hh;
        bf16x4 a, bq;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          a[e] = (bf16)(scale * dkacc[cb][4 * i4 + e]);
          bq[e] = (bf16)dvacc[cb][4 * i4 + e];
        }
        *(bf16x4*)(dkrow + c) = a;
        *(bf16x4*)(dvrow + c) = bq;
      }
  }
}

// dK and dV from the partial sums of the head-split dK/dV launch: out = sum over the hsplit parts,
// in a fixed order (results do not depend on the run), rounded once.
__global__ __launch_bounds__(256) void bwd_reduce_kernel(const float* __restrict__ part, bf16* __restrict__ dk,
                                                         bf16* __restrict__ dv, size_t elems, int hsplit) {
  const size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i >= 2 * elems) return;
  const bool second = i >= elems;
  const size_t j = second ? i - elems : i;
  const float* src = part + (second ? (size_t)hsplit * elems : 0) + j;
  f32x4 acc = *(const f32x4*)src;
  for (int s = 1; s < hsplit; ++s) acc += *(const f32x4*)(src + (size_t)s * elems);
  bf16x4 y = {(bf16)acc[0], (bf16)acc[1], (bf16)acc[2], (bf16)acc[3]};
  *(bf16x4*)((second ? dv : dk) + j) = y;
}

// Workgroups of the dK/dV launch that share one kv head's keys but take different query heads: used
// when the launch would otherwise not fill the chip twice over (grouped-query shapes with few kv
// heads; under the causal mask its workgroups differ many-fold in length and need company).
static int dkv_head_split(const Problem& pb) {
  const int rep = pb.H / pb.Hkv;
  const long long k_units = (long long)pb.B * pb.Hkv * ((pb.Nk + kBwdRows - 1) / kBwdRows);
  return (rep > 1 && k_units < 512) ? rep : 1;
}

size_t attn_bf16_bwd_scratch_bytes(const Problem& pb, int distr) {
  const size_t rows = (size_t)pb.B * pb.H * pb.N;
  const size_t stat = (rows * 4 + 255) & ~(size_t)255;   // D_i, and lse * log2(e)
  const int hsplit = dkv_head_split(pb);
  const size_t part = hsplit > 1 ? ((size_t)2 * hsplit * pb.B * pb.Hkv * pb.Nk * pb.d * 4 + 255) & ~(size_t)255 : 0;
  return 2 * stat + (distr ? ((rows * pb.d * 2 + 255) & ~(size_t)255) : 0) + part;
}

hipError_t launch_attn_bf16_bwd(const void* q, const void* k, const void* v, const void* o, const void* dout,
                                const float* lse, void* dq, void* dk, void* dv, const uint8_t* perm, void* scratch,
                                const Problem& pb, int distr, hipStream_t stream) {
  const int Tq = (pb.N + pb.Br - 1) / pb.Br;
  const int Twq = (pb.N + kBwdRows - 1) / kBwdRows;
  const int Twk = (pb.Nk + kBwdRows - 1) / kBwdRows;
  const long long prep_units = (long long)pb.B * pb.H * Tq;
  const long long q_units = (long long)pb.B * pb.H * Twq;
  const long long k_units = (long long)pb.B * pb.Hkv * Twk;
  if (prep_units > 0x7fffffffLL || q_units > 0x7fffffffLL || k_units > 0x7fffffffLL / 16) return hipErrorInvalidValue;
  if ((pb.d != 64 && pb.d != 128) || pb.Br % 32 != 0 || pb.d % pb.n_groups != 0) return hipErrorInvalidValue;
  // tiles are addressed by 32-bit byte offsets inside a head
  if ((size_t)pb.N * pb.d * 2 >= 0x7fffffffULL || (size_t)pb.Nk * pb.d * 2 >= 0x7fffffffULL) return hipErrorInvalidValue;
  const size_t rows = (size_t)pb.B * pb.H * pb.N;
  const size_t stat = (rows * 4 + 255) & ~(size_t)255;
  float* delta = (float*)scratch;
  float* lse2 = (float*)((char*)scratch + stat);
  bf16* qrep = distr ? (bf16*)((char*)scratch + 2 * stat) : nullptr;
  const int hsplit = dkv_head_split(pb);
  float* part = hsplit > 1 ? (float*)((char*)scratch + 2 * stat + (distr ? ((rows * pb.d * 2 + 255) & ~(size_t)255) : 0)) : nullptr;
  const size_t kv_elems = (size_t)pb.B * pb.Hkv * pb.Nk * pb.d;
  const uint8_t* table = distr ? perm : nullptr;
  const bf16* qx = distr ? qrep : (const bf16*)q;
  const int n_groups = distr ? pb.n_groups : pb.d;
#define DA_BWD(DD)                                                                                                   \
  do {                                                                                                               \
    hipLaunchKernelGGL((bwd_prepare_kernel<DD>), dim3((unsigned)prep_units), dim3(kBwdThreads), 0, stream,           \
                       (const bf16*)q, (const bf16*)o, (const bf16*)dout, lse, table, qrep, delta, lse2, pb.N, pb.Br, Tq, n_groups); \
    hipLaunchKernelGGL((bwd_dq_kernel<DD>), dim3((unsigned)q_units), dim3(kBwdThreads), 0, stream, qx, (const bf16*)k, \
                       (const bf16*)v, (const bf16*)dout, lse2, delta, (bf16*)dq, table, pb.H, pb.Hkv, pb.N, pb.Nk,   \
                       pb.Br, Tq, Twq, n_groups, pb.causal, pb.scale);                                               \
    hipLaunchKernelGGL((bwd_dkv_kernel<DD>), dim3((unsigned)(k_units * hsplit)), dim3(kBwdThreads), 0, stream, qx,   \
                       (const bf16*)k, (const bf16*)v, (const bf16*)dout, lse2, delta, (bf16*)dk, (bf16*)dv, part,    \
                       hsplit, pb.H, pb.Hkv, pb.N, pb.Nk, Twk, pb.causal, pb.scale);                                 \
    if (hsplit > 1)                                                                                                  \
      hipLaunchKernelGGL(bwd_reduce_kernel, dim3((unsigned)((2 * kv_elems / 4 + 255) / 256)), dim3(256), 0, stream,  \
                         part, (bf16*)dk, (bf16*)dv, kv_elems, hsplit);                                              \
  } while (0)
  if (pb.d == 64) DA_BWD(64);
  else DA_BWD(128);
#undef DA_BWD
  return hipGetLastError();
}

}  // namespace da
