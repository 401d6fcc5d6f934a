// Shared declarations of the gfx950 DistrAttention library (device helpers + kernel launchers).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace da {

typedef __bf16 bf16;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;

constexpr int kBc = 64;          // key/value rows per tile of the key pre-pass and the default of the attention kernels
constexpr int kKtPad = 128;      // K^T rows are padded to a multiple of the largest key tile
constexpr int kMaxPlanes = 32;   // sign bits per hash

// Projection matrix entry (plane p, row r) of the LSH stage (Sec. 3.2: a fixed random matrix).
// Counter-based: mix a 64-bit counter, add its four 16-bit fields, centre. The value is an
// integer in [-131070, 131070] times 2^-16, so float holds it exactly on host and device.
__host__ __device__ inline float hyperplane_entry(uint64_t seed, uint32_t p, uint32_t r) {
  uint64_t z = seed + 0x9E3779B97F4A7C15ULL * (((uint64_t)p << 32) + (uint64_t)r + 1ULL);
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
  z ^= z >> 31;
  int sum = (int)(z & 0xFFFF) + (int)((z >> 16) & 0xFFFF) + (int)((z >> 32) & 0xFFFF) + (int)(z >> 48);
  return (float)(sum - 131070) * (1.0f / 65536.0f);
}

// Hash of a channel from the sign word of its projections (Sec. 3.2). gray_mode 1: the Gray code
// of the sign word (literal table lookup); otherwise the position of the sign word in the Gray
// sequence, so that hashes differing by one belong to sign words differing in one projection.
__host__ __device__ inline uint32_t lsh_hash_of_code(uint32_t code, int gray_mode) {
  if (gray_mode == 1) return code ^ (code >> 1);
  uint32_t h = code;
  h ^= h >> 1; h ^= h >> 2; h ^= h >> 4; h ^= h >> 8; h ^= h >> 16;
  return h;
}

// Behind the K^T copy the key pre-pass leaves the projection matrix of the LSH stage (Sec. 3.2),
// split into two bf16 pieces r1 + r2 = R, for the attention kernel's own LSH stage at d = 64,
// which otherwise generates it again in every workgroup: a header (seed, projections, block rows)
// at offset 0 and, from offset kRtabHead on, the two pieces [16][Br + 8] bf16, each padded to a
// whole number of 1 KB blocks (the unit of a direct load into LDS).
struct RtabHeader {
  uint64_t seed;
  int32_t n_planes, Br;
};
constexpr int kRtabHead = 1024;
constexpr int rtab_piece_bytes(int Br) { return (16 * (Br + 8) * 2 + 1023) / 1024 * 1024; }
constexpr int kRtabBytes = kRtabHead + 2 * rtab_piece_bytes(256);
// bytes of the K^T copy itself: [B][Hkv][d][Npad] half
inline size_t kt_copy_bytes(int B, int Hkv, int d, int Nk) {
  const size_t npad = (size_t)((Nk + kKtPad - 1) / kKtPad) * kKtPad;
  return ((size_t)B * Hkv * d * npad * 2 + 255) & ~(size_t)255;
}

struct Problem {
  int B, H, Hkv, N, d, Br, n_groups, causal, n_planes, gray_mode;
  uint64_t seed;
  float scale;
  int Nk;     // keys / values per head (N is the number of queries); causal: key n is visible
              // to query i iff n <= i + (Nk - N)
  int side;   // 0: sample Q, fuse K, one grouping per Q block; 1: sample K, fuse Q, one grouping
              // per K block of Bc rows (float-arithmetic kernel)
  int Bc;     // rows of a K block (only side 1 depends on it)
  float* lse; // optional device [B][H][N]: log-sum-exp of every row's visible scores (natural log)
  uint8_t* perm_w = nullptr;   // optional device [B][H][Tq][d]: where the bf16 attention kernel's own LSH
                               // stage leaves its table
};

// Launchers (defined next to their kernels). All return hipError_t of the launch.
hipError_t launch_lsh_group(const void* q, int dtype, const Problem& pb, uint8_t* perm_out,
                            uint32_t* hash_out, hipStream_t stream);
// K [B][Hkv][Nk][d] bf16 -> K^T [B][Hkv][d][Npad] half (Npad = Nk rounded up to kKtPad), for the distr path,
// followed at kt_copy_bytes() by the projection-matrix table (kRtabBytes) for pb's seed, n_planes and Br.
hipError_t launch_kt_prepass(const void* k, void* kt, const Problem& pb, hipStream_t stream);
// distr != 0: S^ = Q_r K_f^T with the per-block permutation table `perm` [B][H][Tq][d] and the
// transposed keys `kt` written by launch_kt_prepass (k itself is then unused; the table behind the
// copy is used when its header matches the call).
hipError_t launch_attn_bf16(const void* q, const void* k, const void* v, void* o, const uint8_t* perm,
                            const void* kt, const Problem& pb, int distr, hipStream_t stream);
hipError_t launch_attn_f32(const void* q, const void* k, const void* v, void* o, const uint8_t* perm,
                           const Problem& pb, int dtype, int distr, hipStream_t stream);
bool attn_bf16_supported(const Problem& pb, int distr);
// Backward in float arithmetic on the vector ALUs (float tensors): dq [B][H][N][d], dk and dv
// [B][Hkv][Nk][d] from the forward's inputs, its output o, the output gradient dout and the
// forward's row statistics lse; perm as in launch_attn_f32.
hipError_t launch_attn_f32_bwd(const void* q, const void* k, const void* v, const void* o, const void* dout,
                               const float* lse, void* dq, void* dk, void* dv, const uint8_t* perm,
                               const Problem& pb, int distr, hipStream_t stream);
// The same for bf16 tensors on the matrix cores; `scratch` (256-byte aligned,
// attn_bf16_bwd_scratch_bytes) carries D_i and the channel-replicated Q between its kernels.
size_t attn_bf16_bwd_scratch_bytes(const Problem& pb, int distr);
hipError_t launch_attn_bf16_bwd(const void* q, const void* k, const void* v, const void* o, const void* dout,
                                const float* lse, void* dq, void* dk, void* dv, const uint8_t* perm, void* scratch,
                                const Problem& pb, int distr, hipStream_t stream);

}  // namespace da
