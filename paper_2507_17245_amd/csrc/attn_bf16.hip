// Entry of the bf16 attention kernels: which shapes are built, and the dispatch over the K/V tile
// size (one translation unit per tile size: attn_bf16_bc32/64/128.hip, kernel in attn_bf16_impl.h).
#include "da_common.h"

namespace da {

hipError_t launch_attn_bf16_bc32(const void*, const void*, const void*, void*, const uint8_t*, const void*,
                                 const Problem&, int, hipStream_t);
hipError_t launch_attn_bf16_bc64(const void*, const void*, const void*, void*, const uint8_t*, const void*,
                                 const Problem&, int, hipStream_t);
hipError_t launch_attn_bf16_bc128(const void*, const void*, const void*, void*, const uint8_t*, const void*,
                                  const Problem&, int, hipStream_t);

bool attn_bf16_supported(const Problem& pb, int distr) {
  if (pb.d != 64 && pb.d != 128) return false;
  if (pb.Br != 64 && pb.Br != 128 && pb.Br != 256) return false;
  if (pb.Bc != 32 && pb.Bc != 64 && pb.Bc != 128) return false;
  if (distr) {
    // groups of up to 16 channels (G* in {1, 2, 4, 8, 16}, Sec. 3.2 and Table 4); K/V tiles other
    // than 64 rows are built for 16, 32 and 64 groups
    const int kr = pb.n_groups;
    if (kr > pb.d || pb.d % kr != 0 || pb.d / kr > 16) return false;
    if (kr == pb.d) return true;
    if (kr != 4 && kr != 8 && kr != 16 && kr != 32 && kr != 64) return false;
    if (pb.Bc != 64 && kr < 16) return false;
  }
  return true;
}

hipError_t launch_attn_bf16(const void* q, const void* k, const void* v, void* o, const uint8_t* perm,
                            const void* kt, const Problem& pb, int distr, hipStream_t stream) {
  if (!attn_bf16_supported(pb, distr)) return hipErrorInvalidValue;
  if (distr && !kt) return hipErrorInvalidValue;
  if (pb.Bc == 32) return launch_attn_bf16_bc32(q, k, v, o, perm, kt, pb, distr, stream);
  if (pb.Bc == 128) return launch_attn_bf16_bc128(q, k, v, o, perm, kt, pb, distr, stream);
  return launch_attn_bf16_bc64(q, k, v, o, perm, kt, pb, distr, stream);
}

}  // namespace da
