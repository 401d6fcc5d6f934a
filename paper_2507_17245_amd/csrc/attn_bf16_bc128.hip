// bf16 attention kernels (exact and DistrAttention) with K/V tiles of 128 rows: see attn_bf16_impl.h.
#include "attn_bf16_impl.h"

namespace da {

hipError_t launch_attn_bf16_bc128(const void* q, const void* k, const void* v, void* o, const uint8_t* perm,
                                 const void* kt, const Problem& pb, int distr, hipStream_t stream) {
  return dispatch_shape<128>(q, k, v, o, perm, kt, pb, distr, stream);
}

}  // namespace da
