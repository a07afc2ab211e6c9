// Tree attention on the matrix cores (head_dim 128, bf16).  Placeholder: not enabled yet, the
// generic kernel serves every shape.
#include "tr_kernels.h"

namespace tr {

bool attn_mfma_supported(int32_t, int32_t) { return false; }

hipError_t launch_attn_mfma(const bf16_t *, const bf16_t *, const bf16_t *, int32_t, int32_t, int32_t, int32_t,
                            const uint64_t *, const int32_t *, int32_t, float *, float *, bf16_t *, int32_t, hipStream_t) {
  return hipErrorNotSupported;
}

} // namespace tr
