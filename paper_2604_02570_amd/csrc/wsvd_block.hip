// Grouped-query decode attention (more than 4 query heads per kv head) and the W4A8 linear layer of the
// full attention block.
#include "wsvd_attn_common.h"
#include "wsvd_internal.h"

hipError_t wsvd_launch_attn_gqa(const AttnParams&, int, int, dim3, hipStream_t) { return hipErrorNotSupported; }

hipError_t wsvd_launch_linear_w4a8(const int8_t*, const void*, const void*, const void*, int64_t, int64_t, int64_t, float*,
                                   hipStream_t) {
  return hipErrorNotSupported;
}
