// Schedule-3 kernels for bf16 storage (see attn_stitch_impl.h).
#include "attn_stitch_impl.h"

namespace fs {
hipError_t attn_launch_bf16(const AttnArgs& a, int nq, int nk, hipStream_t s) {
  return attn_launch_dtype<bf16_t>(a, nq, nk, s);
}
}  // namespace fs
