// Schedule-3 kernels for f16 storage (see attn_stitch_impl.h).
#include "attn_stitch_impl.h"

namespace fs {
hipError_t attn_launch_f16(const AttnArgs& a, int nq, int nk, hipStream_t s) {
  return attn_launch_dtype<f16_t>(a, nq, nk, s);
}
}  // namespace fs
