// Row-schedule kernels for bf16 storage (see row_stitch_impl.h).
#include "row_stitch_impl.h"

namespace fs {
hipError_t row_launch_bf16(const RowArgs& a, const RowLaunch& rl, hipStream_t s) {
  return row_launch_dtype<bf16_t>(a, rl, s);
}
}  // namespace fs
