// Row-schedule kernels for f16 storage (see row_stitch_impl.h).
#include "row_stitch_impl.h"

namespace fs {
hipError_t row_launch_f16(const RowArgs& a, const RowLaunch& rl, hipStream_t s) {
  return row_launch_dtype<f16_t>(a, rl, s);
}
}  // namespace fs
