// Plain streaming copy: the achievable-bandwidth yardstick beside the stitched kernels and
// the calibration kernel for HBM byte counters.  It uses the same access path as the
// stitched kernels (one-shot grid, 16 bytes per lane, nontemporal loads and stores), the
// fastest copy shape measured on MI355X, so that a byte counter reads it the same way.
#include "dev_common.h"
#include "launchers.h"

namespace fs {

__global__ __launch_bounds__(256) void stream_copy_kernel(u32x4* __restrict__ dst,
                                                          const u32x4* __restrict__ src, int64_t nvec) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < nvec) stream_store16(dst + i, stream_load16(src + i));
}

int stream_copy_launch(void* dst, const void* src, int64_t bytes, void* stream, std::string* err) {
  const int64_t nvec = bytes / 16;
  if (nvec == 0) return 0;
  const int64_t grid = (nvec + 255) / 256;
  if (grid > 0x7fffffff) { *err = "stream_copy: more than 2^31 workgroups"; return -1; }
  hipLaunchKernelGGL(stream_copy_kernel, dim3((unsigned)grid), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<u32x4*>(dst), static_cast<const u32x4*>(src), nvec);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) { *err = std::string("stream_copy launch: ") + hipGetErrorString(e); return -1; }
  return 0;
}

}  // namespace fs
