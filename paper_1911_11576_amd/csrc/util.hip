// Plain streaming copy: the achievable-bandwidth yardstick beside the stitched kernels and
// the calibration kernel for HBM byte counters.
#include "dev_common.h"
#include "launchers.h"

namespace fs {

__global__ __launch_bounds__(256) void stream_copy_kernel(u32x4* __restrict__ dst,
                                                          const u32x4* __restrict__ src, int64_t nvec) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  // four independent 16-byte loads in flight per lane
  for (; i + 3 * stride < nvec; i += 4 * stride) {
    const u32x4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
    dst[i] = a; dst[i + stride] = b; dst[i + 2 * stride] = c; dst[i + 3 * stride] = d;
  }
  for (; i < nvec; i += stride) dst[i] = src[i];
}

int stream_copy_launch(void* dst, const void* src, int64_t bytes, void* stream, std::string* err) {
  const int64_t nvec = bytes / 16;
  if (nvec == 0) return 0;
  int64_t grid = (nvec + 256 * 4 - 1) / (256 * 4);
  if (grid > 256 * 32) grid = 256 * 32;
  hipLaunchKernelGGL(stream_copy_kernel, dim3((unsigned)grid), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<u32x4*>(dst), static_cast<const u32x4*>(src), nvec);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) { *err = std::string("stream_copy launch: ") + hipGetErrorString(e); return -1; }
  return 0;
}

}  // namespace fs
