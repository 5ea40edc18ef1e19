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

// Second step of a column reduction whose first step left one double-precision partial row
// per workgroup: out[r][c] = sum over g of partial[r][g][c], summed in a fixed order (64
// interleaved slices, then the slices in order), stored in the output's dtype.
struct ColCombineArgs {
  void* out[8];
  int dtype[8];
  int is_max[8];     // the reduction is a maximum, not a sum
};

// NT threads: a block owns 16 columns of one run of rows (one 128-byte line of every partial row); its
// threads are NT / 16 slices of that run's partial rows.  256 threads for up to 512 partial rows (measured
// 0.8 us faster than 1024 on 256 partial rows of 2048 columns), 1024 beyond.
template <int NT>
__global__ __launch_bounds__(NT) void col_combine_kernel(const double* __restrict__ partial, int groups, int64_t total_groups,
                                                         int64_t cols, const ColCombineArgs args) {
  constexpr int NS = NT / 16;
  __shared__ double part[NS][17];
  const int64_t col_blocks = (cols + 15) / 16;
  const int64_t seg = blockIdx.x / col_blocks;
  const int r = blockIdx.y, j = threadIdx.x & 15, slice = threadIdx.x >> 4;
  const int64_t c = (blockIdx.x % col_blocks) * 16 + j;
  const bool is_max = args.is_max[r] != 0;
  double s = is_max ? -__builtin_inf() : 0.0;
  if (c < cols) {
    const double* p = partial + ((int64_t)r * total_groups + seg * groups) * cols + c;
    if (is_max) {
      for (int g = slice; g < groups; g += NS) s = fmax(s, p[(int64_t)g * cols]);
    } else {
      // eight partial rows requested at a time (the loads are independent, the additions keep their order)
      int g = slice;
      for (; g + 7 * NS < groups; g += 8 * NS) {
        double v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = p[(int64_t)(g + i * NS) * cols];
#pragma unroll
        for (int i = 0; i < 8; ++i) s += v[i];
      }
      for (; g < groups; g += NS) s += p[(int64_t)g * cols];
    }
  }
  part[slice][j] = s;
  __syncthreads();
  if (slice == 0 && c < cols) {
    double t = part[0][j];
    if (is_max) {
      for (int k = 1; k < NS; ++k) t = fmax(t, part[k][j]);
    } else {
#pragma unroll 8
      for (int k = 1; k < NS; ++k) t += part[k][j];
    }
    void* o = args.out[r];
    const float f = (float)t;
    const int64_t at = seg * cols + c;
    if (args.dtype[r] == DT_F32) static_cast<float*>(o)[at] = f;
    else static_cast<uint16_t*>(o)[at] = (uint16_t)(args.dtype[r] == DT_F16 ? f32_to_f16(f) : f32_to_bf16(f));
  }
}

// partial: [n_red][n_seg * groups][cols] doubles -- for every reduction and every run of rows, `groups`
// partial rows, added in a fixed order into out[r][n_seg][cols].  n_seg = 1: sums over all rows.
int col_combine_launch(const void* partial, int groups, int64_t cols, int n_red, void* const* out, const int* dtype,
                       void* stream, std::string* err, int64_t n_seg, const int* is_max) {
  if (n_red <= 0 || cols <= 0 || n_seg <= 0) return 0;
  const int64_t blocks = n_seg * ((cols + 15) / 16);
  if (blocks > 0x7fffffffLL) { *err = "col_combine launch: too many runs of rows for one grid"; return -1; }
  ColCombineArgs a{};
  for (int r = 0; r < n_red && r < 8; ++r) { a.out[r] = out[r]; a.dtype[r] = dtype[r]; a.is_max[r] = is_max ? is_max[r] : 0; }
  const dim3 grid((unsigned)blocks, (unsigned)n_red);
  if (groups <= 512)
    hipLaunchKernelGGL(col_combine_kernel<256>, grid, dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const double*>(partial), groups, n_seg * (int64_t)groups, cols, a);
  else
    hipLaunchKernelGGL(col_combine_kernel<1024>, grid, dim3(1024), 0, static_cast<hipStream_t>(stream),
                       static_cast<const double*>(partial), groups, n_seg * (int64_t)groups, cols, a);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) { *err = std::string("col_combine launch: ") + hipGetErrorString(e); return -1; }
  return 0;
}

}  // namespace fs
