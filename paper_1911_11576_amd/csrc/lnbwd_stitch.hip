// Schedules 1+2 packed (kernel packing + warp composition + block composition, paper
// Section 5.1): LayerNorm backward as one kernel.  The row path (dx: two row reductions,
// broadcast back through registers) and the column path (dgamma, dbeta: reductions over
// all rows) have no data dependence on each other but share their inputs, so they are
// packed over the same register-resident rows: dy and x are read from HBM exactly once.
//
// Row path: one wavefront per row, lane l owns 16-byte vectors l, l+64, ...; wave64
// all-reduce for sum(g) and sum(g*xhat).
// Column path: every lane accumulates its own columns over all rows its wavefront
// visits (fp64: 32768-term fp32 sums would not meet a 1e-5 absolute bar), the wavefronts
// of a workgroup combine through an LDS array (the `S` hand-off of block composition),
// each workgroup writes one partial row to a plan-owned HBM workspace, and the partials
// are summed in a fixed order by the workgroups that arrive last (two-level ticket tree).
// No floating-point atomics: the result is bit-reproducible.  No workgroup ever waits for
// another one.
#include "dev_common.h"
#include "launchers.h"

namespace fs {

struct LnBwdArgs {
  const float* dy; const float* x; const float* gamma; const float* mean; const float* rstd;
  float* dx; float* dgamma; float* dbeta;
  int64_t rows; int cols; int nvec; float inv_n;
  double* part0;      // [grid][2*cols]   one partial per workgroup
  double* part1;      // [n_groups][2*cols]
  unsigned* tickets;  // [1 + n_groups], zero between launches
  int group;          // workgroups per first-level group
  int n_groups;
};

template <int K, bool WANT_DX, bool WANT_COL>
__global__ __launch_bounds__(512) void lnbwd_stitch_kernel(const LnBwdArgs a) {
  extern __shared__ double lds[];   // [2*cols]: dgamma partials then dbeta partials
  __shared__ unsigned s_ticket;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, waves = blockDim.x >> 6;
  bool vld[K];
  int voff[K];
#pragma unroll
  for (int k = 0; k < K; ++k) {
    const int vi = k * 64 + lane;
    vld[k] = vi < a.nvec;
    voff[k] = (vld[k] ? vi : 0) * 4;
  }
  float gam[K][4];
  if constexpr (WANT_DX) {
#pragma unroll
    for (int k = 0; k < K; ++k) Vec<float>::load(a.gamma + voff[k], gam[k]);
  }
  double dg[K][4], db[K][4];
#pragma unroll
  for (int k = 0; k < K; ++k)
#pragma unroll
    for (int j = 0; j < 4; ++j) { dg[k][j] = 0.0; db[k][j] = 0.0; }

  const int64_t total_waves = (int64_t)gridDim.x * waves;
  for (int64_t row = (int64_t)blockIdx.x * waves + wave; row < a.rows; row += total_waves) {
    float dy[K][4], xv[K][4];
#pragma unroll
    for (int k = 0; k < K; ++k) {
      Vec<float>::load(a.dy + row * a.cols + voff[k], dy[k]);
      if (WANT_DX || a.x) Vec<float>::load(a.x + row * a.cols + voff[k], xv[k]);
    }
    float mu = 0.f, rs = 0.f;
    if (WANT_DX || a.x) { mu = a.mean[row]; rs = a.rstd[row]; }

    if constexpr (WANT_COL) {
      const double mu64 = (double)mu, rs64 = (double)rs;
#pragma unroll
      for (int k = 0; k < K; ++k)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const double d = vld[k] ? (double)dy[k][j] : 0.0;
          db[k][j] += d;
          if (a.x) dg[k][j] += d * (((double)xv[k][j] - mu64) * rs64);
        }
    }
    if constexpr (WANT_DX) {
      float s1 = 0.f, s2 = 0.f;
      float g[K][4];
#pragma unroll
      for (int k = 0; k < K; ++k)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          xv[k][j] = (xv[k][j] - mu) * rs;              // xhat
          g[k][j] = dy[k][j] * gam[k][j];
          s1 += vld[k] ? g[k][j] : 0.f;
          s2 += vld[k] ? g[k][j] * xv[k][j] : 0.f;
        }
      const float c1 = group_allreduce<SumOp, 64>(s1) * a.inv_n;
      const float c2 = group_allreduce<SumOp, 64>(s2) * a.inv_n;
#pragma unroll
      for (int k = 0; k < K; ++k) {
        float o[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) o[j] = ((g[k][j] - c1) - xv[k][j] * c2) * rs;
        if (vld[k]) Vec<float>::store(a.dx + row * a.cols + voff[k], o);
      }
    }
  }

  if constexpr (WANT_COL) {
    // ---- block composition: wavefronts take turns adding their columns into LDS ------
    for (int w = 0; w < waves; ++w) {
      if (wave == w) {
#pragma unroll
        for (int k = 0; k < K; ++k)
          if (vld[k]) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              const int c = voff[k] + j;
              lds[c] = (w == 0 ? 0.0 : lds[c]) + dg[k][j];
              lds[a.cols + c] = (w == 0 ? 0.0 : lds[a.cols + c]) + db[k][j];
            }
          }
      }
      __syncthreads();
    }
    const int n2 = 2 * a.cols;
    double* mine = a.part0 + (int64_t)blockIdx.x * n2;
    for (int c = threadIdx.x; c < n2; c += blockDim.x) mine[c] = lds[c];

    // ---- first-level ticket: the last workgroup of a group sums the group's partials --
    const int grp = blockIdx.x / a.group;
    const int first = grp * a.group;
    const int pop = min(a.group, (int)gridDim.x - first);
    __threadfence();
    __syncthreads();
    if (threadIdx.x == 0) s_ticket = atomicAdd(&a.tickets[1 + grp], 1u);
    __syncthreads();
    if (s_ticket != (unsigned)(pop - 1)) return;
    __threadfence();
    if (threadIdx.x == 0) a.tickets[1 + grp] = 0;
    double* gsum = a.part1 + (int64_t)grp * n2;
    for (int c = threadIdx.x; c < n2; c += blockDim.x) {
      double acc = 0.0;
      for (int b = 0; b < pop; ++b) acc += a.part0[(int64_t)(first + b) * n2 + c];
      gsum[c] = acc;
    }
    // ---- second-level ticket: the last group sums the group sums and writes the outputs
    __threadfence();
    __syncthreads();
    if (threadIdx.x == 0) s_ticket = atomicAdd(&a.tickets[0], 1u);
    __syncthreads();
    if (s_ticket != (unsigned)(a.n_groups - 1)) return;
    __threadfence();
    if (threadIdx.x == 0) a.tickets[0] = 0;
    for (int c = threadIdx.x; c < n2; c += blockDim.x) {
      double acc = 0.0;
      for (int q = 0; q < a.n_groups; ++q) acc += a.part1[(int64_t)q * n2 + c];
      if (c < a.cols) { if (a.dgamma) a.dgamma[c] = (float)acc; }
      else if (a.dbeta) a.dbeta[c - a.cols] = (float)acc;
    }
  }
}

namespace {

constexpr int kKs[] = {1, 2, 3, 4, 6, 8};

template <int K>
hipError_t launch_K(const LnBwdArgs& a, bool want_dx, bool want_col, int grid, int wg, size_t lds,
                    hipStream_t s) {
  if (want_dx && want_col)
    hipLaunchKernelGGL((lnbwd_stitch_kernel<K, true, true>), dim3(grid), dim3(wg), lds, s, a);
  else if (want_dx)
    hipLaunchKernelGGL((lnbwd_stitch_kernel<K, true, false>), dim3(grid), dim3(wg), 0, s, a);
  else
    hipLaunchKernelGGL((lnbwd_stitch_kernel<K, false, true>), dim3(grid), dim3(wg), lds, s, a);
  return hipGetLastError();
}

int64_t align256(int64_t v) { return (v + 255) / 256 * 256; }

}  // namespace

bool lnbwd_stitch_plan(const LnBwdSpec& sp, const LaunchOpts& opt, LnBwdLaunch* out, std::string* err) {
  if (sp.cols % 4 != 0) { *err = "LayerNorm-backward schedule: cols must be a multiple of 4"; return false; }
  if (sp.cols > 2048) { *err = "LayerNorm-backward schedule: cols > 2048 exceed one wavefront's register tile"; return false; }
  LnBwdLaunch l;
  const int need = (int)((sp.cols / 4 + 63) / 64);
  l.K = 8;
  for (int k : kKs) if (k >= need) { l.K = k; break; }
  l.wg = opt.wg_size ? opt.wg_size : 512;
  if (l.wg < 64 || l.wg > 512 || l.wg % 64) { *err = "LayerNorm-backward schedule: wg_size must be a multiple of 64 in [64,512]"; return false; }
  const int waves = l.wg / 64;
  int64_t grid = opt.grid > 0 ? opt.grid : 512;
  const int64_t max_useful = (sp.rows + waves - 1) / waves;
  if (grid > max_useful) grid = max_useful;
  if (grid < 1) grid = 1;
  if (grid > 65536) grid = 65536;
  l.grid = (int)grid;
  // two-level tree with groups of about sqrt(grid) workgroups
  int group = 1;
  while (group * group < l.grid) ++group;
  l.group = group;
  const bool want_col = sp.out_dgamma >= 0 || sp.out_dbeta >= 0;
  const int n_groups = (l.grid + l.group - 1) / l.group;
  l.lds_bytes = want_col ? 16 * sp.cols : 0;
  l.workspace_bytes = want_col ? align256(4 * (1 + n_groups)) + 16 * sp.cols * ((int64_t)l.grid + n_groups) : 0;
  *out = l;
  return true;
}

std::string lnbwd_stitch_describe(const LnBwdSpec& sp, const LnBwdLaunch& l) {
  char buf[512];
  snprintf(buf, sizeof buf,
           "reduce_s1[GRID-WARP,WARP]; reduce_s2[GRID-WARP,WARP]; dx[GRID-WARP,WARP-THREAD_%d]; "
           "reduce_dgamma[GRID-CTA-THREAD,WARP-THREAD_%d]S; reduce_dbeta[GRID-CTA-THREAD,WARP-THREAD_%d]S; "
           "cta_num=%d, cta_size=%d",
           l.K * 4, l.K * 4, l.K * 4, l.grid, l.wg);
  (void)sp;
  return buf;
}

int lnbwd_stitch_launch(const LnBwdSpec& sp, const LnBwdLaunch& l, const void* const* in, void* const* out,
                        void* workspace, void* stream, std::string* err) {
  if (sp.rows == 0 || sp.cols == 0) return 0;   // empty column sums are handled by the caller
  const bool want_dx = sp.out_dx >= 0;
  const bool want_col = sp.out_dgamma >= 0 || sp.out_dbeta >= 0;
  LnBwdArgs a{};
  a.dy = static_cast<const float*>(in[sp.in_dy]);
  a.x = sp.in_x >= 0 ? static_cast<const float*>(in[sp.in_x]) : nullptr;
  a.gamma = sp.in_gamma >= 0 ? static_cast<const float*>(in[sp.in_gamma]) : nullptr;
  a.mean = sp.in_mean >= 0 ? static_cast<const float*>(in[sp.in_mean]) : nullptr;
  a.rstd = sp.in_rstd >= 0 ? static_cast<const float*>(in[sp.in_rstd]) : nullptr;
  a.dx = want_dx ? static_cast<float*>(out[sp.out_dx]) : nullptr;
  a.dgamma = sp.out_dgamma >= 0 ? static_cast<float*>(out[sp.out_dgamma]) : nullptr;
  a.dbeta = sp.out_dbeta >= 0 ? static_cast<float*>(out[sp.out_dbeta]) : nullptr;
  a.rows = sp.rows; a.cols = (int)sp.cols; a.nvec = (int)(sp.cols / 4);
  a.inv_n = (float)(1.0 / (double)sp.cols);
  a.group = l.group;
  a.n_groups = (l.grid + l.group - 1) / l.group;
  if (want_col) {
    char* ws = static_cast<char*>(workspace);
    a.tickets = reinterpret_cast<unsigned*>(ws);
    a.part0 = reinterpret_cast<double*>(ws + align256(4 * (1 + a.n_groups)));
    a.part1 = a.part0 + (int64_t)l.grid * 2 * sp.cols;
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e;
  const size_t lds = (size_t)l.lds_bytes;
  switch (l.K) {
    case 1: e = launch_K<1>(a, want_dx, want_col, l.grid, l.wg, lds, s); break;
    case 2: e = launch_K<2>(a, want_dx, want_col, l.grid, l.wg, lds, s); break;
    case 3: e = launch_K<3>(a, want_dx, want_col, l.grid, l.wg, lds, s); break;
    case 4: e = launch_K<4>(a, want_dx, want_col, l.grid, l.wg, lds, s); break;
    case 6: e = launch_K<6>(a, want_dx, want_col, l.grid, l.wg, lds, s); break;
    default: e = launch_K<8>(a, want_dx, want_col, l.grid, l.wg, lds, s); break;
  }
  if (e != hipSuccess) { *err = std::string("lnbwd_stitch launch: ") + hipGetErrorString(e); return -1; }
  return 0;
}

}  // namespace fs
