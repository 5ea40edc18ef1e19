// Schedules 1+2 packed (kernel packing + warp composition + block composition, paper
// Section 5.1): LayerNorm backward as one kernel.  The row path (dx: two row reductions,
// broadcast back through registers) and the column path (dgamma, dbeta: reductions over
// all rows) have no data dependence on each other but share their inputs, so they are
// packed over the same register-resident rows: dy and x are read from HBM exactly once.
//
// Row path: one wavefront per row, lane l owns 16-byte vectors l, l+64, ...; wave64
// all-reduce for sum(g) and sum(g*xhat).  A wavefront's next row is loaded while the
// current one is processed (register double buffering).
// Column path: every lane accumulates its own columns over all rows its wavefront
// visits, in fp64 (32768-term fp32 sums would not meet a 1e-5 absolute bar), in a
// wavefront-private LDS array (ds_add_f64; 32 accumulators per lane would otherwise take
// 64 VGPRs).  The wavefronts of a workgroup then combine their arrays by a binary tree in
// LDS (the `S` hand-off of block composition), each workgroup writes one partial row to
// a plan-owned HBM workspace, and the partials are summed in a fixed order by the
// workgroups that arrive last (two-level ticket tree).  No floating-point atomics on
// shared data: the result is bit-reproducible.  No workgroup ever waits for another one.
//
// Accumulator slot layout (LDS and workspace): slot (k*4+j)*64 + lane holds column
// (k*64+lane)*4 + j, so that the 64 lanes of one LDS instruction touch 64 consecutive
// doubles (no bank conflicts).  Only the final store maps slots back to columns.
//
// Cross-workgroup hand-off without a device-wide fence: a release fence at agent scope
// writes back the whole L2 of the XCD, which in a kernel that is streaming hundreds of
// megabytes of dx through that L2 costs far more than the reduction itself.  Instead the
// partials are written and read with agent-scope atomic stores/loads (coherent across
// the XCDs' L2s by themselves), every thread waits for its own stores to complete, the
// workgroup barriers, and only then one thread takes the ticket.
#include <mutex>
#include <set>

#include "dev_common.h"
#include "launchers.h"

namespace fs {

// LDS a workgroup of this schedule may use: one workgroup per CU by design, so nearly all
// of the CU's 160 KB (the volume constraint of shared-memory planning for this schedule)
static constexpr int64_t kLdsMax = 160 * 1024 - 1024;

struct LnBwdArgs {
  const float* dy; const float* x; const float* gamma; const float* mean; const float* rstd;
  float* dx; float* dgamma; float* dbeta;
  int64_t rows; int cols; int nvec; float inv_n;
  double* part0;      // [grid][2*K*256]   one partial (slot layout) per workgroup
  double* part1;      // [n_groups][2*K*256]
  unsigned* tickets;  // [1 + n_groups], zero between launches
  int group;          // workgroups per first-level group
  int n_groups;
};

// Register budget of the kernel: asking for 4 wavefronts per SIMD caps it at 128 VGPRs.
#ifndef FS_LNBWD_MIN_WAVES
#define FS_LNBWD_MIN_WAVES 0
#endif
#if FS_LNBWD_MIN_WAVES > 0
#define FS_LNBWD_OCCUPANCY __attribute__((amdgpu_waves_per_eu(FS_LNBWD_MIN_WAVES, 8)))
#else
#define FS_LNBWD_OCCUPANCY
#endif

__device__ __forceinline__ void coherent_store(double* p, double v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ double coherent_load(const double* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// all of this thread's earlier stores have completed at their coherence scope
__device__ __forceinline__ void wait_for_own_stores() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __builtin_amdgcn_s_waitcnt(0);
}

// Sum `count` consecutive partial rows of n2 doubles, in ascending row order.  A thread
// owns four columns at a time and issues the loads of up to 16 partials of all four before
// it uses any of them (64 independent loads in flight), so a finishing workgroup of 512
// threads pays about one memory latency for 16 partials of 2048 columns instead of one
// per load.
template <class Sink>
__device__ __forceinline__ void sum_partials(const double* __restrict__ src, int count, int n2, Sink sink) {
  constexpr int Q = 4, D = 16;
  const int nt = blockDim.x;
  for (int c0 = threadIdx.x; c0 < n2; c0 += Q * nt) {
    double acc[Q];
#pragma unroll
    for (int q = 0; q < Q; ++q) acc[q] = 0.0;
    for (int b0 = 0; b0 < count; b0 += D) {
      double v[Q][D];
#pragma unroll
      for (int q = 0; q < Q; ++q)
#pragma unroll
        for (int j = 0; j < D; ++j) {
          const int c = c0 + q * nt, b = b0 + j;
          v[q][j] = (c < n2 && b < count) ? coherent_load(src + (int64_t)b * n2 + c) : 0.0;
        }
#pragma unroll
      for (int q = 0; q < Q; ++q)
#pragma unroll
        for (int j = 0; j < D; ++j) acc[q] += v[q][j];
    }
#pragma unroll
    for (int q = 0; q < Q; ++q)
      if (c0 + q * nt < n2) sink(c0 + q * nt, acc[q]);
  }
}

// COL: 0 no column outputs, 1 dbeta only (x is not needed), 2 dgamma and dbeta
// EXACT: cols == K*256, no per-vector masking
template <int K, bool WANT_DX, int COL, bool EXACT>
__global__ __launch_bounds__(512) FS_LNBWD_OCCUPANCY
void lnbwd_stitch_kernel(const LnBwdArgs a) {
  extern __shared__ double lds[];   // [waves][2][K*256] accumulator slots
  __shared__ unsigned s_ticket;
  constexpr bool WANT_COL = COL != 0, NEED_X = WANT_DX || COL == 2;
  constexpr int SLOTS = K * 256;    // per quantity
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, waves = blockDim.x >> 6;
  bool vld[K];
  int voff[K];
#pragma unroll
  for (int k = 0; k < K; ++k) {
    const int vi = k * 64 + lane;
    vld[k] = EXACT || vi < a.nvec;
    voff[k] = (vld[k] ? vi : 0) * 4;
  }
  float gam[K][4];
  double* acc = lds + (int64_t)wave * 2 * SLOTS + lane;   // + (k*4+j)*64 (+ SLOTS for dbeta)
#pragma unroll
  for (int k = 0; k < K; ++k) {
    if constexpr (WANT_DX) Vec<float>::load(a.gamma + voff[k], gam[k]);
    if constexpr (WANT_COL) {
#pragma unroll
      for (int j = 0; j < 4; ++j) { acc[(k * 4 + j) * 64] = 0.0; acc[SLOTS + (k * 4 + j) * 64] = 0.0; }
    }
  }

  // All workgroups advance through the rows together (row = step*grid*waves + wg*waves +
  // wave), so at any moment the chip streams one compact window of dy, x and dx, as a
  // one-shot grid would; giving each workgroup its own contiguous block of rows instead
  // measured about 8% slower.
  const int64_t row_end = a.rows;
  const int64_t row_step = (int64_t)gridDim.x * waves;
  int64_t row = (int64_t)blockIdx.x * waves + wave;
  u32x4 dyn[K], xn[K];
  float mun = 0.f, rsn = 0.f;
  if (row < row_end) {
#pragma unroll
    for (int k = 0; k < K; ++k) {
      dyn[k] = stream_load16(a.dy + row * a.cols + voff[k]);
      if constexpr (NEED_X) xn[k] = stream_load16(a.x + row * a.cols + voff[k]);
    }
    if constexpr (NEED_X) { mun = a.mean[row]; rsn = a.rstd[row]; }
  }
  for (; row < row_end; row += row_step) {
    float dy[K][4], xv[K][4];
#pragma unroll
    for (int k = 0; k < K; ++k) {
      Vec<float>::unpack(dyn[k], dy[k]);
      if constexpr (NEED_X) Vec<float>::unpack(xn[k], xv[k]);
    }
    const float mu = mun, rs = rsn;
    // prefetch the next row: issued unconditionally and pinned ahead of the arithmetic (the
    // last iteration reads row 0, which every wavefront does at that point: an L2 hit, no
    // extra HBM traffic)
    const int64_t nrow = row + row_step < row_end ? row + row_step : 0;
#pragma unroll
    for (int k = 0; k < K; ++k) {
      dyn[k] = stream_load16(a.dy + nrow * a.cols + voff[k]);
      if constexpr (NEED_X) xn[k] = stream_load16(a.x + nrow * a.cols + voff[k]);
    }
    if constexpr (NEED_X) { mun = a.mean[nrow]; rsn = a.rstd[nrow]; }
    __builtin_amdgcn_sched_barrier(0);

    if constexpr (WANT_COL) {
      const double mu64 = (double)mu, rs64 = (double)rs;
#pragma unroll
      for (int k = 0; k < K; ++k)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const double d = vld[k] ? (double)dy[k][j] : 0.0;
          __hip_atomic_fetch_add(acc + SLOTS + (k * 4 + j) * 64, d, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
          if constexpr (COL == 2)
            __hip_atomic_fetch_add(acc + (k * 4 + j) * 64, d * (((double)xv[k][j] - mu64) * rs64), __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_WAVEFRONT);
        }
    }
    if constexpr (WANT_DX) {
      float s1 = 0.f, s2 = 0.f;
      float g[K][4];
#pragma unroll
      for (int k = 0; k < K; ++k) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          xv[k][j] = (xv[k][j] - mu) * rs;              // xhat
          g[k][j] = dy[k][j] * gam[k][j];
          s1 += vld[k] ? g[k][j] : 0.f;
          s2 += vld[k] ? g[k][j] * xv[k][j] : 0.f;
        }
      }
      const float c1 = group_allreduce<SumOp, 64>(s1) * a.inv_n;
      const float c2 = group_allreduce<SumOp, 64>(s2) * a.inv_n;
#pragma unroll
      for (int k = 0; k < K; ++k) {
        float o[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) o[j] = ((g[k][j] - c1) - xv[k][j] * c2) * rs;
        if (vld[k]) stream_store16(a.dx + row * a.cols + voff[k], pack16<float>(o));
      }
    }
  }

  if constexpr (WANT_COL) {
    // ---- block composition: binary tree over the wavefronts' LDS arrays, in place -----------
    constexpr int n2 = 2 * SLOTS;
    int P = 1;
    while (P < waves) P <<= 1;
    int wcur = waves;
    for (int s = P >> 1; s >= 1; s >>= 1) {
      __syncthreads();
      if (wave < s && wave + s < wcur) {
        const double* other = acc + (int64_t)s * n2;
#pragma unroll
        for (int q = 0; q < 2 * K * 4; ++q) acc[q * 64] += other[q * 64];
      }
      wcur = min(wcur, s);
    }
    __syncthreads();
    double* mine = a.part0 + (int64_t)blockIdx.x * n2;
    for (int c = threadIdx.x; c < n2; c += blockDim.x) coherent_store(mine + c, lds[c]);

    // ---- first-level ticket: the last workgroup of a group sums the group's partials --
    const int grp = blockIdx.x / a.group;
    const int first = grp * a.group;
    const int pop = min(a.group, (int)gridDim.x - first);
    wait_for_own_stores();
    __syncthreads();
    if (threadIdx.x == 0) s_ticket = atomicAdd(&a.tickets[1 + grp], 1u);
    __syncthreads();
    if (s_ticket != (unsigned)(pop - 1)) return;
    if (threadIdx.x == 0) __hip_atomic_store(&a.tickets[1 + grp], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    double* gsum = a.part1 + (int64_t)grp * n2;
    sum_partials(a.part0 + (int64_t)first * n2, pop, n2, [&](int c, double v) { coherent_store(gsum + c, v); });
    // ---- second-level ticket: the last group sums the group sums and writes the outputs
    wait_for_own_stores();
    __syncthreads();
    if (threadIdx.x == 0) s_ticket = atomicAdd(&a.tickets[0], 1u);
    __syncthreads();
    if (s_ticket != (unsigned)(a.n_groups - 1)) return;
    if (threadIdx.x == 0) __hip_atomic_store(&a.tickets[0], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    sum_partials(a.part1, a.n_groups, n2, [&](int c, double v) {
      // slot -> column
      const int r = c % SLOTS, kj = r >> 6, vi = (kj >> 2) * 64 + (r & 63);
      const int col = vi * 4 + (kj & 3);
      if (vi < a.nvec) {
        if (c < SLOTS) { if (a.dgamma) a.dgamma[col] = (float)v; }
        else if (a.dbeta) a.dbeta[col] = (float)v;
      }
    });
  }
}

namespace {

constexpr int kKs[] = {1, 2, 3, 4};

// more than 64 KB of dynamic LDS has to be enabled once per kernel
template <typename Kern>
hipError_t launch_with_lds(Kern kern, const LnBwdArgs& a, int grid, int wg, size_t lds, hipStream_t s) {
  if (lds > 64 * 1024) {
    static std::mutex mu;
    static std::set<const void*> raised;
    std::lock_guard<std::mutex> lock(mu);
    const void* f = reinterpret_cast<const void*>(kern);
    if (!raised.count(f)) {
      const hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsMax);
      if (e != hipSuccess) return e;
      raised.insert(f);
    }
  }
  hipLaunchKernelGGL(kern, dim3(grid), dim3(wg), lds, s, a);
  return hipGetLastError();
}

template <int K, bool EXACT>
hipError_t launch_KE(const LnBwdArgs& a, bool want_dx, bool want_col, int grid, int wg, size_t lds,
                     hipStream_t s) {
  const bool need_x_cols = a.dgamma != nullptr;
  if (want_dx && want_col)   // with dx the row is loaded anyway: always the full column path
    return launch_with_lds(lnbwd_stitch_kernel<K, true, 2, EXACT>, a, grid, wg, lds, s);
  if (want_dx) return launch_with_lds(lnbwd_stitch_kernel<K, true, 0, EXACT>, a, grid, wg, 0, s);
  if (need_x_cols) return launch_with_lds(lnbwd_stitch_kernel<K, false, 2, EXACT>, a, grid, wg, lds, s);
  return launch_with_lds(lnbwd_stitch_kernel<K, false, 1, EXACT>, a, grid, wg, lds, s);
}

template <int K>
hipError_t launch_K(const LnBwdArgs& a, bool want_dx, bool want_col, int grid, int wg, size_t lds,
                    hipStream_t s) {
  if (a.nvec == K * 64) return launch_KE<K, true>(a, want_dx, want_col, grid, wg, lds, s);
  return launch_KE<K, false>(a, want_dx, want_col, grid, wg, lds, s);
}

int64_t align256(int64_t v) { return (v + 255) / 256 * 256; }

}  // namespace

bool lnbwd_stitch_plan(const LnBwdSpec& sp, const LaunchOpts& opt, LnBwdLaunch* out, std::string* err) {
  if (sp.cols % 4 != 0) { *err = "LayerNorm-backward schedule: cols must be a multiple of 4"; return false; }
  // a lane holds its columns' fp64 accumulators: 4 vectors of 4 columns is what fits
  if (sp.cols > 1024) { *err = "LayerNorm-backward schedule: cols > 1024 exceed one wavefront's register tile"; return false; }
  LnBwdLaunch l;
  const int need = (int)((sp.cols / 4 + 63) / 64);
  l.K = 4;
  for (int k : kKs) if (k >= need) { l.K = k; break; }
  // 8 wavefronts per workgroup and one workgroup per CU: two wavefronts per SIMD is what
  // the kernel's register budget allows (fp64 column accumulators plus a double-buffered
  // row), and fewer, larger workgroups mean fewer partials
  l.wg = opt.wg_size ? opt.wg_size : 512;
  if (l.wg < 64 || l.wg > 512 || l.wg % 64) { *err = "LayerNorm-backward schedule: wg_size must be a multiple of 64 in [64,512]"; return false; }
  const int waves = l.wg / 64;
  int64_t grid = opt.grid > 0 ? opt.grid : 256;
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
  l.lds_bytes = want_col ? (int64_t)waves * 2 * l.K * 256 * 8 : 0;
  if (l.lds_bytes > kLdsMax) {
    *err = "LayerNorm-backward schedule: wg_size needs more LDS for the column accumulators than a CU has";
    return false;
  }
  l.workspace_bytes = want_col ? align256(4 * (1 + n_groups)) + (int64_t)16 * l.K * 256 * ((int64_t)l.grid + n_groups) : 0;
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
  if (sp.cols == 0) return 0;
  if (sp.rows == 0) {
    // sums over zero rows are zero: the combine kernel over zero partial rows writes them
    void* col_out[2];
    int dtype[2] = {DT_F32, DT_F32}, n = 0;
    if (sp.out_dgamma >= 0) col_out[n++] = out[sp.out_dgamma];
    if (sp.out_dbeta >= 0) col_out[n++] = out[sp.out_dbeta];
    return col_combine_launch(nullptr, 0, sp.cols, n, col_out, dtype, stream, err);
  }
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
    a.part1 = a.part0 + (int64_t)l.grid * 2 * l.K * 256;
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e;
  const size_t lds = (size_t)l.lds_bytes;
  switch (l.K) {
    case 1: e = launch_K<1>(a, want_dx, want_col, l.grid, l.wg, lds, s); break;
    case 2: e = launch_K<2>(a, want_dx, want_col, l.grid, l.wg, lds, s); break;
    case 3: e = launch_K<3>(a, want_dx, want_col, l.grid, l.wg, lds, s); break;
    default: e = launch_K<4>(a, want_dx, want_col, l.grid, l.wg, lds, s); break;
  }
  if (e != hipSuccess) { *err = std::string("lnbwd_stitch launch: ") + hipGetErrorString(e); return -1; }
  return 0;
}

}  // namespace fs
