// Schedules 1+2 packed (kernel packing + warp composition + block composition, paper
// Section 5.1): LayerNorm backward, hand-written.  The row path (dx: two row reductions,
// broadcast back through registers) and the column path (dgamma, dbeta: reductions over
// all rows, which Section 4.2 lists among the ops with parallelisation needs of their own)
// have no data dependence on each other but share their inputs, so they are packed over the
// same register-resident rows: dy and x are read from HBM exactly once.
//
// Row path: a fixed grid of workgroups walks the rows together (row = step * grid * waves +
// workgroup * waves + wave), one wavefront per row, lane l owns 16-byte vectors l, l+64, ...;
// wave64 all-reduce for sum(g) and sum(g*xhat).  A wavefront requests its rows two steps
// ahead into three register buffers that take turns (none is ever copied): with one wavefront
// per SIMD the time of a step is otherwise the latency of its loads.
// Column path: every lane keeps double-precision running sums for its own columns over all
// rows its wavefront visits (32768-term fp32 sums would not meet a 1e-5 absolute bar).  At
// the end each wavefront writes its sums to an LDS array of its own (the `S` hand-off of
// block composition), the workgroup adds the arrays in wavefront order and writes ONE partial
// row to a plan-owned workspace; a second, small kernel adds the partial rows in a fixed
// order.  No atomics, no tickets, no waiting between workgroups: the hand-off between the two
// kernels is the stream order, and the result is bit-reproducible.
//
// Slot layout (LDS and workspace): slot q*64 + lane with q = r*4K + k*4 + j holds column
// (k*64+lane)*4 + j of reduction r (0 dbeta, 1 dgamma), so that the 64 lanes of one LDS
// instruction touch 64 consecutive doubles (no bank conflicts).  Only the final store of the
// combine kernel maps slots back to columns.
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
  double* part;       // [grid][2*K*256]   one partial row (slot layout) per workgroup
};

// COL: 0 no column outputs, 1 dbeta only (x is not needed), 2 dgamma and dbeta
// EXACT: cols == K*256, no per-vector masking
// PF: row steps requested ahead of the one being worked on
// MAXWG: largest workgroup the instance is launched with (256: one wavefront per SIMD may use the
// whole register file; 512: two share it)
template <int K, bool WANT_DX, int COL, bool EXACT, int PF, int MAXWG>
__global__ __launch_bounds__(MAXWG)
void lnbwd_rows_kernel(const LnBwdArgs a) {
  extern __shared__ double lds[];   // [waves][2*K*256] slots
  constexpr bool WANT_COL = COL != 0, NEED_X = WANT_DX || COL == 2;
  constexpr int SLOTS = K * 256;    // per reduction
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
  double dg[K][4], db[K][4];
#pragma unroll
  for (int k = 0; k < K; ++k) {
    if constexpr (WANT_DX) Vec<float>::load(a.gamma + voff[k], gam[k]);
#pragma unroll
    for (int j = 0; j < 4; ++j) { dg[k][j] = 0.0; db[k][j] = 0.0; }
  }

  asm volatile("" ::: "memory");   // gamma is requested before the rows (the wait below the row requests counts on it)

  // All workgroups advance through the rows together, so at any moment the chip streams one
  // compact window of dy, x and dx, as a one-shot grid would.
  const int64_t row_end = a.rows;
  const int64_t row_step = (int64_t)gridDim.x * waves;
  int64_t row = (int64_t)blockIdx.x * waves + wave;
  // PF + 1 row buffers that take turns: the loop is unrolled PF + 1 times, step p works on buffer p and
  // first requests the row PF steps ahead into the buffer the step before it has finished with.  No buffer is
  // ever copied (a copy of a buffer that was requested only one step ago would wait for it, which is what
  // shifting the buffers down costs), and every request has PF whole steps to arrive.
  constexpr int NB = PF + 1;
  u32x4 rdy[NB][K], rx[NB][K];
  float rmu[NB], rrs[NB];
  auto request = [&](int b, int64_t want) {
    // past the end: row 0, which is in cache by then (no extra HBM traffic); its values are never used
    const int64_t r = want < row_end ? want : 0;
    // (loads complete in the order they are issued: the row's mean and rstd, needed first, go first)
    if constexpr (NEED_X) { rmu[b] = a.mean[r]; rrs[b] = a.rstd[r]; }
#pragma unroll
    for (int k = 0; k < K; ++k) {
      rdy[b][k] = stream_load16(a.dy + r * a.cols + voff[k]);
      if constexpr (NEED_X) rx[b][k] = stream_load16(a.x + r * a.cols + voff[k]);
    }
  };
#pragma unroll
  for (int p = 0; p < PF; ++p) request(p, row + p * row_step);
  // gamma has arrived before the row loop starts: a load still pending at its top would put a wait into the
  // loop that, trip after trip, also waits for the rows requested ahead.  Loads complete in the order they
  // were issued, gamma's first: the wait lets the row requests just issued stay in flight (vmcnt = their
  // number; bits 3:0 and 15:14 of the operand, the other counters left alone).
  constexpr int kRowLoads = PF * (K + (NEED_X ? K + 2 : 0));
  static_assert(kRowLoads < 64, "the wait counter has six bits");
  __builtin_amdgcn_s_waitcnt((kRowLoads & 15) | ((kRowLoads >> 4) << 14) | 0x0F70);
  // one step: request the row PF steps ahead, then the arithmetic of row r out of buffer p
  auto step = [&](const int p, const int64_t r) {
    request((p + PF) % NB, r + PF * row_step);
    __builtin_amdgcn_sched_barrier(0);                    // the requests stay ahead of the arithmetic
    float dy[K][4], xv[K][4];
#pragma unroll
    for (int k = 0; k < K; ++k) {
      Vec<float>::unpack(rdy[p][k], dy[k]);
      if constexpr (NEED_X) Vec<float>::unpack(rx[p][k], xv[k]);
    }
    const float rs = NEED_X ? rrs[p] : 0.f, nmurs = NEED_X ? -rmu[p] * rs : 0.f;
    float s1 = 0.f, s2 = 0.f;
    constexpr bool KEEP_G = K * (PF + 1) < 12;
    float g[KEEP_G ? K : 1][4];
#pragma unroll
    for (int k = 0; k < K; ++k) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float d = vld[k] ? dy[k][j] : 0.f;
        if constexpr (NEED_X) xv[k][j] = fmaf(xv[k][j], rs, nmurs);      // xhat = (x - mu) * rs
        if constexpr (WANT_COL) db[k][j] += (double)d;
        if constexpr (COL == 2) dg[k][j] += (double)(d * xv[k][j]);
        if constexpr (WANT_DX) {
          const float gj = d * gam[k][j];
          if constexpr (KEEP_G) g[k][j] = gj;
          s1 += gj;
          s2 = fmaf(gj, xv[k][j], s2);
        }
      }
    }
    if constexpr (WANT_DX) {
      // dx = (g - c1 - xhat c2) rs, as two fused multiply-adds per element
      const float nc1 = -(group_allreduce<SumOp, 64>(s1) * a.inv_n) * rs;
      const float nc2 = -(group_allreduce<SumOp, 64>(s2) * a.inv_n) * rs;
#pragma unroll
      for (int k = 0; k < K; ++k) {
        float o[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          // (with four vectors per lane dy * gamma is multiplied out again rather than kept: sixteen registers
          // fewer is what keeps three row buffers, the fp64 sums and gamma inside the 256 vector registers)
          const float gj = KEEP_G ? g[k][j] : (vld[k] ? dy[k][j] : 0.f) * gam[k][j];
          o[j] = fmaf(xv[k][j], nc2, fmaf(gj, rs, nc1));
        }
        if (vld[k]) stream_store16(a.dx + r * a.cols + voff[k], pack16<float>(o));
      }
    }
  };
  // whole trips of PF + 1 steps without a branch inside (one path through the loop: the waits on the
  // requests count exactly), then the last, partial trip
  for (; row + PF * row_step < row_end; row += NB * row_step) {
#pragma unroll
    for (int p = 0; p < NB; ++p) step(p, row + p * row_step);
  }
#pragma unroll
  for (int p = 0; p < NB; ++p)
    if (row + p * row_step < row_end) step(p, row + p * row_step);

  if constexpr (WANT_COL) {
    // ---- block composition: every wavefront's sums into its own LDS array, then the arrays
    // added in wavefront order by all threads, two slots each, straight into the partial row
    constexpr int n2 = 2 * SLOTS;
    double* mine = lds + (int64_t)wave * n2 + lane;
#pragma unroll
    for (int k = 0; k < K; ++k)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        mine[(k * 4 + j) * 64] = db[k][j];
        mine[SLOTS + (k * 4 + j) * 64] = dg[k][j];
      }
    __syncthreads();
    typedef double f64x2 __attribute__((ext_vector_type(2)));
    double* out = a.part + (int64_t)blockIdx.x * n2;
    for (int s = threadIdx.x * 2; s < n2; s += blockDim.x * 2) {
      f64x2 t = *reinterpret_cast<const f64x2*>(lds + s);
      for (int w = 1; w < waves; ++w) t += *reinterpret_cast<const f64x2*>(lds + (int64_t)w * n2 + s);
      *reinterpret_cast<f64x2*>(out + s) = t;
    }
  }
}

// Second kernel of the plan: out[col(slot)] = sum over the workgroups' partial rows, in a fixed order
// (256 / SL interleaved slices of partial rows, then the slices in order).  A block owns SL consecutive slots:
// with 16 the 16 lanes of a slice read one whole 128-byte line of a partial row.
template <int SL, int NT = 256, int NL = 8>
__global__ __launch_bounds__(NT)
void lnbwd_combine_kernel(const double* __restrict__ part, int groups, int K, int nvec, float* dgamma, float* dbeta) {
  constexpr int NS = NT / SL;           // slices
  __shared__ double stage[NS][SL + 1];
  const int n2 = 2 * K * 256;
  const int j = threadIdx.x % SL, slice = threadIdx.x / SL;
  const int s = blockIdx.x * SL + j;
  const double* p = part + s;
  double acc = 0.0;
  int g = slice;
  // NL partial rows requested at a time (the loads are independent, the additions keep their order)
  for (; g + (NL - 1) * NS < groups; g += NL * NS) {
    double v[NL];
#pragma unroll
    for (int i = 0; i < NL; ++i) v[i] = p[(int64_t)(g + i * NS) * n2];
#pragma unroll
    for (int i = 0; i < NL; ++i) acc += v[i];
  }
  for (; g < groups; g += NS) acc += p[(int64_t)g * n2];
  stage[slice][j] = acc;
  __syncthreads();
  if (slice == 0) {
    double t = stage[0][j];
#pragma unroll
    for (int k = 1; k < NS; ++k) t += stage[k][j];
    // slot -> column
    const int slots = K * 256;
    const int r = s >= slots ? 1 : 0, q = (s - r * slots) >> 6, vi = (q >> 2) * 64 + (s & 63);
    const int col = vi * 4 + (q & 3);
    float* o = r ? dgamma : dbeta;
    if (vi < nvec && o) o[col] = (float)t;
  }
}
constexpr int kCombineSlots = 16;

namespace {

constexpr int kKs[] = {1, 2, 3, 4};
constexpr int kPrefetch = 2;

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

template <int K, bool EXACT, int MAXWG>
hipError_t launch_KEW(const LnBwdArgs& a, bool want_dx, bool want_col, int grid, int wg, size_t lds,
                      hipStream_t s) {
  const bool need_x_cols = a.dgamma != nullptr;
  if (want_dx && want_col)   // with dx the row is loaded anyway: always the full column path
    return launch_with_lds(lnbwd_rows_kernel<K, true, 2, EXACT, kPrefetch, MAXWG>, a, grid, wg, lds, s);
  if (want_dx) return launch_with_lds(lnbwd_rows_kernel<K, true, 0, EXACT, kPrefetch, MAXWG>, a, grid, wg, 0, s);
  if (need_x_cols) return launch_with_lds(lnbwd_rows_kernel<K, false, 2, EXACT, kPrefetch, MAXWG>, a, grid, wg, lds, s);
  return launch_with_lds(lnbwd_rows_kernel<K, false, 1, EXACT, kPrefetch, MAXWG>, a, grid, wg, lds, s);
}

template <int K>
hipError_t launch_K(const LnBwdArgs& a, bool want_dx, bool want_col, int grid, int wg, size_t lds,
                    hipStream_t s) {
  const bool exact = a.nvec == K * 64;
  if (wg <= 256) return exact ? launch_KEW<K, true, 256>(a, want_dx, want_col, grid, wg, lds, s)
                              : launch_KEW<K, false, 256>(a, want_dx, want_col, grid, wg, lds, s);
  return exact ? launch_KEW<K, true, 512>(a, want_dx, want_col, grid, wg, lds, s)
               : launch_KEW<K, false, 512>(a, want_dx, want_col, grid, wg, lds, s);
}

}  // namespace

bool lnbwd_stitch_plan(const LnBwdSpec& sp, const LaunchOpts& opt, LnBwdLaunch* out, std::string* err) {
  if (sp.cols % 4 != 0) { *err = "LayerNorm-backward schedule: cols must be a multiple of 4"; return false; }
  // a lane holds its columns' fp64 running sums: 4 vectors of 4 columns is what fits
  if (sp.cols > 1024) { *err = "LayerNorm-backward schedule: cols > 1024 exceed one wavefront's register tile"; return false; }
  LnBwdLaunch l;
  const int need = (int)((sp.cols / 4 + 63) / 64);
  l.K = 4;
  for (int k : kKs) if (k >= need) { l.K = k; break; }
  // 4 wavefronts per workgroup and one workgroup per CU: one wavefront per SIMD has the whole
  // register file for its running sums and three row buffers; more wavefronts measured slower
  l.wg = opt.wg_size ? opt.wg_size : 256;
  if (l.wg < 64 || l.wg > 512 || l.wg % 64) { *err = "LayerNorm-backward schedule: wg_size must be a multiple of 64 in [64,512]"; return false; }
  const int waves = l.wg / 64;
  int64_t grid = opt.grid > 0 ? opt.grid : 256;
  const int64_t max_useful = (sp.rows + waves - 1) / waves;
  if (grid > max_useful) grid = max_useful;
  if (grid < 1) grid = 1;
  if (grid > 4096) grid = 4096;
  l.grid = (int)grid;
  const bool want_col = sp.out_dgamma >= 0 || sp.out_dbeta >= 0;
  l.n_kernels = want_col ? 2 : 1;
  l.lds_bytes = want_col ? (int64_t)waves * 2 * l.K * 256 * 8 : 0;
  if (l.lds_bytes > kLdsMax) {
    *err = "LayerNorm-backward schedule: wg_size needs more LDS for the column sums than a CU has";
    return false;
  }
  l.workspace_bytes = want_col ? (int64_t)16 * l.K * 256 * (int64_t)l.grid : 0;
  *out = l;
  return true;
}

std::string lnbwd_stitch_describe(const LnBwdSpec& sp, const LnBwdLaunch& l) {
  char buf[512];
  snprintf(buf, sizeof buf,
           "reduce_s1[GRID-WARP,WARP]; reduce_s2[GRID-WARP,WARP]; dx[GRID-WARP,WARP-THREAD_%d]; "
           "reduce_dgamma[GRID-CTA-THREAD,WARP-THREAD_%d]S; reduce_dbeta[GRID-CTA-THREAD,WARP-THREAD_%d]S "
           "(hand-written kernel; %d partial rows, then a combine kernel); cta_num=%d, cta_size=%d",
           l.K * 4, l.K * 4, l.K * 4, l.grid, l.grid, l.wg);
  (void)sp;
  return buf;
}

int lnbwd_stitch_launch(const LnBwdSpec& sp, const LnBwdLaunch& l, const void* const* in, void* const* out,
                        void* workspace, void* stream, std::string* err) {
  if (sp.cols == 0) return 0;
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
  a.part = static_cast<double*>(workspace);
  hipStream_t s = static_cast<hipStream_t>(stream);
  int groups = 0;
  if (sp.rows > 0) {
    if (want_col && !workspace) { *err = "lnbwd_stitch launch: no workspace"; return -1; }
    hipError_t e;
    const size_t lds = (size_t)l.lds_bytes;
    switch (l.K) {
      case 1: e = launch_K<1>(a, want_dx, want_col, l.grid, l.wg, lds, s); break;
      case 2: e = launch_K<2>(a, want_dx, want_col, l.grid, l.wg, lds, s); break;
      case 3: e = launch_K<3>(a, want_dx, want_col, l.grid, l.wg, lds, s); break;
      default: e = launch_K<4>(a, want_dx, want_col, l.grid, l.wg, lds, s); break;
    }
    if (e != hipSuccess) { *err = std::string("lnbwd_stitch launch: ") + hipGetErrorString(e); return -1; }
    groups = l.grid;
  }
  if (want_col) {
    // sums over zero rows are zero: the combine kernel over zero partial rows writes them
    hipLaunchKernelGGL(lnbwd_combine_kernel<kCombineSlots>, dim3(2 * l.K * 256 / kCombineSlots), dim3(256), 0, s, a.part, groups, l.K, a.nvec, a.dgamma, a.dbeta);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) { *err = std::string("lnbwd_combine launch: ") + hipGetErrorString(e); return -1; }
  }
  return 0;
}

}  // namespace fs
