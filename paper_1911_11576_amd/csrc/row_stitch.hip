// Schedule 1 (warp composition, paper Section 5.1): an elementwise prologue, one or two
// row reductions whose results are broadcast back to the row, and an elementwise
// epilogue, stitched into one kernel.  A row (or a group of 64/L short rows) lives in
// the VGPRs of one wavefront from its single HBM read to its single HBM write; the
// reductions are wave64 DPP/permlane all-reduces, so the reduced value reaches every
// dependent op through registers and nothing goes through LDS.
//
// Layout: rows are contiguous, `cols` a multiple of the 16-byte vector width V.  Lane l
// of a row group owns vectors l, l+L, ..., l+(K-1)L of the row (consecutive lanes read
// consecutive 16-byte vectors: fully coalesced).  A wavefront keeps U independent row
// groups in flight per loop iteration.
#include "dev_common.h"
#include "launchers.h"

namespace fs {

struct RowArgs {
  const void* x; const void* res; const void* bias; const void* gamma; const void* beta;
  const void* mask; void* y;
  int64_t rows; int cols; int nvec;
  float scale, eps, inv_n, g_half, g_k0, g_k1;
  int mask_general; uint32_t mask_d1, mask_d2; int64_t ms0, ms1, ms2;
};

// VARIANT: 0 LayerNorm, 1 prologue(bias,GELU,residual)+LayerNorm, 2 softmax, 3 masked softmax
template <typename T, int VARIANT, int K, int L, int U>
__global__ __launch_bounds__(512) void row_stitch_kernel(const RowArgs a) {
  constexpr int V = Vec<T>::V;
  constexpr int G = 64 / L;
  constexpr bool kLN = VARIANT <= 1, kGelu = VARIANT == 1, kMask = VARIANT == 3;
  const int lane = threadIdx.x & 63;
  const int sub = lane / L, l = lane % L;
  const int waves = blockDim.x >> 6;
  const T* __restrict__ x = static_cast<const T*>(a.x);
  T* __restrict__ y = static_cast<T*>(a.y);

  bool vld[K];
  int voff[K];
#pragma unroll
  for (int k = 0; k < K; ++k) {
    const int vi = k * L + l;
    vld[k] = vi < a.nvec;
    voff[k] = (vld[k] ? vi : 0) * V;   // masked-off lanes re-read vector 0: always in bounds
  }

  // per-column operands: read once per wavefront and kept (still packed in their storage
  // dtype) in registers for all its rows
  u32x4 gam[K], bet[K], bia[K];
  if constexpr (kLN) {
#pragma unroll
    for (int k = 0; k < K; ++k) {
      if (a.gamma) gam[k] = Vec<T>::load_raw(static_cast<const T*>(a.gamma) + voff[k]);
      if (a.beta) bet[k] = Vec<T>::load_raw(static_cast<const T*>(a.beta) + voff[k]);
      if constexpr (kGelu) if (a.bias) bia[k] = Vec<T>::load_raw(static_cast<const T*>(a.bias) + voff[k]);
    }
  }

  const int64_t n_groups = (a.rows + G - 1) / G;
  const int64_t n_iters = (n_groups + U - 1) / U;
  for (int64_t it = (int64_t)blockIdx.x * waves + (threadIdx.x >> 6); it < n_iters;
       it += (int64_t)gridDim.x * waves) {
    float v[U][K][V];
    int64_t row[U];
    bool rok[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t r = (it * U + u) * G + sub;
      rok[u] = r < a.rows;
      row[u] = rok[u] ? r : a.rows - 1;
#pragma unroll
      for (int k = 0; k < K; ++k) Vec<T>::load(x + row[u] * a.cols + voff[k], v[u][k]);
    }

    // ---- thread-composed prologue ---------------------------------------------------
    if constexpr (kGelu) {
      u32x4 rs[U][K];
      if (a.res) {
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
          for (int k = 0; k < K; ++k)
            rs[u][k] = Vec<T>::load_raw(static_cast<const T*>(a.res) + row[u] * a.cols + voff[k]);
      }
#pragma unroll
      for (int k = 0; k < K; ++k) {
        float b[V];
        if (a.bias) Vec<T>::unpack(bia[k], b);
#pragma unroll
        for (int u = 0; u < U; ++u) {
          float r[V];
          if (a.res) Vec<T>::unpack(rs[u][k], r);
#pragma unroll
          for (int j = 0; j < V; ++j) {
            const float h = a.bias ? v[u][k][j] + b[j] : v[u][k][j];
            const float w = a.g_k0 * (h + a.g_k1 * (h * h * h));
            // tanh(w) = 1 - 2/(exp(2w)+1); exp overflow to +inf gives exactly 1
            const float t = 1.f - 2.f / (__expf(2.f * w) + 1.f);
            const float g = (a.g_half * h) * (1.f + t);
            v[u][k][j] = a.res ? g + r[j] : g;
          }
        }
      }
    }
    if constexpr (VARIANT >= 2) {
      if constexpr (kMask) {
        u32x4 m[U][K];
        const T* __restrict__ mk = static_cast<const T*>(a.mask);
#pragma unroll
        for (int u = 0; u < U; ++u) {
          int64_t mrow = row[u];
          if (a.mask_general) {
            const uint32_t r32 = (uint32_t)row[u];
            const uint32_t i2 = r32 % a.mask_d2, t = r32 / a.mask_d2;
            const uint32_t i1 = t % a.mask_d1, i0 = t / a.mask_d1;
            mrow = i0 * a.ms0 + i1 * a.ms1 + i2 * a.ms2;
          }
#pragma unroll
          for (int k = 0; k < K; ++k) m[u][k] = Vec<T>::load_raw(mk + mrow * a.cols + voff[k]);
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
          for (int k = 0; k < K; ++k) {
            float mm[V];
            Vec<T>::unpack(m[u][k], mm);
#pragma unroll
            for (int j = 0; j < V; ++j) v[u][k][j] = v[u][k][j] * a.scale + mm[j];
          }
      } else {
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
          for (int k = 0; k < K; ++k)
#pragma unroll
            for (int j = 0; j < V; ++j) v[u][k][j] *= a.scale;
      }
    }

    // ---- row reductions with register broadcast, epilogue, store ---------------------
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if constexpr (kLN) {
        float s = 0.f;
#pragma unroll
        for (int k = 0; k < K; ++k)
#pragma unroll
          for (int j = 0; j < V; ++j) s += vld[k] ? v[u][k][j] : 0.f;
        const float mean = group_allreduce<SumOp, L>(s) * a.inv_n;
        float q = 0.f;
#pragma unroll
        for (int k = 0; k < K; ++k)
#pragma unroll
          for (int j = 0; j < V; ++j) {
            v[u][k][j] -= mean;
            q += vld[k] ? v[u][k][j] * v[u][k][j] : 0.f;
          }
        const float var = group_allreduce<SumOp, L>(q) * a.inv_n;
        const float rstd = 1.f / sqrtf(var + a.eps);
#pragma unroll
        for (int k = 0; k < K; ++k) {
          float o[V], gk[V], bk[V];
          if (a.gamma) Vec<T>::unpack(gam[k], gk);
          if (a.beta) Vec<T>::unpack(bet[k], bk);
#pragma unroll
          for (int j = 0; j < V; ++j) {
            o[j] = v[u][k][j] * rstd;
            if (a.gamma) o[j] *= gk[j];
            if (a.beta) o[j] += bk[j];
          }
          if (rok[u] && vld[k]) Vec<T>::store(y + row[u] * a.cols + voff[k], o);
        }
      } else {
        float mx = -INFINITY;
#pragma unroll
        for (int k = 0; k < K; ++k)
#pragma unroll
          for (int j = 0; j < V; ++j) mx = fmaxf(mx, vld[k] ? v[u][k][j] : -INFINITY);
        mx = group_allreduce<MaxOp, L>(mx);
        float s = 0.f;
#pragma unroll
        for (int k = 0; k < K; ++k)
#pragma unroll
          for (int j = 0; j < V; ++j) {
            const float e = vld[k] ? __expf(v[u][k][j] - mx) : 0.f;
            v[u][k][j] = e;
            s += e;
          }
        s = group_allreduce<SumOp, L>(s);
        const float inv = 1.f / s;
#pragma unroll
        for (int k = 0; k < K; ++k) {
          float o[V];
#pragma unroll
          for (int j = 0; j < V; ++j) o[j] = v[u][k][j] * inv;
          if (rok[u] && vld[k]) Vec<T>::store(y + row[u] * a.cols + voff[k], o);
        }
      }
    }
  }
}

// ----------------------------------------------------------------------------------------
// host side
// ----------------------------------------------------------------------------------------
namespace {

// K*U vectors per lane in flight; instantiated combinations only
constexpr int kKs[] = {1, 2, 3, 4, 6, 8};

int pick_K(int nvec) {
  const int need = (nvec + 63) / 64;
  for (int k : kKs) if (k >= need) return k;
  return -1;
}

int pick_L(int nvec) {
  if (nvec >= 64) return 64;
  int L = 8;
  while (L < nvec) L *= 2;
  return L;
}

template <typename T, int VARIANT, int K, int L, int U>
hipError_t launch_one(const RowArgs& a, int grid, int wg, hipStream_t s) {
  hipLaunchKernelGGL((row_stitch_kernel<T, VARIANT, K, L, U>), dim3(grid), dim3(wg), 0, s, a);
  return hipGetLastError();
}

template <typename T, int VARIANT, int K, int L>
hipError_t launch_U(const RowArgs& a, int U, int grid, int wg, hipStream_t s) {
  constexpr int kMaxU = (K * Vec<T>::V <= 8) ? 4 : (K * Vec<T>::V <= 16) ? 2 : 1;
  if constexpr (kMaxU >= 4) if (U == 4) return launch_one<T, VARIANT, K, L, 4>(a, grid, wg, s);
  if constexpr (kMaxU >= 2) if (U == 2) return launch_one<T, VARIANT, K, L, 2>(a, grid, wg, s);
  return launch_one<T, VARIANT, K, L, 1>(a, grid, wg, s);
}

template <typename T, int VARIANT>
hipError_t launch_KL(const RowArgs& a, int K, int L, int U, int grid, int wg, hipStream_t s) {
  if (K == 1) {
    switch (L) {
      case 8: return launch_U<T, VARIANT, 1, 8>(a, U, grid, wg, s);
      case 16: return launch_U<T, VARIANT, 1, 16>(a, U, grid, wg, s);
      case 32: return launch_U<T, VARIANT, 1, 32>(a, U, grid, wg, s);
      default: return launch_U<T, VARIANT, 1, 64>(a, U, grid, wg, s);
    }
  }
  switch (K) {
    case 2: return launch_U<T, VARIANT, 2, 64>(a, U, grid, wg, s);
    case 3: return launch_U<T, VARIANT, 3, 64>(a, U, grid, wg, s);
    case 4: return launch_U<T, VARIANT, 4, 64>(a, U, grid, wg, s);
    default: break;
  }
  // 6 or 8 vectors per lane fit the register file only for 4-byte elements
  if constexpr (Vec<T>::V == 4) {
    if (K == 6) return launch_U<T, VARIANT, 6, 64>(a, U, grid, wg, s);
    if (K == 8) return launch_U<T, VARIANT, 8, 64>(a, U, grid, wg, s);
  }
  return hipErrorInvalidValue;
}

template <typename T>
hipError_t launch_variant(const RowArgs& a, int variant, int K, int L, int U, int grid, int wg,
                          hipStream_t s) {
  switch (variant) {
    case 0: return launch_KL<T, 0>(a, K, L, U, grid, wg, s);
    case 1: return launch_KL<T, 1>(a, K, L, U, grid, wg, s);
    case 2: return launch_KL<T, 2>(a, K, L, U, grid, wg, s);
    default: return launch_KL<T, 3>(a, K, L, U, grid, wg, s);
  }
}

int max_U(int K, int V) { return K * V <= 8 ? 4 : K * V <= 16 ? 2 : 1; }

}  // namespace

bool row_stitch_plan(const RowSpec& sp, const LaunchOpts& opt, RowLaunch* out, std::string* err) {
  const int V = 16 / dtype_size(sp.dtype);
  if (sp.cols % V != 0) { *err = "row schedule: cols must be a multiple of the 16-byte vector width"; return false; }
  const int64_t nvec = sp.cols / V;
  // one wavefront holds a whole row in registers: at most 32 fp32 values per lane
  if (sp.cols > 2048) { *err = "row schedule: row longer than one wavefront's register tile (cols > 2048)"; return false; }
  if (sp.rows >= (int64_t)1 << 31) { *err = "row schedule: rows >= 2^31"; return false; }
  RowLaunch rl;
  rl.K = pick_K((int)nvec);
  rl.L = pick_L((int)nvec);
  rl.wg = opt.wg_size ? opt.wg_size : 256;
  if (rl.wg < 64 || rl.wg > 512 || rl.wg % 64) { *err = "row schedule: wg_size must be a multiple of 64 in [64,512]"; return false; }
  int U = opt.rows_per_wave ? opt.rows_per_wave : max_U(rl.K, V);
  if (U < 1 || U > 8) { *err = "rows_per_wave out of range [1,8]"; return false; }
  const int mu = max_U(rl.K, V);
  rl.U = U >= 4 && mu >= 4 ? 4 : U >= 2 && mu >= 2 ? 2 : 1;
  const int G = 64 / rl.L;
  const int64_t n_groups = (sp.rows + G - 1) / G;
  const int64_t n_iters = (n_groups + rl.U - 1) / rl.U;
  const int waves = rl.wg / 64;
  int64_t grid = (n_iters + waves - 1) / waves;
  if (opt.grid > 0 && opt.grid < grid) grid = opt.grid;
  if (grid > 0x7fffffff) grid = 0x7fffffff;
  rl.grid = (int)grid;
  rl.variant = sp.core == CORE_LAYERNORM ? (sp.gelu ? 1 : 0) : (sp.in_mask >= 0 ? 3 : 2);
  *out = rl;
  return true;
}

std::string row_stitch_describe(const RowSpec& sp, const RowLaunch& rl) {
  // one schedule per reduction and per output, in the template notation of Section 5.2:
  // rows are tiled GRID then WARP (U row groups of 64/L rows per wavefront), columns are
  // WARP-parallel with K vectors per lane; nothing carries the S attribute
  char buf[512];
  const int G = 64 / rl.L;
  const char* r1 = sp.core == CORE_LAYERNORM ? "reduce_mean" : "reduce_max";
  const char* r2 = sp.core == CORE_LAYERNORM ? "reduce_var" : "reduce_sum";
  snprintf(buf, sizeof buf,
           "%s[GRID-WARP_%d,WARP]; %s[GRID-WARP_%d,WARP]; out[GRID-WARP_%d,WARP-THREAD_%d]; "
           "cta_num=%d, cta_size=%d",
           r1, rl.U * G, r2, rl.U * G, rl.U * G, rl.K * (16 / dtype_size(sp.dtype)), rl.grid, rl.wg);
  return buf;
}

int row_stitch_launch(const RowSpec& sp, const RowLaunch& rl, const void* const* in, void* const* out,
                      void* stream, std::string* err) {
  if (sp.rows == 0 || sp.cols == 0) return 0;
  RowArgs a{};
  a.x = in[sp.in_x];
  a.res = sp.in_res >= 0 ? in[sp.in_res] : nullptr;
  a.bias = sp.in_bias >= 0 ? in[sp.in_bias] : nullptr;
  a.gamma = sp.in_gamma >= 0 ? in[sp.in_gamma] : nullptr;
  a.beta = sp.in_beta >= 0 ? in[sp.in_beta] : nullptr;
  a.mask = sp.in_mask >= 0 ? in[sp.in_mask] : nullptr;
  a.y = out[0];
  a.rows = sp.rows;
  a.cols = (int)sp.cols;
  a.nvec = (int)(sp.cols / (16 / dtype_size(sp.dtype)));
  a.scale = sp.scale; a.eps = sp.eps; a.inv_n = (float)(1.0 / (double)sp.cols);
  a.g_half = sp.gelu_half; a.g_k0 = sp.gelu_k0; a.g_k1 = sp.gelu_k1;
  a.mask_general = !(sp.mask_d1 == 1 && sp.mask_d2 == 1 && sp.mask_stride[0] == 1);
  a.mask_d1 = (uint32_t)sp.mask_d1; a.mask_d2 = (uint32_t)sp.mask_d2;
  a.ms0 = sp.mask_stride[0]; a.ms1 = sp.mask_stride[1]; a.ms2 = sp.mask_stride[2];
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e;
  switch (sp.dtype) {
    case DT_F32: e = launch_variant<float>(a, rl.variant, rl.K, rl.L, rl.U, rl.grid, rl.wg, s); break;
    case DT_F16: e = launch_variant<f16_t>(a, rl.variant, rl.K, rl.L, rl.U, rl.grid, rl.wg, s); break;
    default: e = launch_variant<bf16_t>(a, rl.variant, rl.K, rl.L, rl.U, rl.grid, rl.wg, s); break;
  }
  if (e != hipSuccess) { *err = std::string("row_stitch launch: ") + hipGetErrorString(e); return -1; }
  return 0;
}

}  // namespace fs
