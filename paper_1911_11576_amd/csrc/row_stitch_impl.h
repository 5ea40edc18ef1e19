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
// groups in flight per loop iteration; consecutive wavefronts take consecutive row
// groups, so at any moment the chip streams one compact window of the tensors.
//
// This header holds the kernel template and its per-dtype dispatcher; one translation
// unit per storage dtype instantiates it (row_stitch_f32.hip, ...).
#pragma once
#include "dev_common.h"
#include "launchers.h"

namespace fs {

// Unsigned 32-bit division by a launch-time constant as multiply-high, subtract, shifts
// (Granlund & Montgomery's round-up method): q = (t + ((n - t) >> sh1)) >> sh2 with
// t = mulhi(m, n).  Exact for every n < 2^32.
struct FastDiv {
  uint32_t d = 1, m = 1, sh1 = 0, sh2 = 0;
  static FastDiv make(uint32_t d) {
    FastDiv f;
    f.d = d;
    uint32_t l = 0;
    while (l < 32 && ((uint64_t)1 << l) < d) ++l;            // ceil(log2 d)
    f.m = (uint32_t)((((uint64_t)1 << 32) * (((uint64_t)1 << l) - d)) / d + 1);
    f.sh1 = l < 1 ? l : 1;
    f.sh2 = l > 0 ? l - 1 : 0;
    return f;
  }
  __device__ __forceinline__ uint32_t div(uint32_t n) const {
    const uint32_t t = __umulhi(m, n);
    return (t + ((n - t) >> sh1)) >> sh2;
  }
};

struct RowArgs {
  const void* x; const void* res; const void* bias; const void* gamma; const void* beta;
  const void* mask; void* y;
  int64_t rows; int cols; int nvec;
  float scale, eps, inv_n;
  float g_mul, g_a0, g_a1;   // gelu: g = g_mul * h / (1 + exp2(h * (g_a0 + g_a1*h*h)))
  FastDiv mask_d1, mask_d2; int64_t ms0, ms1, ms2;
};

constexpr float kLog2e = 1.4426950408889634f;

// VARIANT: 0 LayerNorm, 1 prologue(bias,GELU,residual)+LayerNorm, 2 softmax, 3 softmax with a
// mask of the scores' shape, 4 softmax with a mask broadcast over leading dims
// EXACT: the row fills the lane tile exactly (cols == K*L*V): no per-vector masking
template <typename T, int VARIANT, int K, int L, int U, bool EXACT>
__global__ __launch_bounds__(512) void row_stitch_kernel(const RowArgs a) {
  constexpr int V = Vec<T>::V;
  constexpr int G = 64 / L;
  constexpr bool kLN = VARIANT <= 1, kGelu = VARIANT == 1, kMask = VARIANT >= 3, kMaskBcast = VARIANT == 4;
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
    vld[k] = EXACT || vi < a.nvec;
    voff[k] = (vld[k] ? vi : 0) * V;   // masked-off lanes re-read vector 0: always in bounds
  }

  // per-column operands (cached loads, kept packed in their storage dtype); an absent
  // operand becomes its neutral element so the per-element code has no conditionals.
  // The bias is needed first and is read up front; gamma and beta are read inside the
  // loop right where the epilogue needs them, which keeps them out of the register budget
  // while the row is being reduced (a one-shot grid visits one row group per wavefront, so
  // nothing is read twice; a persistent grid re-reads them from L1).
  constexpr uint32_t kOne = sizeof(T) == 4 ? 0x3F800000u : (Vec<T>::kOneBits | (Vec<T>::kOneBits << 16));
  u32x4 bia[K];
  if constexpr (kGelu) {
#pragma unroll
    for (int k = 0; k < K; ++k) {
      bia[k] = u32x4{0u, 0u, 0u, 0u};
      if (a.bias) bia[k] = Vec<T>::load_raw(static_cast<const T*>(a.bias) + voff[k]);
    }
  }

  const int64_t n_groups = (a.rows + G - 1) / G;
  const int64_t n_iters = (n_groups + U - 1) / U;
  const int64_t first = (int64_t)blockIdx.x * waves + (threadIdx.x >> 6);
  const int64_t stride = (int64_t)gridDim.x * waves;

  // all HBM reads of one iteration: the row groups of x and of the second streamed operand
  // (`aux`: the residual, or the mask)
  auto load_groups = [&](int64_t it, u32x4 (&raw)[U][K], u32x4 (&aux)[U][K], int64_t (&row)[U], bool (&rok)[U]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t r = (it * U + u) * G + sub;
      rok[u] = r < a.rows;
      row[u] = rok[u] ? r : a.rows - 1;
#pragma unroll
      for (int k = 0; k < K; ++k) {
        raw[u][k] = stream_load16(x + row[u] * a.cols + voff[k]);
        aux[u][k] = u32x4{0u, 0u, 0u, 0u};
      }
    }
    if constexpr (kGelu) {
      if (a.res) {
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
          for (int k = 0; k < K; ++k)
            aux[u][k] = stream_load16(static_cast<const T*>(a.res) + row[u] * a.cols + voff[k]);
      }
    }
    if constexpr (kMask) {
      const T* __restrict__ mk = static_cast<const T*>(a.mask);
#pragma unroll
      for (int u = 0; u < U; ++u) {
        int64_t mrow = row[u];
        if constexpr (kMaskBcast) {
          const uint32_t r32 = (uint32_t)row[u];
          const uint32_t t = a.mask_d2.div(r32), i2 = r32 - t * a.mask_d2.d;
          const uint32_t i0 = a.mask_d1.div(t), i1 = t - i0 * a.mask_d1.d;
          mrow = i0 * a.ms0 + i1 * a.ms1 + i2 * a.ms2;
        }
        // a broadcast mask row is shared by many score rows: cached load; a full mask is
        // touched once: streaming load
#pragma unroll
        for (int k = 0; k < K; ++k)
          aux[u][k] = kMaskBcast ? Vec<T>::load_raw(mk + mrow * a.cols + voff[k]) : stream_load16(mk + mrow * a.cols + voff[k]);
      }
    }
  };

  // (Register double buffering of the next iteration's loads on a persistent grid was tried
  // and measured 10-30% slower than this one-shot form on MI355X.)
  for (int64_t it = first; it < n_iters; it += stride) {
    float v[U][K][V];
    int64_t row[U];
    bool rok[U];
    u32x4 raw[U][K], aux[U][K];
    load_groups(it, raw, aux, row, rok);

    // ---- thread-composed prologue ---------------------------------------------------
    if constexpr (kGelu) {
#pragma unroll
      for (int k = 0; k < K; ++k) {
        float b[V];
        Vec<T>::unpack(bia[k], b);
#pragma unroll
        for (int u = 0; u < U; ++u) {
          float r[V];
          Vec<T>::unpack(raw[u][k], v[u][k]);
          Vec<T>::unpack(aux[u][k], r);
#pragma unroll
          for (int j = 0; j < V; ++j) {
            const float h = v[u][k][j] + b[j];
            // c*h*(1 + tanh(w)) == 2c*h / (1 + exp(-2w)); exp2 overflow gives rcp(inf) = 0
            const float e = __builtin_amdgcn_exp2f(h * (a.g_a0 + a.g_a1 * (h * h)));
            const float g = (a.g_mul * h) * __builtin_amdgcn_rcpf(1.f + e);
            v[u][k][j] = g + r[j];
          }
        }
      }
    } else if constexpr (kMask) {
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int k = 0; k < K; ++k) {
          float mm[V];
          Vec<T>::unpack(raw[u][k], v[u][k]);
          Vec<T>::unpack(aux[u][k], mm);
#pragma unroll
          for (int j = 0; j < V; ++j) v[u][k][j] = v[u][k][j] * a.scale + mm[j];
        }
    } else {
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int k = 0; k < K; ++k) {
          Vec<T>::unpack(raw[u][k], v[u][k]);
          if constexpr (VARIANT == 2) {
#pragma unroll
            for (int j = 0; j < V; ++j) v[u][k][j] *= a.scale;
          }
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
        u32x4 gam[K], bet[K];
#pragma unroll
        for (int k = 0; k < K; ++k) {
          gam[k] = u32x4{kOne, kOne, kOne, kOne};
          bet[k] = u32x4{0u, 0u, 0u, 0u};
          if (a.gamma) gam[k] = Vec<T>::load_raw(static_cast<const T*>(a.gamma) + voff[k]);
          if (a.beta) bet[k] = Vec<T>::load_raw(static_cast<const T*>(a.beta) + voff[k]);
        }
        const float var = group_allreduce<SumOp, L>(q) * a.inv_n;
        const float rstd = 1.f / sqrtf(var + a.eps);
#pragma unroll
        for (int k = 0; k < K; ++k) {
          float o[V], gk[V], bk[V];
          Vec<T>::unpack(gam[k], gk);
          Vec<T>::unpack(bet[k], bk);
#pragma unroll
          for (int j = 0; j < V; ++j) o[j] = (v[u][k][j] * rstd) * gk[j] + bk[j];
          if (rok[u] && vld[k]) stream_store16(y + row[u] * a.cols + voff[k], pack16<T>(o));
        }
      } else {
        float mx = -INFINITY;
#pragma unroll
        for (int k = 0; k < K; ++k)
#pragma unroll
          for (int j = 0; j < V; ++j) mx = fmaxf(mx, vld[k] ? v[u][k][j] : -INFINITY);
        mx = group_allreduce<MaxOp, L>(mx);
        const float nmx = -mx * kLog2e;
        float s = 0.f;
#pragma unroll
        for (int k = 0; k < K; ++k)
#pragma unroll
          for (int j = 0; j < V; ++j) {
            // exp(z - max) as one fma and one exp2
            const float e = vld[k] ? __builtin_amdgcn_exp2f(fmaf(v[u][k][j], kLog2e, nmx)) : 0.f;
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
          if (rok[u] && vld[k]) stream_store16(y + row[u] * a.cols + voff[k], pack16<T>(o));
        }
      }
    }
  }
}

// ---- per-dtype dispatch over (VARIANT, K, L, U, EXACT) --------------------------------
template <int KV> constexpr int max_rows_in_flight() { return KV <= 8 ? 4 : KV <= 16 ? 2 : 1; }

template <typename T, int VARIANT, int K, int L, int U>
hipError_t row_launch_exact(const RowArgs& a, bool exact, int grid, int wg, hipStream_t s) {
  if (exact) hipLaunchKernelGGL((row_stitch_kernel<T, VARIANT, K, L, U, true>), dim3(grid), dim3(wg), 0, s, a);
  else hipLaunchKernelGGL((row_stitch_kernel<T, VARIANT, K, L, U, false>), dim3(grid), dim3(wg), 0, s, a);
  return hipGetLastError();
}

template <typename T, int VARIANT, int K, int L>
hipError_t row_launch_U(const RowArgs& a, int U, bool exact, int grid, int wg, hipStream_t s) {
  constexpr int kMaxU = max_rows_in_flight<K * Vec<T>::V>();
  if constexpr (kMaxU >= 4) if (U == 4) return row_launch_exact<T, VARIANT, K, L, 4>(a, exact, grid, wg, s);
  if constexpr (kMaxU >= 2) if (U == 2) return row_launch_exact<T, VARIANT, K, L, 2>(a, exact, grid, wg, s);
  return row_launch_exact<T, VARIANT, K, L, 1>(a, exact, grid, wg, s);
}

template <typename T, int VARIANT>
hipError_t row_launch_KL(const RowArgs& a, int K, int L, int U, bool exact, int grid, int wg, hipStream_t s) {
  if (K == 1) {
    switch (L) {
      case 8: return row_launch_U<T, VARIANT, 1, 8>(a, U, exact, grid, wg, s);
      case 16: return row_launch_U<T, VARIANT, 1, 16>(a, U, exact, grid, wg, s);
      case 32: return row_launch_U<T, VARIANT, 1, 32>(a, U, exact, grid, wg, s);
      default: return row_launch_U<T, VARIANT, 1, 64>(a, U, exact, grid, wg, s);
    }
  }
  switch (K) {
    case 2: return row_launch_U<T, VARIANT, 2, 64>(a, U, exact, grid, wg, s);
    case 3: return row_launch_U<T, VARIANT, 3, 64>(a, U, exact, grid, wg, s);
    case 4: return row_launch_U<T, VARIANT, 4, 64>(a, U, exact, grid, wg, s);
    default: break;
  }
  // 6 or 8 vectors per lane fit the register file only for 4-byte elements
  if constexpr (Vec<T>::V == 4) {
    if (K == 6) return row_launch_U<T, VARIANT, 6, 64>(a, U, exact, grid, wg, s);
    if (K == 8) return row_launch_U<T, VARIANT, 8, 64>(a, U, exact, grid, wg, s);
  }
  return hipErrorInvalidValue;
}

template <typename T>
hipError_t row_launch_dtype(const RowArgs& a, const RowLaunch& rl, hipStream_t s) {
  const bool exact = a.nvec == rl.K * rl.L;
  switch (rl.variant) {
    case 0: return row_launch_KL<T, 0>(a, rl.K, rl.L, rl.U, exact, rl.grid, rl.wg, s);
    case 1: return row_launch_KL<T, 1>(a, rl.K, rl.L, rl.U, exact, rl.grid, rl.wg, s);
    case 2: return row_launch_KL<T, 2>(a, rl.K, rl.L, rl.U, exact, rl.grid, rl.wg, s);
    case 3: return row_launch_KL<T, 3>(a, rl.K, rl.L, rl.U, exact, rl.grid, rl.wg, s);
    default: return row_launch_KL<T, 4>(a, rl.K, rl.L, rl.U, exact, rl.grid, rl.wg, s);
  }
}

// defined one per translation unit
hipError_t row_launch_f32(const RowArgs& a, const RowLaunch& rl, hipStream_t s);
hipError_t row_launch_f16(const RowArgs& a, const RowLaunch& rl, hipStream_t s);
hipError_t row_launch_bf16(const RowArgs& a, const RowLaunch& rl, hipStream_t s);

}  // namespace fs
