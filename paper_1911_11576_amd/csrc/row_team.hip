// Schedule 1, wavefront-team form: rows of 2049..32768 elements (a multiple of the
// 16-byte vector width) stay register-resident like in row_stitch, but one row is held by a
// team of W wavefronts (one workgroup).  Wavefront w of the team owns the 1 KB chunks
// w, w+W, w+2W, ... of the row (K chunks per wavefront), so the team reads W consecutive
// kilobytes per step.  Each row reduction is a wave64 all-reduce followed by one exchange
// of W partial values through LDS (block composition for the reduction only; the row
// itself never leaves the registers).
#include "row_stitch_impl.h"

namespace fs {

template <class Op>
__device__ __forceinline__ float team_allreduce(float v, float* slot, int waves, float identity) {
  v = group_allreduce<Op, 64>(v);
  if ((threadIdx.x & 63) == 0) slot[threadIdx.x >> 6] = v;
  __syncthreads();
  float r = identity;
  for (int w = 0; w < waves; ++w) r = Op::apply(r, slot[w]);   // same order in every thread
  return r;
}

template <typename T, int VARIANT, int K, bool EXACT>
__global__ __launch_bounds__(1024) void row_team_kernel(const RowArgs a) {
  constexpr int V = Vec<T>::V;
  constexpr bool kLN = VARIANT <= 1, kGelu = VARIANT == 1, kMask = VARIANT >= 3, kMaskBcast = VARIANT == 4;
  // two exchange buffers used alternately: a buffer is rewritten only after the barrier of
  // the other reduction has been passed by every wavefront
  __shared__ float exch[2][16];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, waves = blockDim.x >> 6;
  const T* __restrict__ x = static_cast<const T*>(a.x);
  T* __restrict__ y = static_cast<T*>(a.y);
  constexpr uint32_t kOne = sizeof(T) == 4 ? 0x3F800000u : (Vec<T>::kOneBits | (Vec<T>::kOneBits << 16));

  bool vld[K];
  int voff[K];
#pragma unroll
  for (int k = 0; k < K; ++k) {
    const int vi = (k * waves + w) * 64 + lane;
    vld[k] = EXACT || vi < a.nvec;
    voff[k] = (vld[k] ? vi : 0) * V;
  }

  for (int64_t row = blockIdx.x; row < a.rows; row += gridDim.x) {
    float v[K][V];
    u32x4 raw[K], aux[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
      raw[k] = stream_load16(x + row * a.cols + voff[k]);
      aux[k] = u32x4{0u, 0u, 0u, 0u};
    }
    if constexpr (kGelu) {
      if (a.res) {
#pragma unroll
        for (int k = 0; k < K; ++k) aux[k] = stream_load16(static_cast<const T*>(a.res) + row * a.cols + voff[k]);
      }
    }
    if constexpr (kMask) {
      const T* __restrict__ mk = static_cast<const T*>(a.mask);
      int64_t mrow = row;
      if constexpr (kMaskBcast) {
        const uint32_t r32 = (uint32_t)row;
        const uint32_t t = a.mask_d2.div(r32), i2 = r32 - t * a.mask_d2.d;
        const uint32_t i0 = a.mask_d1.div(t), i1 = t - i0 * a.mask_d1.d;
        mrow = i0 * a.ms0 + i1 * a.ms1 + i2 * a.ms2;
      }
#pragma unroll
      for (int k = 0; k < K; ++k)
        aux[k] = kMaskBcast ? Vec<T>::load_raw(mk + mrow * a.cols + voff[k]) : stream_load16(mk + mrow * a.cols + voff[k]);
    }
    // ---- thread-composed prologue ------------------------------------------------------
#pragma unroll
    for (int k = 0; k < K; ++k) {
      float av[V];
      Vec<T>::unpack(raw[k], v[k]);
      Vec<T>::unpack(aux[k], av);
      if constexpr (kGelu) {
        float b[V];
        u32x4 braw = u32x4{0u, 0u, 0u, 0u};
        if (a.bias) braw = Vec<T>::load_raw(static_cast<const T*>(a.bias) + voff[k]);
        Vec<T>::unpack(braw, b);
#pragma unroll
        for (int j = 0; j < V; ++j) {
          const float h = v[k][j] + b[j];
          const float e = __builtin_amdgcn_exp2f(h * (a.g_a0 + a.g_a1 * (h * h)));
          v[k][j] = (a.g_mul * h) * __builtin_amdgcn_rcpf(1.f + e) + av[j];
        }
      } else if constexpr (kMask) {
#pragma unroll
        for (int j = 0; j < V; ++j) v[k][j] = v[k][j] * a.scale + av[j];
      } else if constexpr (VARIANT == 2) {
#pragma unroll
        for (int j = 0; j < V; ++j) v[k][j] *= a.scale;
      }
    }
    // ---- row reductions across the team, epilogue, store ---------------------------------
    if constexpr (kLN) {
      float s = 0.f;
#pragma unroll
      for (int k = 0; k < K; ++k)
#pragma unroll
        for (int j = 0; j < V; ++j) s += vld[k] ? v[k][j] : 0.f;
      const float mean = team_allreduce<SumOp>(s, exch[0], waves, 0.f) * a.inv_n;
      float q = 0.f;
#pragma unroll
      for (int k = 0; k < K; ++k)
#pragma unroll
        for (int j = 0; j < V; ++j) {
          v[k][j] -= mean;
          q += vld[k] ? v[k][j] * v[k][j] : 0.f;
        }
      const float var = team_allreduce<SumOp>(q, exch[1], waves, 0.f) * a.inv_n;
      const float rstd = 1.f / sqrtf(var + a.eps);
#pragma unroll
      for (int k = 0; k < K; ++k) {
        u32x4 graw = u32x4{kOne, kOne, kOne, kOne}, braw = u32x4{0u, 0u, 0u, 0u};
        if (a.gamma) graw = Vec<T>::load_raw(static_cast<const T*>(a.gamma) + voff[k]);
        if (a.beta) braw = Vec<T>::load_raw(static_cast<const T*>(a.beta) + voff[k]);
        float o[V], gk[V], bk[V];
        Vec<T>::unpack(graw, gk);
        Vec<T>::unpack(braw, bk);
#pragma unroll
        for (int j = 0; j < V; ++j) o[j] = (v[k][j] * rstd) * gk[j] + bk[j];
        if (vld[k]) stream_store16(y + row * a.cols + voff[k], pack16<T>(o));
      }
    } else {
      float mx = -INFINITY;
#pragma unroll
      for (int k = 0; k < K; ++k)
#pragma unroll
        for (int j = 0; j < V; ++j) mx = fmaxf(mx, vld[k] ? v[k][j] : -INFINITY);
      mx = team_allreduce<MaxOp>(mx, exch[0], waves, -INFINITY);
      const float nmx = -mx * kLog2e;
      float s = 0.f;
#pragma unroll
      for (int k = 0; k < K; ++k)
#pragma unroll
        for (int j = 0; j < V; ++j) {
          const float e = vld[k] ? __builtin_amdgcn_exp2f(fmaf(v[k][j], kLog2e, nmx)) : 0.f;
          v[k][j] = e;
          s += e;
        }
      s = team_allreduce<SumOp>(s, exch[1], waves, 0.f);
      const float inv = 1.f / s;
#pragma unroll
      for (int k = 0; k < K; ++k) {
        float o[V];
#pragma unroll
        for (int j = 0; j < V; ++j) o[j] = v[k][j] * inv;
        if (vld[k]) stream_store16(y + row * a.cols + voff[k], pack16<T>(o));
      }
    }
  }
}

namespace {

template <typename T, int VARIANT, int K>
hipError_t team_launch_exact(const RowArgs& a, bool exact, int grid, int wg, hipStream_t s) {
  if (exact) hipLaunchKernelGGL((row_team_kernel<T, VARIANT, K, true>), dim3(grid), dim3(wg), 0, s, a);
  else hipLaunchKernelGGL((row_team_kernel<T, VARIANT, K, false>), dim3(grid), dim3(wg), 0, s, a);
  return hipGetLastError();
}

template <typename T, int VARIANT>
hipError_t team_launch_K(const RowArgs& a, int K, bool exact, int grid, int wg, hipStream_t s) {
  switch (K) {
    case 1: return team_launch_exact<T, VARIANT, 1>(a, exact, grid, wg, s);
    case 2: return team_launch_exact<T, VARIANT, 2>(a, exact, grid, wg, s);
    case 3: return team_launch_exact<T, VARIANT, 3>(a, exact, grid, wg, s);
    case 4: return team_launch_exact<T, VARIANT, 4>(a, exact, grid, wg, s);
    default: break;
  }
  if constexpr (Vec<T>::V == 4) {
    if (K == 6) return team_launch_exact<T, VARIANT, 6>(a, exact, grid, wg, s);
    if (K == 8) return team_launch_exact<T, VARIANT, 8>(a, exact, grid, wg, s);
  }
  return hipErrorInvalidValue;
}

template <typename T>
hipError_t team_launch_variant(const RowArgs& a, const RowTeamLaunch& l, hipStream_t s) {
  const bool exact = a.nvec == l.K * (l.wg / 64) * 64;
  switch (l.variant) {
    case 0: return team_launch_K<T, 0>(a, l.K, exact, l.grid, l.wg, s);
    case 1: return team_launch_K<T, 1>(a, l.K, exact, l.grid, l.wg, s);
    case 2: return team_launch_K<T, 2>(a, l.K, exact, l.grid, l.wg, s);
    case 3: return team_launch_K<T, 3>(a, l.K, exact, l.grid, l.wg, s);
    default: return team_launch_K<T, 4>(a, l.K, exact, l.grid, l.wg, s);
  }
}

int pick_team_K(int need, int kmax) {
  for (int k : {1, 2, 3, 4, 6, 8}) if (k >= need && k <= kmax) return k;
  return -1;
}

}  // namespace

bool row_team_plan(const RowSpec& sp, const LaunchOpts& opt, RowTeamLaunch* out, std::string* err) {
  const int V = 16 / dtype_size(sp.dtype);
  if (sp.cols % V != 0) { *err = "row schedule (team form): cols must be a multiple of the 16-byte vector width"; return false; }
  if (sp.rows >= (int64_t)1 << 31) { *err = "row schedule: rows >= 2^31"; return false; }
  const int64_t nvec = sp.cols / V;
  const int kmax = V == 4 ? 8 : 4;       // at most 32 fp32 values of a row per lane
  // smallest team whose lanes hold at most 16 values each, else the smallest that fits at all
  RowTeamLaunch l;
  int waves = 0;
  if (opt.wg_size) {
    if (opt.wg_size < 128 || opt.wg_size > 1024 || (opt.wg_size & (opt.wg_size - 1))) {
      *err = "row schedule (team form): wg_size must be a power of two in [128,1024]";
      return false;
    }
    waves = opt.wg_size / 64;
  } else {
    for (int wv = 2; wv <= 16 && !waves; wv *= 2)
      if (nvec <= (int64_t)wv * 64 * (16 / V)) waves = wv;
    for (int wv = 2; wv <= 16 && !waves; wv *= 2)
      if (nvec <= (int64_t)wv * 64 * kmax) waves = wv;
  }
  if (!waves) { *err = "row schedule (team form): row longer than 16 wavefronts' register tiles (cols > 32768)"; return false; }
  const int need = (int)((nvec + (int64_t)waves * 64 - 1) / ((int64_t)waves * 64));
  l.K = pick_team_K(need, kmax);
  if (l.K < 0) { *err = "row schedule (team form): row does not fit the team's registers"; return false; }
  l.wg = waves * 64;
  int64_t grid = sp.rows;
  if (opt.grid > 0 && opt.grid < grid) grid = opt.grid;
  if (grid > 0x7fffffff) grid = 0x7fffffff;
  l.grid = (int)(grid < 1 ? 1 : grid);
  const bool mask_bcast = !(sp.mask_d1 == 1 && sp.mask_d2 == 1 && sp.mask_stride[0] == 1);
  l.variant = sp.core == CORE_LAYERNORM ? (sp.gelu ? 1 : 0) : (sp.in_mask < 0 ? 2 : mask_bcast ? 4 : 3);
  *out = l;
  return true;
}

std::string row_team_describe(const RowSpec& sp, const RowTeamLaunch& l) {
  char buf[512];
  const char* r1 = sp.core == CORE_LAYERNORM ? "reduce_mean" : "reduce_max";
  const char* r2 = sp.core == CORE_LAYERNORM ? "reduce_var" : "reduce_sum";
  snprintf(buf, sizeof buf, "%s[GRID,CTA]; %s[GRID,CTA]; out[GRID,CTA-THREAD_%d]; cta_num=%d, cta_size=%d", r1, r2,
           l.K * (16 / dtype_size(sp.dtype)), l.grid, l.wg);
  return buf;
}

void row_fill_args(const RowSpec& sp, const void* const* in, void* const* out, RowArgs* a);

int row_team_launch(const RowSpec& sp, const RowTeamLaunch& l, const void* const* in, void* const* out,
                    void* stream, std::string* err) {
  if (sp.rows == 0 || sp.cols == 0) return 0;
  RowArgs a{};
  row_fill_args(sp, in, out, &a);
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e;
  switch (sp.dtype) {
    case DT_F32: e = team_launch_variant<float>(a, l, s); break;
    case DT_F16: e = team_launch_variant<f16_t>(a, l, s); break;
    default: e = team_launch_variant<bf16_t>(a, l, s); break;
  }
  if (e != hipSuccess) { *err = std::string("row_team launch: ") + hipGetErrorString(e); return -1; }
  return 0;
}

}  // namespace fs
