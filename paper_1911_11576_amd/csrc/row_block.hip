// Schedule 1, block-composed form (paper Section 5.1: a reduction schedule may use warp or
// block composition, Section 5.3): the same groups as row_stitch, for rows that do not
// fit one wavefront's register tile (cols > 2048) or whose length is not a multiple of the
// 16-byte vector width.  One workgroup owns a row: the prologue's result is cached in LDS
// as fp32 (the `S` attribute), the two row reductions are wavefront all-reduces combined
// across wavefronts through LDS, and the epilogue reads the row back from LDS.  Every
// element of HBM is still touched exactly once.
//
// Rows whose length is a multiple of the vector width use 16-byte streaming loads and
// stores; other rows (row starts are then unaligned) use element accesses.
#include <mutex>
#include <set>

#include "row_stitch_impl.h"

namespace fs {

static constexpr int64_t kRowBlockLdsMax = 160 * 1024 - 1024;

template <class Op>
__device__ __forceinline__ float block_allreduce(float v, float* scratch, float identity) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, waves = blockDim.x >> 6;
  v = group_allreduce<Op, 64>(v);
  if (lane == 0) scratch[wave] = v;
  __syncthreads();
  float r = identity;
  for (int w = 0; w < waves; ++w) r = Op::apply(r, scratch[w]);   // same order in every thread
  __syncthreads();
  return r;
}

template <typename T, int VARIANT, bool VECTOR>
__global__ __launch_bounds__(1024) void row_block_kernel(const RowArgs a) {
  constexpr int V = Vec<T>::V;
  constexpr bool kLN = VARIANT <= 1, kGelu = VARIANT == 1, kMask = VARIANT >= 3, kMaskBcast = VARIANT == 4;
  extern __shared__ float row_lds[];            // [cols] then [16] reduction scratch
  float* scratch = row_lds + ((a.cols + 3) & ~3);
  const T* __restrict__ x = static_cast<const T*>(a.x);
  const T* __restrict__ res = static_cast<const T*>(a.res);
  const T* __restrict__ bias = static_cast<const T*>(a.bias);
  const T* __restrict__ gamma = static_cast<const T*>(a.gamma);
  const T* __restrict__ beta = static_cast<const T*>(a.beta);
  const T* __restrict__ mask = static_cast<const T*>(a.mask);
  T* __restrict__ y = static_cast<T*>(a.y);
  const int nt = blockDim.x;

  auto prologue = [&](float xv, float aux, int c) -> float {
    if constexpr (kGelu) {
      const float h = xv + (bias ? Vec<T>::load1(bias + c) : 0.f);
      const float e = __builtin_amdgcn_exp2f(h * (a.g_a0 + a.g_a1 * (h * h)));
      return (a.g_mul * h) * __builtin_amdgcn_rcpf(1.f + e) + aux;
    } else if constexpr (kMask) {
      return xv * a.scale + aux;
    } else if constexpr (VARIANT == 2) {
      return xv * a.scale;
    } else {
      return xv;
    }
  };

  for (int64_t row = blockIdx.x; row < a.rows; row += gridDim.x) {
    const int64_t base = row * a.cols;
    int64_t abase = base;                        // row start of the second streamed operand
    if constexpr (kMaskBcast) {
      const uint32_t r32 = (uint32_t)row;
      const uint32_t t = a.mask_d2.div(r32), i2 = r32 - t * a.mask_d2.d;
      const uint32_t i0 = a.mask_d1.div(t), i1 = t - i0 * a.mask_d1.d;
      abase = (i0 * a.ms0 + i1 * a.ms1 + i2 * a.ms2) * a.cols;
    }
    const T* auxp = kGelu ? res : mask;          // null when absent
    // ---- phase A: load, prologue, cache in LDS, first reduction -----------------------
    float red = kLN ? 0.f : -INFINITY;
    if constexpr (VECTOR) {
      for (int vi = threadIdx.x; vi < a.nvec; vi += nt) {
        float xv[V], av[V];
        Vec<T>::unpack(stream_load16(x + base + vi * V), xv);
#pragma unroll
        for (int j = 0; j < V; ++j) av[j] = 0.f;
        if ((kGelu || kMask) && auxp) {
          const u32x4 r = kMaskBcast ? Vec<T>::load_raw(auxp + abase + vi * V) : stream_load16(auxp + abase + vi * V);
          Vec<T>::unpack(r, av);
        }
#pragma unroll
        for (int j = 0; j < V; ++j) {
          const float v = prologue(xv[j], av[j], vi * V + j);
          row_lds[vi * V + j] = v;
          red = kLN ? red + v : fmaxf(red, v);
        }
      }
    } else {
      for (int c = threadIdx.x; c < a.cols; c += nt) {
        const float xv = Vec<T>::load1(x + base + c);
        const float av = ((kGelu || kMask) && auxp) ? Vec<T>::load1(auxp + abase + c) : 0.f;
        const float v = prologue(xv, av, c);
        row_lds[c] = v;
        red = kLN ? red + v : fmaxf(red, v);
      }
    }
    const float r1 = kLN ? block_allreduce<SumOp>(red, scratch, 0.f) * a.inv_n
                         : block_allreduce<MaxOp>(red, scratch, -INFINITY);
    // ---- phase B: second reduction over the cached row -----------------------------------
    float acc = 0.f;
    const float nmx = -r1 * kLog2e;
    for (int c = threadIdx.x; c < a.cols; c += nt) {
      if constexpr (kLN) {
        const float d = row_lds[c] - r1;
        row_lds[c] = d;
        acc += d * d;
      } else {
        const float e = __builtin_amdgcn_exp2f(fmaf(row_lds[c], kLog2e, nmx));
        row_lds[c] = e;
        acc += e;
      }
    }
    const float r2 = block_allreduce<SumOp>(acc, scratch, 0.f);
    const float mul = kLN ? 1.f / sqrtf(r2 * a.inv_n + a.eps) : 1.f / r2;
    // ---- phase C: epilogue from LDS, store ---------------------------------------------------
    if constexpr (VECTOR) {
      for (int vi = threadIdx.x; vi < a.nvec; vi += nt) {
        float o[V];
#pragma unroll
        for (int j = 0; j < V; ++j) {
          const int c = vi * V + j;
          o[j] = row_lds[c] * mul;
          if constexpr (kLN) {
            if (gamma) o[j] *= Vec<T>::load1(gamma + c);
            if (beta) o[j] += Vec<T>::load1(beta + c);
          }
        }
        stream_store16(y + base + vi * V, pack16<T>(o));
      }
    } else {
      for (int c = threadIdx.x; c < a.cols; c += nt) {
        float o = row_lds[c] * mul;
        if constexpr (kLN) {
          if (gamma) o *= Vec<T>::load1(gamma + c);
          if (beta) o += Vec<T>::load1(beta + c);
        }
        Vec<T>::store1(y + base + c, o);
      }
    }
    __syncthreads();   // the row buffer is reused by the next row
  }
}

namespace {

template <typename Kern>
hipError_t launch_block(Kern kern, const RowArgs& a, int grid, int wg, size_t lds, hipStream_t s) {
  if (lds > 64 * 1024) {   // more than 64 KB of dynamic LDS has to be enabled once per kernel
    static std::mutex mu;
    static std::set<const void*> raised;
    std::lock_guard<std::mutex> lock(mu);
    const void* f = reinterpret_cast<const void*>(kern);
    if (!raised.count(f)) {
      const hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kRowBlockLdsMax);
      if (e != hipSuccess) return e;
      raised.insert(f);
    }
  }
  hipLaunchKernelGGL(kern, dim3(grid), dim3(wg), lds, s, a);
  return hipGetLastError();
}

template <typename T, int VARIANT>
hipError_t launch_vec(const RowArgs& a, bool vec, int grid, int wg, size_t lds, hipStream_t s) {
  if (vec) return launch_block(row_block_kernel<T, VARIANT, true>, a, grid, wg, lds, s);
  return launch_block(row_block_kernel<T, VARIANT, false>, a, grid, wg, lds, s);
}

template <typename T>
hipError_t launch_variant(const RowArgs& a, int variant, bool vec, int grid, int wg, size_t lds, hipStream_t s) {
  switch (variant) {
    case 0: return launch_vec<T, 0>(a, vec, grid, wg, lds, s);
    case 1: return launch_vec<T, 1>(a, vec, grid, wg, lds, s);
    case 2: return launch_vec<T, 2>(a, vec, grid, wg, lds, s);
    case 3: return launch_vec<T, 3>(a, vec, grid, wg, lds, s);
    default: return launch_vec<T, 4>(a, vec, grid, wg, lds, s);
  }
}

}  // namespace

bool row_block_plan(const RowSpec& sp, const LaunchOpts& opt, RowBlockLaunch* out, int* status, std::string* err) {
  *status = 2;   // FS_ERR_UNSUPPORTED
  RowBlockLaunch l;
  l.lds_bytes = ((sp.cols + 3) / 4 * 4 + 16) * 4;
  if (l.lds_bytes > kRowBlockLdsMax) {
    *err = "row schedule (block form): the row does not fit the LDS row cache (cols > 40000)";
    *status = 3;  // FS_ERR_LDS
    return false;
  }
  if (sp.rows >= (int64_t)1 << 31 || sp.cols >= (int64_t)1 << 31) { *err = "row schedule: extent >= 2^31"; return false; }
  const int V = 16 / dtype_size(sp.dtype);
  l.vector = sp.cols % V == 0;
  int wg = 64;
  while (wg < 1024 && (int64_t)wg * 8 < sp.cols) wg *= 2;   // about 8 elements per thread and pass
  if (opt.wg_size) wg = opt.wg_size;
  if (wg < 64 || wg > 1024 || wg % 64) { *err = "row schedule (block form): wg_size must be a multiple of 64 in [64,1024]"; *status = 1; return false; }
  l.wg = wg;
  int64_t grid = sp.rows;
  const int64_t cap = 256 * 16;   // persistent beyond 16 workgroups per CU
  if (grid > cap) grid = cap;
  if (opt.grid > 0 && opt.grid < grid) grid = opt.grid;
  l.grid = (int)(grid < 1 ? 1 : grid);
  const bool mask_bcast = !(sp.mask_d1 == 1 && sp.mask_d2 == 1 && sp.mask_stride[0] == 1);
  l.variant = sp.core == CORE_LAYERNORM ? (sp.gelu ? 1 : 0) : (sp.in_mask < 0 ? 2 : mask_bcast ? 4 : 3);
  *out = l;
  *status = 0;
  return true;
}

std::string row_block_describe(const RowSpec& sp, const RowBlockLaunch& l) {
  char buf[512];
  const char* r1 = sp.core == CORE_LAYERNORM ? "reduce_mean" : "reduce_max";
  const char* r2 = sp.core == CORE_LAYERNORM ? "reduce_var" : "reduce_sum";
  snprintf(buf, sizeof buf, "prologue[GRID,CTA]S; %s[GRID,CTA]; %s[GRID,CTA]; out[GRID,CTA%s]; cta_num=%d, cta_size=%d, lds=%lld",
           r1, r2, l.vector ? "-THREAD_V" : "", l.grid, l.wg, (long long)l.lds_bytes);
  return buf;
}

void row_fill_args(const RowSpec& sp, const void* const* in, void* const* out, RowArgs* a);

int row_block_launch(const RowSpec& sp, const RowBlockLaunch& l, const void* const* in, void* const* out,
                     void* stream, std::string* err) {
  if (sp.rows == 0 || sp.cols == 0) return 0;
  RowArgs a{};
  row_fill_args(sp, in, out, &a);
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e;
  const size_t lds = (size_t)l.lds_bytes;
  switch (sp.dtype) {
    case DT_F32: e = launch_variant<float>(a, l.variant, l.vector, l.grid, l.wg, lds, s); break;
    case DT_F16: e = launch_variant<f16_t>(a, l.variant, l.vector, l.grid, l.wg, lds, s); break;
    default: e = launch_variant<bf16_t>(a, l.variant, l.vector, l.grid, l.wg, lds, s); break;
  }
  if (e != hipSuccess) { *err = std::string("row_block launch: ") + hipGetErrorString(e); return -1; }
  return 0;
}

}  // namespace fs
