// Per-op baseline: generic one-kernel-per-op execution of a fusion group (see per_op.h).
// Elementwise kernels move 16 bytes per lane where shapes allow, reductions are one
// wavefront per row or two-stage over columns, the batched dot is a plain LDS-tiled FMA
// kernel: the same care a framework's stock kernels get, but every intermediate makes a
// round trip through HBM.
#include "dev_common.h"
#include "per_op.h"

namespace fs {

// how `n` (a value of the consumer's shape) maps onto memory
PerOpView view_of(const Graph& g, int n) {
  const Node& x = g[n];
  PerOpView v;
  if (x.kind == FS_CONSTANT) { v.base = -1; v.cval = (float)x.attr; v.full = false; return v; }
  if (x.kind == FS_BROADCAST) {
    const PerOpView o = view_of(g, x.operand[0]);
    const Node& a = g[x.operand[0]];
    v.base = o.base; v.full = false;
    for (int d = 0; d < a.rank; ++d) v.stride[x.axis + d] = a.shape[d] == 1 ? 0 : o.stride[d];
    return v;
  }
  if (x.kind == FS_OUTPUT) return view_of(g, x.operand[0]);
  v.base = n; v.full = true;
  int64_t s = 1;
  for (int d = x.rank - 1; d >= 0; --d) { v.stride[d] = s; s *= x.shape[d]; }
  return v;
}

namespace {

// ------------------------------------------------------------------------------------
// device
// ------------------------------------------------------------------------------------
struct EwOperand {
  const void* p;
  float cval;
  int is_const, full;
  int64_t s[FS_MAX_RANK];
};
struct EwArgs {
  EwOperand a, b;
  void* out;
  int64_t n;
  int kind, rank;
  int64_t shape[FS_MAX_RANK];
  float attr;
};

__device__ __forceinline__ float ew_apply(int kind, float x, float y) {
  switch (kind) {
    case FS_ADD: return x + y;
    case FS_SUBTRACT: return x - y;
    case FS_MULTIPLY: return x * y;
    case FS_DIVIDE: return x / y;
    case FS_MAXIMUM: return fmaxf(x, y);
    case FS_NEGATE: return -x;
    case FS_EXP: return expf(x);
    case FS_LOG: return logf(x);
    case FS_TANH: return tanhf(x);
    case FS_RSQRT: return 1.f / sqrtf(x);
    case FS_SQRT: return sqrtf(x);
    case FS_ERF: return erff(x);
    case FS_LOGISTIC: return 1.f / (1.f + expf(-x));
    default: return x;   // convert, copy
  }
}

template <typename T> __device__ __forceinline__ void load8(const T* p, float (&o)[8]);
template <> __device__ __forceinline__ void load8<float>(const float* p, float (&o)[8]) {
  float lo[4], hi[4];
  Vec<float>::load(p, lo); Vec<float>::load(p + 4, hi);
#pragma unroll
  for (int i = 0; i < 4; ++i) { o[i] = lo[i]; o[4 + i] = hi[i]; }
}
template <> __device__ __forceinline__ void load8<f16_t>(const f16_t* p, float (&o)[8]) { Vec<f16_t>::load(p, o); }
template <> __device__ __forceinline__ void load8<bf16_t>(const bf16_t* p, float (&o)[8]) { Vec<bf16_t>::load(p, o); }

template <typename T> __device__ __forceinline__ void store8(T* p, const float (&v)[8]);
template <> __device__ __forceinline__ void store8<float>(float* p, const float (&v)[8]) {
  const float lo[4] = {v[0], v[1], v[2], v[3]}, hi[4] = {v[4], v[5], v[6], v[7]};
  Vec<float>::store(p, lo); Vec<float>::store(p + 4, hi);
}
template <> __device__ __forceinline__ void store8<f16_t>(f16_t* p, const float (&v)[8]) { Vec<f16_t>::store(p, v); }
template <> __device__ __forceinline__ void store8<bf16_t>(bf16_t* p, const float (&v)[8]) { Vec<bf16_t>::store(p, v); }

__device__ __forceinline__ void decompose(int64_t e, int rank, const int64_t* shape, int64_t (&idx)[FS_MAX_RANK]) {
#pragma unroll
  for (int d = FS_MAX_RANK - 1; d >= 0; --d) {
    if (d < rank) { idx[d] = e % shape[d]; e /= shape[d]; } else idx[d] = 0;
  }
}

template <typename Tin>
__device__ __forceinline__ void fetch8(const EwOperand& o, int64_t e0, const int64_t (&idx)[FS_MAX_RANK], int rank,
                                       float (&v)[8]) {
  if (o.is_const) {
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = o.cval;
  } else if (o.full) {
    load8<Tin>(static_cast<const Tin*>(o.p) + e0, v);
  } else {
    int64_t off = 0;
    for (int d = 0; d < rank; ++d) off += idx[d] * o.s[d];
    if (o.s[rank - 1] == 1) load8<Tin>(static_cast<const Tin*>(o.p) + off, v);
    else {
      const float x = Vec<Tin>::load1(static_cast<const Tin*>(o.p) + off);
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] = x;
    }
  }
}

// 8 elements per thread; needs n % 8 == 0 and the last extent % 8 == 0
template <typename Tin, typename Tout>
__global__ __launch_bounds__(256) void ew_vec_kernel(const EwArgs a) {
  const int64_t nchunk = a.n / 8;
  const bool need_idx = (!a.a.is_const && !a.a.full) || (!a.b.is_const && !a.b.full) || a.kind == FS_CAUSAL_MASK;
  for (int64_t ci = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; ci < nchunk; ci += (int64_t)gridDim.x * blockDim.x) {
    const int64_t e0 = ci * 8;
    int64_t idx[FS_MAX_RANK] = {0, 0, 0, 0};
    if (need_idx) decompose(e0, a.rank, a.shape, idx);
    float x[8], y[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}, r[8];
    fetch8<Tin>(a.a, e0, idx, a.rank, x);
    if (a.kind >= FS_ADD && a.kind <= FS_MAXIMUM) fetch8<Tin>(a.b, e0, idx, a.rank, y);
    if (a.kind == FS_CAUSAL_MASK) {
      const int64_t i = idx[a.rank - 2], j0 = idx[a.rank - 1];
#pragma unroll
      for (int k = 0; k < 8; ++k) r[k] = (j0 + k <= i) ? x[k] : a.attr;
    } else {
#pragma unroll
      for (int k = 0; k < 8; ++k) r[k] = ew_apply(a.kind, x[k], y[k]);
    }
    store8<Tout>(static_cast<Tout*>(a.out) + e0, r);
  }
}

template <typename Tin, typename Tout>
__global__ __launch_bounds__(256) void ew_scalar_kernel(const EwArgs a) {
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < a.n; e += (int64_t)gridDim.x * blockDim.x) {
    int64_t idx[FS_MAX_RANK];
    decompose(e, a.rank, a.shape, idx);
    float v[2] = {0.f, 0.f};
    const EwOperand* ops[2] = {&a.a, &a.b};
    const int nop = (a.kind >= FS_ADD && a.kind <= FS_MAXIMUM) ? 2 : 1;
    for (int k = 0; k < nop; ++k) {
      const EwOperand& o = *ops[k];
      if (o.is_const) v[k] = o.cval;
      else {
        int64_t off = e;
        if (!o.full) { off = 0; for (int d = 0; d < a.rank; ++d) off += idx[d] * o.s[d]; }
        v[k] = Vec<Tin>::load1(static_cast<const Tin*>(o.p) + off);
      }
    }
    float r;
    if (a.kind == FS_CAUSAL_MASK) r = idx[a.rank - 1] <= idx[a.rank - 2] ? v[0] : a.attr;
    else r = ew_apply(a.kind, v[0], v[1]);
    Vec<Tout>::store1(static_cast<Tout*>(a.out) + e, r);
  }
}

// one wavefront per row of [outer, red]
template <typename T>
__global__ __launch_bounds__(256) void row_reduce_kernel(const T* __restrict__ in, T* __restrict__ out,
                                                         int64_t outer, int64_t red, int is_max, int vec) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (row >= outer) return;   // whole wavefront leaves together
  const T* p = in + row * red;
  float acc = is_max ? -INFINITY : 0.f;
  if (vec) {
    for (int64_t c = lane * 8; c < red; c += 64 * 8) {
      float v[8];
      load8<T>(p + c, v);
#pragma unroll
      for (int k = 0; k < 8; ++k) acc = is_max ? fmaxf(acc, v[k]) : acc + v[k];
    }
  } else {
    for (int64_t c = lane; c < red; c += 64) {
      const float v = Vec<T>::load1(p + c);
      acc = is_max ? fmaxf(acc, v) : acc + v;
    }
  }
  acc = is_max ? group_allreduce<MaxOp, 64>(acc) : group_allreduce<SumOp, 64>(acc);
  if (lane == 0) Vec<T>::store1(out + row, acc);
}

// [outer, red, inner] -> partial[outer, chunks, inner] (fp64 sums / fp32-exact max)
template <typename T>
__global__ __launch_bounds__(256) void col_reduce_stage1(const T* __restrict__ in, double* __restrict__ part,
                                                         int64_t red, int64_t inner, int chunks, int is_max) {
  const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= inner) return;
  const int chunk = blockIdx.y;
  const int64_t o = blockIdx.z;
  const int64_t per = (red + chunks - 1) / chunks;
  const int64_t r0 = chunk * per, r1 = min(red, r0 + per);
  double acc = is_max ? -INFINITY : 0.0;
  const T* p = in + o * red * inner + c;
  for (int64_t r = r0; r < r1; ++r) {
    const double v = (double)Vec<T>::load1(p + r * inner);
    acc = is_max ? fmax(acc, v) : acc + v;
  }
  part[(o * chunks + chunk) * inner + c] = acc;
}

template <typename T>
__global__ __launch_bounds__(256) void col_reduce_stage2(const double* __restrict__ part, T* __restrict__ out,
                                                         int64_t inner, int chunks, int is_max) {
  const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= inner) return;
  const int64_t o = blockIdx.y;
  double acc = is_max ? -INFINITY : 0.0;
  int k = 0;
  for (; k + 8 <= chunks; k += 8) {   // eight independent loads in flight
    double v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = part[(o * chunks + k + j) * inner + c];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc = is_max ? fmax(acc, v[j]) : acc + v[j];
  }
  for (; k < chunks; ++k) {
    const double v = part[(o * chunks + k) * inner + c];
    acc = is_max ? fmax(acc, v) : acc + v;
  }
  Vec<T>::store1(out + o * inner + c, (float)acc);
}

// C[b] = A[b] (M x K) . B[b] (K x N, or N x K when transpose_b); 64x64 tile, 4x4 per thread
template <typename Tin, typename Tout>
__global__ __launch_bounds__(256) void dot_kernel(const Tin* __restrict__ A, const Tin* __restrict__ B,
                                                  Tout* __restrict__ C, int M, int N, int K, int transpose_b) {
  __shared__ float As[16][65], Bs[16][65];
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  const int64_t bz = blockIdx.z;
  A += bz * M * K; B += bz * (int64_t)K * N; C += bz * M * N;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += 16) {
    for (int t = threadIdx.x; t < 64 * 16; t += 256) {
      const int kk = t & 15, r = t >> 4;
      const int m = m0 + r, n = n0 + r, k = k0 + kk;
      As[kk][r] = (m < M && k < K) ? Vec<Tin>::load1(A + (int64_t)m * K + k) : 0.f;
      Bs[kk][r] = (n < N && k < K)
                      ? Vec<Tin>::load1(transpose_b ? B + (int64_t)n * K + k : B + (int64_t)k * N + n)
                      : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float av[4], bv[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { av[i] = As[kk][ty * 4 + i]; bv[i] = Bs[kk][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += av[i] * bv[j];
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
      if (m < M && n < N) Vec<Tout>::store1(C + (int64_t)m * N + n, acc[i][j]);
    }
}

// ------------------------------------------------------------------------------------
// host
// ------------------------------------------------------------------------------------
int64_t align256(int64_t v) { return (v + 255) / 256 * 256; }
int64_t bytes_of(const Node& n) { return n.numel() * (n.dtype == FS_F32 ? 4 : 2); }

bool materialised(const Node& n) {
  return n.kind != FS_PARAMETER && n.kind != FS_CONSTANT && n.kind != FS_BROADCAST && n.kind != FS_OUTPUT;
}

bool view_vector_ok(const PerOpView& v, const Node& res) {
  if (v.base < 0 || v.full) return true;
  const int64_t last = v.stride[res.rank - 1];
  if (last != 0 && last != 1) return false;
  for (int d = 0; d + 1 < res.rank; ++d) if (last == 1 && v.stride[d] % 8 != 0) return false;
  return true;
}

template <typename Tin, typename Tout>
hipError_t launch_ew(const EwArgs& a, bool vec, hipStream_t s) {
  const int64_t work = vec ? a.n / 8 : a.n;
  int64_t grid = (work + 255) / 256;
  if (grid > 65536) grid = 65536;
  if (vec) hipLaunchKernelGGL((ew_vec_kernel<Tin, Tout>), dim3((unsigned)grid), dim3(256), 0, s, a);
  else hipLaunchKernelGGL((ew_scalar_kernel<Tin, Tout>), dim3((unsigned)grid), dim3(256), 0, s, a);
  return hipGetLastError();
}

template <typename Tin>
hipError_t launch_ew_out(const EwArgs& a, int out_dt, bool vec, hipStream_t s) {
  switch (out_dt) {
    case FS_F32: return launch_ew<Tin, float>(a, vec, s);
    case FS_F16: return launch_ew<Tin, f16_t>(a, vec, s);
    default: return launch_ew<Tin, bf16_t>(a, vec, s);
  }
}

hipError_t launch_ew_any(const EwArgs& a, int in_dt, int out_dt, bool vec, hipStream_t s) {
  switch (in_dt) {
    case FS_F32: return launch_ew_out<float>(a, out_dt, vec, s);
    case FS_F16: return launch_ew_out<f16_t>(a, out_dt, vec, s);
    default: return launch_ew_out<bf16_t>(a, out_dt, vec, s);
  }
}

template <typename T>
hipError_t launch_reduce(const PerOpStep& st, const void* in, void* out, double* scratch, int chunks, bool is_max,
                         hipStream_t s) {
  if (st.inner == 1) {
    const int64_t grid = (st.outer + 3) / 4;
    hipLaunchKernelGGL((row_reduce_kernel<T>), dim3((unsigned)grid), dim3(256), 0, s, static_cast<const T*>(in),
                       static_cast<T*>(out), st.outer, st.red, is_max ? 1 : 0, st.vector_ok ? 1 : 0);
    return hipGetLastError();
  }
  const unsigned gx = (unsigned)((st.inner + 255) / 256);
  hipLaunchKernelGGL((col_reduce_stage1<T>), dim3(gx, chunks, (unsigned)st.outer), dim3(256), 0, s,
                     static_cast<const T*>(in), scratch, st.red, st.inner, chunks, is_max ? 1 : 0);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((col_reduce_stage2<T>), dim3(gx, (unsigned)st.outer), dim3(256), 0, s, scratch,
                     static_cast<T*>(out), st.inner, chunks, is_max ? 1 : 0);
  return hipGetLastError();
}

template <typename Tin, typename Tout>
hipError_t launch_dot_t(const void* A, const void* B, void* C, int batch, int M, int N, int K, int tb, hipStream_t s) {
  hipLaunchKernelGGL((dot_kernel<Tin, Tout>), dim3((N + 63) / 64, (M + 63) / 64, batch), dim3(256), 0, s,
                     static_cast<const Tin*>(A), static_cast<const Tin*>(B), static_cast<Tout*>(C), M, N, K, tb);
  return hipGetLastError();
}

template <typename Tin>
hipError_t launch_dot_out(int out_dt, const void* A, const void* B, void* C, int batch, int M, int N, int K, int tb,
                          hipStream_t s) {
  switch (out_dt) {
    case FS_F32: return launch_dot_t<Tin, float>(A, B, C, batch, M, N, K, tb, s);
    case FS_F16: return launch_dot_t<Tin, f16_t>(A, B, C, batch, M, N, K, tb, s);
    default: return launch_dot_t<Tin, bf16_t>(A, B, C, batch, M, N, K, tb, s);
  }
}

int col_chunks(const PerOpStep& st) {
  // enough workgroups to fill the chip: about 1024 in total
  const int64_t gx = (st.inner + 255) / 256;
  int64_t chunks = 1024 / (gx * st.outer);
  if (chunks < 1) chunks = 1;
  if (chunks > st.red) chunks = st.red > 0 ? st.red : 1;
  if (chunks > 256) chunks = 256;
  return (int)chunks;
}

}  // namespace

bool per_op_plan(const Graph& g, PerOpPlan* plan, std::string* err) {
  PerOpPlan p;
  const int n = g.size();
  p.offset.assign(n, -1);
  p.out_of.assign(n, -1);
  // a materialised op that feeds an output writes straight into the output buffer
  for (int o : g.outputs) {
    const int src = g[o].operand[0];
    if (materialised(g[src])) p.out_of[src] = g[o].ordinal;
  }
  int64_t ws = 0;
  for (int i = 0; i < n; ++i) {
    const Node& x = g[i];
    if (x.kind == FS_OUTPUT) {
      if (materialised(g[x.operand[0]])) continue;
      // output of a parameter or of a broadcast view: one copy kernel
      PerOpStep st;
      st.node = i; st.kind = FS_OUTPUT;
      st.a = view_of(g, x.operand[0]);
      st.vector_ok = x.numel() % 8 == 0 && x.rank >= 1 && x.shape[x.rank - 1] % 8 == 0 && view_vector_ok(st.a, x);
      p.steps.push_back(st);
      p.n_kernels += 1;
      p.moved_bytes += bytes_of(g[st.a.base]) + bytes_of(x);
      continue;
    }
    if (!materialised(x)) continue;
    if (p.out_of[i] < 0) { p.offset[i] = ws; ws += align256(bytes_of(x)); }
    PerOpStep st;
    st.node = i; st.kind = x.kind;
    if (x.numel() >= ((int64_t)1 << 31) * 8) { *err = "per-op baseline: tensor too large"; return false; }
    if (is_binary(x.kind) || is_unary(x.kind) || x.kind == FS_CONVERT || x.kind == FS_CAUSAL_MASK) {
      st.a = view_of(g, x.operand[0]);
      if (is_binary(x.kind)) st.b = view_of(g, x.operand[1]);
      st.vector_ok = x.rank >= 1 && x.numel() % 8 == 0 && x.shape[x.rank - 1] % 8 == 0 &&
                     view_vector_ok(st.a, x) && (!is_binary(x.kind) || view_vector_ok(st.b, x));
      p.moved_bytes += bytes_of(x);
      if (st.a.base >= 0) p.moved_bytes += bytes_of(g[st.a.base]);
      if (is_binary(x.kind) && st.b.base >= 0) p.moved_bytes += bytes_of(g[st.b.base]);
    } else if (x.kind == FS_REDUCE_SUM || x.kind == FS_REDUCE_MAX) {
      const Node& a = g[x.operand[0]];
      st.a = view_of(g, x.operand[0]);
      if (!st.a.full) { *err = "per-op baseline: reduce of a broadcast view"; return false; }
      st.outer = 1; st.inner = 1;
      for (int d = 0; d < x.axis; ++d) st.outer *= a.shape[d];
      for (int d = x.axis + 1; d < a.rank; ++d) st.inner *= a.shape[d];
      st.red = a.shape[x.axis];
      st.vector_ok = st.inner == 1 && st.red % 8 == 0;
      if (st.inner > 1) {
        st.launches = 2;
        const int64_t need = 8 * st.outer * (int64_t)col_chunks(st) * st.inner;
        if (need > p.scratch_bytes) p.scratch_bytes = need;
        p.moved_bytes += 2 * need;
      }
      if (st.outer > 0x7fffffff / 4 || (st.inner > 1 && st.outer > 65535)) { *err = "per-op baseline: reduce too large"; return false; }
      p.moved_bytes += bytes_of(a) + bytes_of(x);
    } else if (x.kind == FS_DOT) {
      st.a = view_of(g, x.operand[0]);
      st.b = view_of(g, x.operand[1]);
      if (!st.a.full || !st.b.full) { *err = "per-op baseline: dot of a broadcast view"; return false; }
      if (x.shape[0] > 65535) { *err = "per-op baseline: dot batch > 65535"; return false; }
      p.moved_bytes += bytes_of(g[x.operand[0]]) + bytes_of(g[x.operand[1]]) + bytes_of(x);
    } else {
      *err = std::string("per-op baseline: no kernel for op ") + kind_name(x.kind);
      return false;
    }
    p.n_kernels += st.launches;
    p.steps.push_back(st);
  }
  p.scratch_offset = ws;
  ws += align256(p.scratch_bytes);
  p.workspace_bytes = ws;
  *plan = p;
  return true;
}

std::string per_op_describe(const PerOpPlan& plan) {
  char buf[160];
  snprintf(buf, sizeof buf, "per-op baseline: %d kernels, %lld bytes of HBM workspace", plan.n_kernels,
           (long long)plan.workspace_bytes);
  return buf;
}

__global__ __launch_bounds__(256) void zero_bytes_kernel(unsigned char* p, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

int per_op_launch(const Graph& g, const PerOpPlan& plan, const void* const* in, void* const* out, void* workspace,
                  void* stream, std::string* err) {
  hipStream_t s = static_cast<hipStream_t>(stream);
  char* ws = static_cast<char*>(workspace);
  auto addr = [&](int node) -> const void* {
    const Node& x = g[node];
    if (x.kind == FS_PARAMETER) return in[x.ordinal];
    if (plan.out_of[node] >= 0) return out[plan.out_of[node]];
    return ws + plan.offset[node];
  };
  auto operand = [&](const PerOpView& v, EwOperand* o) {
    o->is_const = v.base < 0; o->cval = v.cval; o->full = v.full ? 1 : 0;
    o->p = v.base >= 0 ? addr(v.base) : nullptr;
    for (int d = 0; d < FS_MAX_RANK; ++d) o->s[d] = v.stride[d];
  };
  for (const PerOpStep& st : plan.steps) {
    const Node& x = g[st.node];
    if (x.numel() == 0) continue;
    hipError_t e = hipSuccess;
    if (st.kind == FS_REDUCE_SUM || st.kind == FS_REDUCE_MAX) {
      const bool is_max = st.kind == FS_REDUCE_MAX;
      const void* src = addr(st.a.base);
      void* dst = const_cast<void*>(addr(st.node));
      double* scratch = reinterpret_cast<double*>(ws + plan.scratch_offset);
      if (st.red == 0) {
        // nothing to reduce: zeros, written by a kernel (a memset node recorded into a captured graph is avoided)
        const int64_t nbytes = x.numel() * (x.dtype == FS_F32 ? 4 : 2);
        hipLaunchKernelGGL(zero_bytes_kernel, dim3((unsigned)((nbytes + 255) / 256)), dim3(256), 0, s, static_cast<unsigned char*>(dst), nbytes);
        e = hipGetLastError();
      }
      else {
        const int chunks = col_chunks(st);
        switch (x.dtype) {
          case FS_F32: e = launch_reduce<float>(st, src, dst, scratch, chunks, is_max, s); break;
          case FS_F16: e = launch_reduce<f16_t>(st, src, dst, scratch, chunks, is_max, s); break;
          default: e = launch_reduce<bf16_t>(st, src, dst, scratch, chunks, is_max, s); break;
        }
      }
    } else if (st.kind == FS_DOT) {
      const Node& a = g[x.operand[0]];
      const int M = (int)x.shape[1], N = (int)x.shape[2], K = (int)a.shape[2];
      const void* A = addr(st.a.base); const void* B = addr(st.b.base);
      void* C = const_cast<void*>(addr(st.node));
      switch (a.dtype) {
        case FS_F32: e = launch_dot_out<float>(x.dtype, A, B, C, (int)x.shape[0], M, N, K, x.axis, s); break;
        case FS_F16: e = launch_dot_out<f16_t>(x.dtype, A, B, C, (int)x.shape[0], M, N, K, x.axis, s); break;
        default: e = launch_dot_out<bf16_t>(x.dtype, A, B, C, (int)x.shape[0], M, N, K, x.axis, s); break;
      }
    } else {
      EwArgs a{};
      operand(st.a, &a.a);
      operand(st.b, &a.b);
      a.out = st.kind == FS_OUTPUT ? out[x.ordinal] : const_cast<void*>(addr(st.node));
      a.n = x.numel(); a.kind = st.kind; a.rank = x.rank; a.attr = (float)x.attr;
      for (int d = 0; d < FS_MAX_RANK; ++d) a.shape[d] = d < x.rank ? x.shape[d] : 1;
      const int in_dt = st.a.base >= 0 ? g[st.a.base].dtype : (st.b.base >= 0 ? g[st.b.base].dtype : x.dtype);
      e = launch_ew_any(a, in_dt, x.dtype, st.vector_ok, s);
    }
    if (e != hipSuccess) {
      *err = std::string("per-op baseline, op ") + std::to_string(st.node) + " (" + kind_name(st.kind) + "): " + hipGetErrorString(e);
      return -1;
    }
  }
  return 0;
}

}  // namespace fs
