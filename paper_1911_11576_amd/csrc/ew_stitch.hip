// Schedule 0, generic elementwise stitching (paper Section 5.1: thread composition of
// data-dependent elementwise ops, and kernel packing of independent ones, merged into one
// loop): ANY group made only of elementwise ops, converts, broadcasts and constants, with
// up to 8 outputs, runs as one kernel that reads every parameter once and writes every
// output once.
//
// This file holds the analysis of such a group (resolved ops, operand views), the plan and
// launch steps, and the form that needs no compiler at run time: the group compiled into a
// short register program (load, ALU op, store; at most 64 steps) that an interpreter kernel
// executes.  The program counter is uniform across the chip, so each step is a scalar
// branch tree.  Values used by the next step stay in a VGPR accumulator; values with a later
// use live in a per-thread LDS slot (a register file of float4 slots, slot-major so that a
// wavefront's access is conflict-free), reused by liveness.  RegisterPlanning in the
// paper's sense falls out: an op with several consumers is computed once.
// The default form, a kernel generated for the group, is in ew_codegen.cpp.
#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <functional>
#include <memory>
#include <vector>

#include "dev_common.h"
#include "ew_ir.h"
#include "match.h"
#include "launchers.h"
#include "per_op.h"
#include "../../include/fs.h"

namespace fs {

enum EwKind : uint8_t { EW_LOAD = 0, EW_ALU = 1, EW_STORE = 2 };
enum : uint8_t { EW_ACC = 255 };                 // operand code: the accumulator
enum : uint8_t { EW_ROUND_F16 = 100, EW_ROUND_BF16 = 101 };
enum : uint8_t { EW_A_IMM = 1, EW_B_IMM = 2, EW_KEEP = 4 };

struct EwInstr {
  uint8_t kind, op, dst, a, b, flags, dtype, pad;
  int32_t arg;      // LOAD: view index; STORE: output index
  float imm;
};
struct EwView {
  const void* p;
  int64_t s[FS_MAX_RANK];
  int32_t full, pad;
};
static constexpr int kEwMaxInstr = 64, kEwMaxViews = 12, kEwMaxOuts = 8;

// What the kernel reads: one field per dword (a scalar load hands each to a register of its
// own, nothing to unpack), operands as ready-made LDS indices (-1: the accumulator).
struct EwStep {
  int32_t kind, op, a, b, dst, flags, arg;   // flags: EW_KEEP | storage dtype << 8
  float imm;
};

struct EwProgram {
  EwStep ins[kEwMaxInstr];
  EwView views[kEwMaxViews];
  void* outs[kEwMaxOuts];
  int64_t shape[FS_MAX_RANK];
  int64_t n;
  int32_t n_ins, rank, need_idx, pad;
};

// N floats held as one SSA vector: static element indices only, so it never leaves registers
template <int N> using ew_vec = float __attribute__((ext_vector_type(N)));

// One ALU step on all N elements a thread carries.  The first operand is always the
// accumulator and the result replaces it (the plan normalises every op to that form: a slot
// operand is first loaded into the accumulator, swapped operands become the reversed ops).
// The dispatch on `op` is uniform and sits outside the element loop: a step costs one scalar
// branch tree however many elements it covers.
enum : int { EW_RSUB = 102, EW_RDIV = 103 };   // y - x, y / x
enum : int { EW_B_SELF = 0, EW_B_SLOT = 1, EW_B_IMM_MODE = 2 };

#define EW_FOR_ALL(expr)                          \
  _Pragma("unroll") for (int i = 0; i < N; ++i) { \
    const float p = acc[i], q = EW_Q;             \
    (void)q;                                      \
    acc[i] = (expr);                              \
  }
#define EW_BINARY_CASES                              \
  case FS_ADD: EW_FOR_ALL(p + q) break;              \
  case FS_SUBTRACT: EW_FOR_ALL(p - q) break;         \
  case EW_RSUB: EW_FOR_ALL(q - p) break;             \
  case FS_MULTIPLY: EW_FOR_ALL(p * q) break;         \
  case FS_DIVIDE: EW_FOR_ALL(p / q) break;           \
  case EW_RDIV: EW_FOR_ALL(q / p) break;             \
  case FS_MAXIMUM: EW_FOR_ALL(fmaxf(p, q)) break;

// second operand in registers
template <int N>
__device__ __forceinline__ void ew_alu_vec(int op, ew_vec<N>& acc, const ew_vec<N> y) {
#define EW_Q y[i]
  switch (op) { EW_BINARY_CASES default: break; }
#undef EW_Q
}
// second operand a constant of the group: it stays in a scalar register
template <int N>
__device__ __forceinline__ void ew_alu_imm(int op, ew_vec<N>& acc, const float imm) {
#define EW_Q imm
  switch (op) { EW_BINARY_CASES default: break; }
#undef EW_Q
}
// unary ops, and binary ops whose two operands are the same value
template <int N>
__device__ __forceinline__ void ew_alu_self(int op, ew_vec<N>& acc) {
#define EW_Q p
  switch (op) {
    case FS_ADD: EW_FOR_ALL(p + q) break;
    case FS_SUBTRACT: EW_FOR_ALL(p - q) break;
    case FS_MULTIPLY: EW_FOR_ALL(p * q) break;
    case FS_DIVIDE: EW_FOR_ALL(p / q) break;
    case FS_NEGATE: EW_FOR_ALL(-p) break;
    case FS_EXP: EW_FOR_ALL(expf(p)) break;
    case FS_LOG: EW_FOR_ALL(logf(p)) break;
    case FS_TANH: EW_FOR_ALL(tanhf(p)) break;
    case FS_RSQRT: EW_FOR_ALL(1.f / sqrtf(p)) break;
    case FS_SQRT: EW_FOR_ALL(sqrtf(p)) break;
    case FS_ERF: EW_FOR_ALL(erff(p)) break;
    case FS_LOGISTIC: EW_FOR_ALL(1.f / (1.f + expf(-p))) break;
    case EW_ROUND_F16: EW_FOR_ALL(f16_to_f32(f32_to_f16(p))) break;
    case EW_ROUND_BF16: EW_FOR_ALL(bf16_to_f32(f32_to_bf16(p))) break;
    default: break;              // maximum(x, x) = x
  }
#undef EW_Q
}
#undef EW_BINARY_CASES
#undef EW_FOR_ALL

template <typename T> __device__ __forceinline__ f32x4 ew_load4(const T* p);
template <> __device__ __forceinline__ f32x4 ew_load4<float>(const float* p) {
  const u32x4 t = stream_load16(p);
  return f32x4{as_f32(t[0]), as_f32(t[1]), as_f32(t[2]), as_f32(t[3])};
}
template <> __device__ __forceinline__ f32x4 ew_load4<bf16_t>(const bf16_t* p) {
  const u32x2 t = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(p));
  return f32x4{as_f32(t[0] << 16), as_f32(t[0] & 0xFFFF0000u), as_f32(t[1] << 16), as_f32(t[1] & 0xFFFF0000u)};
}
template <> __device__ __forceinline__ f32x4 ew_load4<f16_t>(const f16_t* p) {
  const u32x2 t = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(p));
  return f32x4{f16_to_f32(t[0] & 0xFFFFu), f16_to_f32(t[0] >> 16), f16_to_f32(t[1] & 0xFFFFu), f16_to_f32(t[1] >> 16)};
}

__device__ __forceinline__ float ew_load1(const void* p, int64_t off, int dtype) {
  if (dtype == DT_F32) return static_cast<const float*>(p)[off];
  if (dtype == DT_F16) return f16_to_f32(static_cast<const uint16_t*>(p)[off]);
  return bf16_to_f32(static_cast<const uint16_t*>(p)[off]);
}

// VEC: a chunk is 4 consecutive elements (last extent a multiple of 4, operand rows
// 4-aligned); otherwise a chunk is one element.  Every thread carries U chunks through the
// program in lock step (chunk u of thread t is element block base + u*blockDim + t, so each
// access of a wavefront is one contiguous run), which spreads the cost of fetching and
// decoding a program step over 4U elements per thread.
template <bool VEC, int U>
__global__ __launch_bounds__(256) void ew_stitch_kernel(const EwProgram prog) {
  extern __shared__ f32x4 slot_file[];          // [slot][U][blockDim.x]
  // The program is read from LDS: a step is one broadcast read plus lane-0 extracts.  (Read
  // step by step from the kernel-argument segment, every step costs a scalar-memory round
  // trip that the few resident wavefronts cannot hide.)
  __shared__ uint32_t step_lds[kEwMaxInstr * 8];
  const int nt = blockDim.x;
  {
    const uint32_t* src = reinterpret_cast<const uint32_t*>(prog.ins);
    for (int i = threadIdx.x; i < prog.n_ins * 8; i += nt) step_lds[i] = src[i];
    __syncthreads();
  }
  f32x4* mine = slot_file + threadIdx.x;
  constexpr int W = VEC ? 4 : 1;
  const int64_t nchunk = prog.n / W;
  const int64_t per_wg = (int64_t)nt * U;
  for (int64_t base = (int64_t)blockIdx.x * per_wg; base < nchunk; base += (int64_t)gridDim.x * per_wg) {
    int64_t e0[U];
    bool live[U];
    uint32_t idx[U][FS_MAX_RANK];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t ci = base + (int64_t)u * nt + threadIdx.x;
      live[u] = ci < nchunk;
      e0[u] = (live[u] ? ci : nchunk - 1) * W;   // dead chunks recompute the last one and store nothing
#pragma unroll
      for (int d = 0; d < FS_MAX_RANK; ++d) idx[u][d] = 0;
      if (prog.need_idx) {
        // dims are right-aligned in shape[] (leading extents 1), so the loop is static
        if (prog.n <= 0x7fffffff) {
          uint32_t e = (uint32_t)e0[u];
#pragma unroll
          for (int d = FS_MAX_RANK - 1; d >= 0; --d) {
            const uint32_t ext = (uint32_t)prog.shape[d];
            if (ext == 1) continue;
            const uint32_t q = e / ext;
            idx[u][d] = e - q * ext;
            e = q;
          }
        } else {
          int64_t e = e0[u];
#pragma unroll
          for (int d = FS_MAX_RANK - 1; d >= 0; --d) {
            const int64_t ext = prog.shape[d];
            if (ext == 1) continue;
            const int64_t q = e / ext;
            idx[u][d] = (uint32_t)(e - q * ext);
            e = q;
          }
        }
      }
    }
    constexpr int N = U * W;
    ew_vec<N> acc;
#pragma unroll
    for (int i = 0; i < N; ++i) acc[i] = 0.f;
    for (int pc = 0; pc < prog.n_ins; ++pc) {
      EwStep in;                                 // uniform: scalar registers and branches
      {
        const u32x4 lo = *reinterpret_cast<const u32x4*>(&step_lds[pc * 8]);
        const u32x4 hi = *reinterpret_cast<const u32x4*>(&step_lds[pc * 8 + 4]);
        in.kind = __builtin_amdgcn_readfirstlane(lo[0]);
        in.op = __builtin_amdgcn_readfirstlane(lo[1]);
        in.a = __builtin_amdgcn_readfirstlane(lo[2]);
        in.b = __builtin_amdgcn_readfirstlane(lo[3]);
        in.dst = __builtin_amdgcn_readfirstlane(hi[0]);
        in.flags = __builtin_amdgcn_readfirstlane(hi[1]);
        in.arg = __builtin_amdgcn_readfirstlane(hi[2]);
        in.imm = as_f32(__builtin_amdgcn_readfirstlane(hi[3]));
      }
      const int dtype = (in.flags >> 8) & 3;
      if (in.kind == EW_LOAD) {
        const EwView& v = prog.views[in.arg];
        const bool splat = !v.full && v.s[FS_MAX_RANK - 1] == 0;
#pragma unroll
        for (int u = 0; u < U; ++u) {
          int64_t off = e0[u];
          if (!v.full) {
            off = 0;
#pragma unroll
            for (int d = 0; d < FS_MAX_RANK; ++d) off += (int64_t)idx[u][d] * v.s[d];
          }
          f32x4 t;
          if (!VEC || splat) {
            const float t1 = ew_load1(v.p, off, dtype);
            t = f32x4{t1, t1, t1, t1};
          } else if (dtype == DT_F32) t = ew_load4<float>(static_cast<const float*>(v.p) + off);
          else if (dtype == DT_F16) t = ew_load4<f16_t>(static_cast<const f16_t*>(v.p) + off);
          else t = ew_load4<bf16_t>(static_cast<const bf16_t*>(v.p) + off);
#pragma unroll
          for (int j = 0; j < W; ++j) acc[u * W + j] = t[j];
        }
      } else if (in.kind == EW_ALU) {
        if (in.a >= 0) {                           // first operand from a slot: straight into the accumulator
#pragma unroll
          for (int u = 0; u < U; ++u) {
            const f32x4 t = mine[in.a + u * nt];
#pragma unroll
            for (int j = 0; j < W; ++j) acc[u * W + j] = t[j];
          }
        }
        if (in.b == EW_B_IMM_MODE) {
          ew_alu_imm<N>(in.op, acc, in.imm);
        } else if (in.b == EW_B_SLOT) {
          ew_vec<N> y;
#pragma unroll
          for (int u = 0; u < U; ++u) {
            const f32x4 t = mine[in.arg + u * nt];
#pragma unroll
            for (int j = 0; j < W; ++j) y[u * W + j] = t[j];
          }
          ew_alu_vec<N>(in.op, acc, y);
        } else {
          ew_alu_self<N>(in.op, acc);
        }
      } else {
        void* o = prog.outs[in.arg];
        ew_vec<N> x = acc;
        if (in.a >= 0) {
#pragma unroll
          for (int u = 0; u < U; ++u) {
            const f32x4 t = mine[in.a + u * nt];
#pragma unroll
            for (int j = 0; j < W; ++j) x[u * W + j] = t[j];
          }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
          if (!live[u]) continue;
          if (VEC) {
            const int b = u * W;
            if (dtype == DT_F32) {
              stream_store16(static_cast<float*>(o) + e0[u],
                             u32x4{as_u32(x[b]), as_u32(x[b + 1]), as_u32(x[b + 2]), as_u32(x[b + 3])});
            } else {
              u32x2 t;
              if (dtype == DT_F16) { t[0] = pack2_f16(x[b], x[b + 1]); t[1] = pack2_f16(x[b + 2], x[b + 3]); }
              else { t[0] = pack2_bf16(x[b], x[b + 1]); t[1] = pack2_bf16(x[b + 2], x[b + 3]); }
              __builtin_nontemporal_store(t, reinterpret_cast<u32x2*>(static_cast<uint16_t*>(o) + e0[u]));
            }
          } else if (dtype == DT_F32) static_cast<float*>(o)[e0[u]] = x[u];
          else static_cast<uint16_t*>(o)[e0[u]] = (uint16_t)(dtype == DT_F16 ? f32_to_f16(x[u]) : f32_to_bf16(x[u]));
        }
        continue;
      }
      if (in.flags & EW_KEEP) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
          f32x4 t = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int j = 0; j < W; ++j) t[j] = acc[u * W + j];
          mine[in.dst + u * nt] = t;
        }
      }
    }
  }
}

// ----------------------------------------------------------------------------------------
// host: compile the group into a program
// ----------------------------------------------------------------------------------------
struct EwCompiled {
  EwProgram prog{};
  EwInstr code[kEwMaxInstr];     // compact form written by the compiler; expanded into prog.ins
  int view_param[kEwMaxViews];   // parameter ordinal of each view
  int n_views = 0;
};

static bool ew_is_elementwise(int k) { return is_binary(k) || is_unary(k) || k == FS_CONVERT || k == FS_CAUSAL_MASK; }

namespace {

// Compiler state for one group.
struct EwCompiler {
  const Graph& g;
  EwCompiled c;
  EwIr ir;
  std::string err;
  int S = -1;                       // node that fixes the iteration shape
  bool vec = true;
  std::vector<int> order;           // compute nodes (elementwise ops that are not aliases), in list order
  std::vector<int> last_use;        // per node: index into `order` of the last op reading it
  std::vector<int> slot_of;
  std::vector<int> out_ord, out_dtype;
  std::vector<int> free_slots;
  int n_slots = 0;
  int acc_holds = -1;
  std::vector<char> active;         // if not empty: the compute ops this compiler looks at (one part of a packed group)

  explicit EwCompiler(const Graph& gr) : g(gr) {}

  // a convert to f32 changes nothing in registers (all arithmetic is fp32): alias of its operand
  int canon(int n) const {
    while (g[n].kind == FS_CONVERT && g[n].dtype == FS_F32) n = g[n].operand[0];
    return n;
  }
  bool is_compute(int n) const { return ew_is_elementwise(g[n].kind) && canon(n) == n; }
  int n_operands(int n) const { return is_binary(g[n].kind) ? 2 : 1; }

  bool fail(const std::string& m) { err = m; return false; }

  bool emit(const EwInstr& in) {
    if (c.prog.n_ins == kEwMaxInstr) return fail("elementwise schedule: program longer than 64 instructions");
    c.code[c.prog.n_ins++] = in;
    return true;
  }
  int take_slot() {
    if (!free_slots.empty()) { const int s = free_slots.back(); free_slots.pop_back(); return s; }
    return n_slots++;
  }

  // like view_of, but widening converts are looked through (they cost nothing here)
  PerOpView resolve(int n) const {
    n = canon(n);
    const Node& x = g[n];
    PerOpView v;
    if (x.kind == FS_CONSTANT) { v.base = -1; v.cval = (float)x.attr; v.full = false; return v; }
    if (x.kind == FS_BROADCAST) {
      const PerOpView o = resolve(x.operand[0]);
      const Node& a = g[x.operand[0]];
      v.base = o.base; v.full = false;
      for (int d = 0; d < a.rank; ++d) v.stride[x.axis + d] = a.shape[d] == 1 ? 0 : o.stride[d];
      return v;
    }
    v.base = n; v.full = true;
    int64_t st = 1;
    for (int d = x.rank - 1; d >= 0; --d) { v.stride[d] = st; st *= x.shape[d]; }
    return v;
  }

  // leaf -> view index (-1: constant, value in *cval); false if not expressible
  bool leaf(int node, int* view, bool* is_const, float* cval) {
    const PerOpView pv = resolve(node);
    *is_const = pv.base < 0;
    if (*is_const) { *cval = pv.cval; return true; }
    if (g[pv.base].kind != FS_PARAMETER) return fail("elementwise schedule: broadcast of a computed value");
    EwProgram& P = c.prog;
    const Node& shape = g[S];
    for (int k = 0; k < c.n_views; ++k) {
      bool same = c.view_param[k] == g[pv.base].ordinal && (P.views[k].full != 0) == pv.full;
      for (int d = 0; d < shape.rank && same && !pv.full; ++d)
        same = P.views[k].s[d + FS_MAX_RANK - shape.rank] == pv.stride[d];
      if (same) { *view = k; return true; }
    }
    if (c.n_views == kEwMaxViews) return fail("elementwise schedule: more than 12 distinct operand views");
    EwView& ev = P.views[c.n_views];
    ev.full = pv.full ? 1 : 0;
    // the kernel sees the dims right-aligned in its 4 slots (leading extents 1)
    const int shift = FS_MAX_RANK - shape.rank;
    for (int d = 0; d < FS_MAX_RANK; ++d) ev.s[d] = d >= shift ? pv.stride[d - shift] : 0;
    if (pv.full) {
      if (!g[pv.base].same_shape(shape)) return fail("elementwise schedule: parameter shape differs from the group's");
    } else {
      P.need_idx = 1;
      const int64_t last = shape.rank > 0 ? pv.stride[shape.rank - 1] : 0;
      if (last != 0 && last != 1) vec = false;
      for (int d = 0; d + 1 < shape.rank; ++d) if (last == 1 && pv.stride[d] % 4 != 0) vec = false;
    }
    c.view_param[c.n_views] = g[pv.base].ordinal;
    EwIrView iv;
    iv.param = g[pv.base].ordinal;
    iv.dtype = g[pv.base].dtype;
    iv.full = pv.full;
    for (int d = 0; d < FS_MAX_RANK; ++d) iv.stride[d] = ev.s[d];
    ir.views.push_back(iv);
    *view = c.n_views++;
    return true;
  }

  // shape checks, outputs, and the group as a list of resolved ops
  bool analyse() {
    const int n = g.size();
    for (int i = 0; i < n; ++i) {
      const Node& x = g[i];
      if (ew_is_elementwise(x.kind)) {
        if (!is_compute(i)) continue;            // a widening convert: an alias of its operand
        if (!active.empty() && !active[i]) continue;
        if (S < 0) S = i;
        else if (!x.same_shape(g[S])) return fail("elementwise schedule: ops of different shapes in one group");
        order.push_back(i);
      } else if (x.kind != FS_PARAMETER && x.kind != FS_CONSTANT && x.kind != FS_BROADCAST && x.kind != FS_OUTPUT) {
        return fail(std::string("no stitched schedule matches this group (op ") + kind_name(x.kind) +
                    " outside the recognised patterns)");
      }
    }
    if (S < 0 || order.empty()) return fail("elementwise schedule: the group computes nothing");
    if (active.empty() && (int)g.outputs.size() > kEwMaxOuts) return fail("elementwise schedule: more than 8 outputs");
    EwProgram& P = c.prog;
    // a group of scalars (rank 0: arithmetic on fully reduced values) runs as a group of shape [1]
    P.rank = g[S].rank < 1 ? 1 : g[S].rank;
    P.n = g[S].numel();
    for (int d = 0; d < FS_MAX_RANK; ++d) {
      const int src = d - (FS_MAX_RANK - g[S].rank);
      P.shape[d] = src >= 0 ? g[S].shape[src] : 1;
    }
    vec = g[S].rank >= 1 && g[S].shape[g[S].rank - 1] % 4 == 0;

    last_use.assign(n, -1);
    slot_of.assign(n, -1);
    out_ord.assign(n, -1);
    out_dtype.assign(n, 0);
    for (size_t k = 0; k < order.size(); ++k)
      for (int j = 0; j < n_operands(order[k]); ++j) {
        const int a = canon(g[order[k]].operand[j]);
        if (is_compute(a)) last_use[a] = (int)k;
      }
    int n_my_outputs = 0;
    for (int o : g.outputs) {
      const int src = canon(g[o].operand[0]);
      if (!is_compute(src)) return fail("elementwise schedule: an output that is a plain copy of an input");
      if (!active.empty() && !active[src]) continue;
      ++n_my_outputs;
      if (out_ord[src] >= 0) return fail("elementwise schedule: one value feeds two outputs");
      out_ord[src] = g[o].ordinal;
      out_dtype[src] = g[o].dtype;
    }

    ir.rank = P.rank;
    ir.n = P.n;
    ir.n_outputs = n_my_outputs;
    if (n_my_outputs == 0) return fail("elementwise schedule: ops that reach no output");
    for (int d = 0; d < FS_MAX_RANK; ++d) ir.shape[d] = P.shape[d];
    // the tanh-form GELU is generated as one op (the interpreter's program keeps the ops spelled out)
    std::vector<int> idiom_of(n, -1);
    std::vector<char> inside_idiom(n, 0);
    const std::vector<GeluIdiom> idioms = find_gelu_idioms(g);
    for (size_t q = 0; q < idioms.size(); ++q) {
      bool plain = true;   // an interior value that is a group output keeps the ops spelled out
      for (int v : idioms[q].interior) if (out_ord[v] >= 0) plain = false;
      if (!plain) continue;
      idiom_of[idioms[q].out] = (int)q;
      for (int v : idioms[q].interior) inside_idiom[v] = 1;
    }
    for (int node : order) {
      const Node& x = g[node];
      if (inside_idiom[node]) continue;
      EwIrNode in;
      in.id = node;
      in.op = x.kind == FS_CONVERT ? (x.dtype == FS_F16 ? (int)EW_OP_ROUND_F16 : (int)EW_OP_ROUND_BF16) : x.kind;
      in.n_operands = n_operands(node);
      if (idiom_of[node] >= 0) {
        const GeluIdiom& id = idioms[idiom_of[node]];
        in.op = EW_OP_GELU_TANH;
        in.n_operands = 1;
        gelu_constants(id, in.gelu);
        const int a = canon(id.h);
        if (is_compute(a)) { in.opnd[0].kind = EW_FROM_NODE; in.opnd[0].index = a; }
        else {
          bool is_const = false;
          if (!leaf(a, &in.opnd[0].index, &is_const, &in.opnd[0].cval)) return false;
          in.opnd[0].kind = is_const ? EW_FROM_CONST : EW_FROM_VIEW;
        }
        in.out_ordinal = out_ord[node];
        in.out_dtype = out_dtype[node];
        ir.nodes.push_back(in);
        continue;
      }
      if (x.kind == FS_CAUSAL_MASK) {
        if (x.rank < 2) return fail("elementwise schedule: causal_mask below rank 2");
        in.opnd[1].cval = (float)x.attr;       // the fill value rides in the unused second operand
      }
      for (int j = 0; j < in.n_operands; ++j) {
        const int a = canon(x.operand[j]);
        if (is_compute(a)) { in.opnd[j].kind = EW_FROM_NODE; in.opnd[j].index = a; continue; }
        bool is_const = false;
        if (!leaf(a, &in.opnd[j].index, &is_const, &in.opnd[j].cval)) return false;
        in.opnd[j].kind = is_const ? EW_FROM_CONST : EW_FROM_VIEW;
      }
      if (in.n_operands == 2 && in.opnd[0].kind == EW_FROM_CONST && in.opnd[1].kind == EW_FROM_CONST)
        return fail("elementwise schedule: op of two constants");
      in.out_ordinal = out_ord[node];
      in.out_dtype = out_dtype[node];
      ir.nodes.push_back(in);
    }
    // a rounding read by nothing but the store of the same dtype is left to the store
    std::vector<char> read(g.size(), 0);
    for (const EwIrNode& r : ir.nodes)
      for (int j = 0; j < r.n_operands; ++j) if (r.opnd[j].kind == EW_FROM_NODE) read[r.opnd[j].index] = 1;
    for (EwIrNode& r : ir.nodes) {
      const bool rounds = (r.op == EW_OP_ROUND_F16 && r.out_dtype == FS_F16) || (r.op == EW_OP_ROUND_BF16 && r.out_dtype == FS_BF16);
      if (rounds && r.out_ordinal >= 0 && !read[r.id]) r.op = EW_OP_COPY;
    }
    return true;
  }

  // the register program for the interpreter kernel; false (with the reason in err) if the
  // group is too long or keeps too many values alive for it
  bool program() {
    for (size_t k = 0; k < order.size(); ++k) {
      const int node = order[k];
      const Node& x = g[node];
      if (x.kind == FS_CAUSAL_MASK) return fail("elementwise schedule: the interpreter has no causal_mask step");
      const int nop = n_operands(node);
      EwInstr alu{};
      alu.kind = EW_ALU;
      alu.op = x.kind == FS_CONVERT ? (x.dtype == FS_F16 ? (uint8_t)EW_ROUND_F16 : (uint8_t)EW_ROUND_BF16) : (uint8_t)x.kind;
      uint8_t opnd[2] = {EW_ACC, EW_ACC};
      bool temp_slot[2] = {false, false};
      int ops[2] = {canon(x.operand[0]), nop == 2 ? canon(x.operand[1]) : -1};
      // how many operands need a LOAD (non-constant leaves)
      int view[2] = {-1, -1};
      bool is_const[2] = {false, false};
      int n_loads = 0;
      for (int j = 0; j < nop; ++j) {
        if (is_compute(ops[j])) continue;
        float cv = 0.f;
        if (!leaf(ops[j], &view[j], &is_const[j], &cv)) return false;
        if (is_const[j]) { alu.flags |= j == 0 ? EW_A_IMM : EW_B_IMM; alu.imm = cv; }
        else ++n_loads;
      }
      if (is_const[0] && nop == 2 && is_const[1]) return fail("elementwise schedule: op of two constants");
      // loads: all but the last one go to a temporary slot, the last one stays in the accumulator
      int done = 0;
      for (int j = 0; j < nop; ++j) {
        if (is_compute(ops[j]) || is_const[j]) continue;
        if (nop == 2 && ops[0] == ops[1] && j == 1) { opnd[1] = opnd[0]; continue; }   // same leaf twice
        EwInstr ld{};
        ld.kind = EW_LOAD;
        ld.arg = view[j];
        ld.dtype = (uint8_t)g[resolve(ops[j]).base].dtype;
        ++done;
        const bool same_twice = nop == 2 && ops[0] == ops[1];
        if (done < n_loads && !same_twice) {
          ld.flags |= EW_KEEP;
          ld.dst = (uint8_t)take_slot();
          opnd[j] = ld.dst;
          temp_slot[j] = true;
        }
        if (!emit(ld)) return false;
        acc_holds = -2;   // a leaf value
      }
      for (int j = 0; j < nop; ++j) {
        if (!is_compute(ops[j])) continue;
        if (acc_holds == ops[j]) opnd[j] = EW_ACC;
        else if (slot_of[ops[j]] >= 0) opnd[j] = (uint8_t)slot_of[ops[j]];
        else return fail("elementwise schedule: internal error (value lost)");
      }
      alu.a = opnd[0];
      alu.b = opnd[1];
      for (int j = 0; j < nop; ++j) {
        if (temp_slot[j]) free_slots.push_back(opnd[j]);
        else if (is_compute(ops[j]) && last_use[ops[j]] == (int)k && slot_of[ops[j]] >= 0) {
          free_slots.push_back(slot_of[ops[j]]);
          slot_of[ops[j]] = -1;
        }
      }
      // The result stays only in the accumulator if its single consumer is the next op and
      // that op loads nothing before reading it; otherwise it gets a slot.
      bool keep = false;
      if (last_use[node] >= 0) {
        keep = true;
        if (last_use[node] == (int)k + 1) {
          const int nx = order[k + 1];
          bool next_loads = false;
          for (int j = 0; j < n_operands(nx); ++j) {
            const int a = canon(g[nx].operand[j]);
            if (!is_compute(a) && g[a].kind != FS_CONSTANT) next_loads = true;
          }
          keep = next_loads;   // every use is in op k+1 (last use), so the accumulator suffices
        }
      }
      if (keep) { alu.flags |= EW_KEEP; alu.dst = (uint8_t)take_slot(); slot_of[node] = alu.dst; }
      if (!emit(alu)) return false;
      acc_holds = node;
      if (out_ord[node] >= 0) {
        EwInstr st{};
        st.kind = EW_STORE; st.a = EW_ACC; st.arg = out_ord[node]; st.dtype = (uint8_t)out_dtype[node];
        if (!emit(st)) return false;
      }
      if (n_slots > 250) return fail("elementwise schedule: too many live values");
    }
    return true;
  }
};

}  // namespace

// The generated kernel's arguments: one pointer per operand view, one per output.
struct EwGenArgs { const void* in[64]; void* out[16]; void* ws; };
static_assert(kEwMaxViews <= 64 && kEwMaxOuts <= 16, "EwGenArgs mirrors the Args struct of the generated source");

// Kernel packing of independent elementwise computations (Section 5.1): the group falls into parts
// that share no computed value -- typically the same update applied to tensors of different
// shapes -- and each part is an elementwise group of its own shape.  One generated kernel runs
// them all, each part on its own run of workgroups.
static bool ew_plan_packed(const Graph& g, const LaunchOpts& opt, EwLaunch* out, int* status, std::string* err) {
  *status = FS_ERR_UNSUPPORTED;
  const int n = g.size();
  EwCompiler probe(g);
  // parts = connected components of the compute ops under "reads the value of"
  std::vector<int> part(n, -1);
  std::function<int(int)> find = [&](int v) { return part[v] == v ? v : part[v] = find(part[v]); };
  for (int i = 0; i < n; ++i) if (probe.is_compute(i)) part[i] = i;
  for (int i = 0; i < n; ++i) {
    if (part[i] < 0) continue;
    for (int j = 0; j < probe.n_operands(i); ++j) {
      const int a = probe.canon(g[i].operand[j]);
      if (probe.is_compute(a)) part[find(i)] = find(a);
    }
  }
  // parts that reach no output compute nothing anyone sees: left out
  std::vector<char> reaches_output(n, 0);
  for (int o : g.outputs) {
    const int src = probe.canon(g[o].operand[0]);
    if (part[src] >= 0) reaches_output[find(src)] = 1;
  }
  std::vector<int> roots;
  for (int i = 0; i < n; ++i) if (part[i] >= 0 && find(i) == i && reaches_output[i]) roots.push_back(i);
  if (roots.size() < 2) { *err = "elementwise schedule: ops of different shapes in one group"; return false; }
  if (roots.size() > 16) { *err = "elementwise schedule: more than 16 independent parts in one group"; return false; }
  if (g.outputs.size() > 16) { *err = "elementwise schedule: more than 16 outputs"; return false; }
  if (opt.wg_size && (opt.wg_size < 64 || opt.wg_size > 256 || opt.wg_size % 64)) {
    *status = FS_ERR_INVALID;
    *err = "elementwise schedule: wg_size must be 64, 128, 192 or 256";
    return false;
  }
  std::vector<std::unique_ptr<EwCompiler>> cs;
  std::vector<const EwIr*> irs;
  EwLaunch l;
  int n_views = 0;
  for (int r : roots) {
    cs.emplace_back(new EwCompiler(g));
    EwCompiler& cc = *cs.back();
    cc.active.assign(n, 0);
    for (int i = 0; i < n; ++i) if (part[i] >= 0 && find(i) == r) cc.active[i] = 1;
    if (!cc.analyse()) { *err = cc.err; return false; }
    if (cc.ir.n_outputs > kEwMaxOuts) { *err = "elementwise schedule: more than 8 outputs in one part"; return false; }
    irs.push_back(&cc.ir);
    l.n_ops += (int)cc.ir.nodes.size();
    for (int k = 0; k < cc.c.n_views; ++k) { l.view_param.push_back(cc.c.view_param[k]); l.view_full.push_back(cc.ir.views[k].full ? 1 : 0); }
    n_views += cc.c.n_views;
    l.n += cc.ir.n;
  }
  if (n_views > 64) { *err = "elementwise schedule: more than 64 operand views over all parts"; return false; }
  l.wg = opt.wg_size ? opt.wg_size : 256;
  std::vector<int> widths, blocks;
  const std::string src = ew_emit_packed(irs, l.wg, &widths, &blocks, &l.kernel_name);
  if (const char* dump = getenv("FS_DUMP_SOURCE")) {
    if (FILE* f = fopen(dump, "a")) { fputs(src.c_str(), f); fputs("\n// ----\n", f); fclose(f); }
  }
  std::string gen_err;
  if (!ew_compile_source(src, &l.code_object, &gen_err)) { *err = "elementwise schedule: " + gen_err; return false; }
  l.generated = true;
  l.parts = (int)roots.size();
  l.width = *std::max_element(widths.begin(), widths.end());
  int64_t grid = 0;
  for (int b : blocks) grid += b;
  l.grid = (int)grid;          // at most 16 * 2^20
  l.lds_bytes = 0;
  *out = l;
  *status = FS_OK;
  return true;
}

bool ew_stitch_plan(const Graph& g, const LaunchOpts& opt, EwLaunch* out, int* status, std::string* err) {
  *status = FS_ERR_UNSUPPORTED;
  EwCompiler cc(g);
  if (!cc.analyse()) {
    *err = cc.err;
    // several shapes: perhaps independent parts that can be packed into one kernel
    if (opt.codegen && cc.err.find("ops of different shapes") != std::string::npos) {
      std::string perr;
      int pst = FS_ERR_UNSUPPORTED;
      if (ew_plan_packed(g, opt, out, &pst, &perr)) { *status = FS_OK; return true; }
      if (pst == FS_ERR_INVALID) *status = pst;
      if (perr != cc.err) *err = cc.err + " (as independent parts: " + perr + ")";
    }
    return false;
  }
  EwLaunch l;
  *status = FS_ERR_INVALID;
  if (opt.wg_size && (opt.wg_size < 64 || opt.wg_size > 256 || opt.wg_size % 64)) {
    *err = "elementwise schedule: wg_size must be 64, 128, 192 or 256";
    return false;
  }
  if (opt.rows_per_wave && opt.rows_per_wave != 1 && opt.rows_per_wave != 2 && opt.rows_per_wave != 4) {
    *err = "elementwise schedule: rows_per_wave (chunks a thread carries in lock step) must be 1, 2 or 4";
    return false;
  }
  l.n_ops = (int)cc.ir.nodes.size();
  l.view_param.assign(cc.c.view_param, cc.c.view_param + cc.c.n_views);
  for (const EwIrView& v : cc.ir.views) l.view_full.push_back(v.full ? 1 : 0);

  // First choice: generate the kernel (the paper's way).  The interpreter below is the form
  // that needs no compiler at run time; it also takes over if generation fails.
  std::string gen_err;
  if (opt.codegen) {
    int width = 1, unroll = 1;
    const std::string src = ew_emit_source(cc.ir, &width, &unroll, &l.kernel_name);
    if (const char* dump = getenv("FS_DUMP_SOURCE")) {        // debugging aid: append what was generated
      if (FILE* f = fopen(dump, "a")) { fputs(src.c_str(), f); fputs("\n// ----\n", f); fclose(f); }
    }
    if (ew_compile_source(src, &l.code_object, &gen_err)) {
      l.generated = true;
      l.width = width;
      l.wg = opt.wg_size ? opt.wg_size : 256;
      l.n = cc.ir.n;
      const int64_t chunks = cc.ir.n / width;
      int64_t grid = (chunks + l.wg - 1) / l.wg;
      if (grid > (1 << 22)) grid = 1 << 22;
      if (opt.grid > 0 && opt.grid < grid) grid = opt.grid;
      l.grid = (int)(grid < 1 ? 1 : grid);
      l.lds_bytes = 0;
      *out = l;
      *status = FS_OK;
      return true;
    }
  }

  *status = FS_ERR_UNSUPPORTED;
  if (!cc.program()) {
    *err = cc.err + (gen_err.empty() ? "" : " (and kernel generation failed: " + gen_err + ")");
    return false;
  }
  l.note = gen_err;
  l.vector = cc.vec;
  l.n_slots = cc.n_slots;
  *status = FS_ERR_INVALID;
  // Geometry under the LDS volume constraint: slots * chunks * threads * 16 bytes + the
  // program <= 64 KB.
  // More chunks per thread amortise the decode of a program step; small problems keep one
  // chunk per thread so that the work still covers the chip.
  const int64_t work = cc.vec ? cc.c.prog.n / 4 : cc.c.prog.n;
  const int64_t kProgLds = kEwMaxInstr * 32;          // the program's own copy in LDS
  const int64_t kLds = 64 * 1024 - kProgLds;
  int wg = 0, U = 0;
  for (int u : {4, 2, 1}) {
    if (opt.rows_per_wave ? u != opt.rows_per_wave : (u > 1 && work < (int64_t)u * 256 * 512)) continue;
    for (int w : {256, 128, 64}) {
      if (opt.wg_size && w != opt.wg_size && !(opt.wg_size == 192 && w == 128)) continue;
      if ((int64_t)cc.n_slots * u * w * 16 <= kLds) { wg = w; U = u; break; }
    }
    if (U) break;
  }
  if (!U) {
    *err = "elementwise schedule: the group keeps more values alive than the LDS slot file holds";
    *status = FS_ERR_LDS;
    return false;
  }
  l.wg = wg;
  l.U = U;
  l.lds_bytes = (int64_t)cc.n_slots * U * wg * 16 + kProgLds;
  int64_t grid = (work + (int64_t)wg * U - 1) / ((int64_t)wg * U);
  if (grid > (1 << 20)) grid = 1 << 20;
  if (opt.grid > 0 && opt.grid < grid) grid = opt.grid;
  l.grid = (int)(grid < 1 ? 1 : grid);
  // Expand the program for this geometry (slot s of chunk u of thread t is float4 number
  // (s*U + u)*wg + t of the slot file) and normalise every ALU step to "accumulator op y":
  //   a: slot to load into the accumulator first, or -1;  b: where y comes from (itself, a
  //   slot whose index is in arg, or the immediate);  operands in the other order use the
  //   reversed ops
  for (int k = 0; k < cc.c.prog.n_ins; ++k) {
    const EwInstr& in = cc.c.code[k];
    EwStep& st = cc.c.prog.ins[k];
    auto slot = [&](uint8_t v) { return (int32_t)v * U * wg; };
    st.kind = in.kind; st.op = in.op; st.flags = in.flags | ((int32_t)in.dtype << 8); st.arg = in.arg; st.imm = in.imm;
    st.a = in.a == EW_ACC ? -1 : slot(in.a);
    st.b = EW_B_SELF;
    st.dst = slot(in.dst);
    if (in.kind != EW_ALU) continue;
    const bool binary = is_binary(in.op);
    if (!binary) continue;                       // unary: a is the accumulator or a slot to preload
    const int rev = in.op == FS_SUBTRACT ? EW_RSUB : in.op == FS_DIVIDE ? EW_RDIV : in.op;
    const bool a_imm = in.flags & EW_A_IMM, b_imm = in.flags & EW_B_IMM;
    const bool a_acc = !a_imm && in.a == EW_ACC, b_acc = !b_imm && in.b == EW_ACC;
    if (a_imm) {                                 // (imm, acc) or (imm, slot): reversed, y = imm
      st.op = rev; st.b = EW_B_IMM_MODE;
      st.a = b_acc ? -1 : slot(in.b);
    } else if (b_imm) {                          // (acc, imm) or (slot, imm)
      st.b = EW_B_IMM_MODE;
    } else if (a_acc && b_acc) {                 // the same value twice
      st.b = EW_B_SELF;
    } else if (a_acc) {                          // (acc, slot)
      st.b = EW_B_SLOT; st.arg = slot(in.b);
    } else if (b_acc) {                          // (slot, acc): reversed, y = the slot
      st.op = rev; st.a = -1; st.b = EW_B_SLOT; st.arg = slot(in.a);
    } else if (in.a == in.b) {                   // one slot twice
      st.b = EW_B_SELF;
    } else {                                     // (slot, slot): preload a, y = slot b
      st.b = EW_B_SLOT; st.arg = slot(in.b);
    }
  }
  l.blob.resize(sizeof(EwCompiled));
  memcpy(l.blob.data(), &cc.c, sizeof(EwCompiled));
  l.n_ins = cc.c.prog.n_ins;
  *out = l;
  *status = FS_OK;
  return true;
}

std::string ew_stitch_describe(const EwLaunch& l) {
  char buf[320];
  if (l.generated && l.parts > 1)
    snprintf(buf, sizeof buf, "elementwise[GRID,CTA-THREAD_%d] x%d packed in %d independent parts (generated kernel %s, %zu bytes of code); cta_num=%d, cta_size=%d, lds=0",
             l.width, l.n_ops, l.parts, l.kernel_name.c_str(), l.code_object.size(), l.grid, l.wg);
  else if (l.generated)
    snprintf(buf, sizeof buf, "elementwise[GRID,CTA-THREAD_%d] x%d merged (generated kernel %s, %zu bytes of code); cta_num=%d, cta_size=%d, lds=0",
             l.width, l.n_ops, l.kernel_name.c_str(), l.code_object.size(), l.grid, l.wg);
  else
    snprintf(buf, sizeof buf, "elementwise[GRID,CTA-THREAD_%d] x%d merged (interpreted: %d program steps, %d LDS slots); cta_num=%d, cta_size=%d, lds=%lld",
             (l.vector ? 4 : 1) * l.U, l.n_ops, l.n_ins, l.n_slots, l.grid, l.wg, (long long)l.lds_bytes);
  return buf;
}

template <bool VEC>
static void ew_launch_u(const EwLaunch& l, hipStream_t s, const EwProgram& prog) {
  const dim3 grid(l.grid), block(l.wg);
  const size_t lds = (size_t)(l.lds_bytes - kEwMaxInstr * 32);   // dynamic part: the slot file
  if (l.U == 4) hipLaunchKernelGGL((ew_stitch_kernel<VEC, 4>), grid, block, lds, s, prog);
  else if (l.U == 2) hipLaunchKernelGGL((ew_stitch_kernel<VEC, 2>), grid, block, lds, s, prog);
  else hipLaunchKernelGGL((ew_stitch_kernel<VEC, 1>), grid, block, lds, s, prog);
}

void ew_stitch_release(EwLaunch& l) { ew_module_release(&l.loaded); }

int ew_stitch_launch(EwLaunch& l, const void* const* in, void* const* out, int n_out, void* stream, std::string* err) {
  if (l.generated) {
    if (l.n == 0) return 0;
    EwGenArgs args{};
    for (size_t k = 0; k < l.view_param.size(); ++k) args.in[k] = in[l.view_param[k]];
    for (int k = 0; k < n_out && k < 16; ++k) args.out[k] = out[k];
    return ew_module_launch(&l.loaded, l.code_object, l.kernel_name, &args, sizeof args, l.grid, l.wg, stream, err);
  }
  EwCompiled c;
  memcpy(&c, l.blob.data(), sizeof(EwCompiled));
  if (c.prog.n == 0) return 0;
  for (int k = 0; k < c.n_views; ++k) c.prog.views[k].p = in[c.view_param[k]];
  for (int k = 0; k < n_out; ++k) c.prog.outs[k] = out[k];
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (l.vector) ew_launch_u<true>(l, s, c.prog);
  else ew_launch_u<false>(l, s, c.prog);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) { *err = std::string("ew_stitch launch: ") + hipGetErrorString(e); return -1; }
  return 0;
}

}  // namespace fs
