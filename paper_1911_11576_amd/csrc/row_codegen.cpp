// Kernel generation for row groups (paper Section 5.1, warp composition: a reduction and the
// ops that consume its result run in one kernel, the reduced value handed over in
// registers; Section 5.3: the stitched op is emitted as code).
//
// A row group has one "full" shape [R..., C]; its values are either full (one per element) or
// per-row (shape [R...]: results of reductions over the last dim and arithmetic on them).
// Any DAG of elementwise ops on full values, reductions full -> per-row, elementwise ops on
// per-row values, and per-row values broadcast back into full ops is accepted, with full
// and per-row outputs in any number up to 8.  The generated kernel gives each row to L
// lanes (L = 1: the THREAD template of Section 5.2 for tiny rows, sequential reduction in
// one thread; L = 2..64: the WARP template, lanes combine with DPP / permlane steps;
// L = 128..1024: the block-composed template, one workgroup per row, wavefronts combine
// through one float each in LDS and a barrier); a lane keeps its K chunks of W consecutive
// elements of every live full value in registers from the row's one read to its one write.
//
// Packed with the row work (kernel packing, Section 5.1): reductions over the rows -- sums and maxima
// of a full value over all rows, or over each run of consecutive rows ([B, S, H] -> [B, H]) -- kept as
// running values per lane and column while a fixed grid of workgroups loops over the rows; small batched
// dots whose operands are a row's registers.  Rows too long for registers are streamed in passes by one
// workgroup, with LDS row buffers laid out by the shared-memory optimisation (Section 5.4, Algorithm 4).
#include "row_codegen.h"
#include "shared_plan.h"
#include "launchers.h"
#include "match.h"

#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <hip/hip_runtime.h>

#include <cstring>
#include <algorithm>
#include <functional>
#include <map>

namespace fs {

const char* ew_preamble();   // ew_codegen.cpp: typedefs, Args, dtype conversion helpers

namespace {

enum Cls : int { CLS_NONE = 0, CLS_FULL = 1, CLS_ROW = 2, CLS_COL = 3, CLS_DOT_OUT = 4 };   // COL: one value per column (reduced over the rows); DOT_OUT: [B, M, D] result of a consuming dot on the matrix unit
enum OpndKind : int { OP_NODE = 0, OP_ROWB = 1, OP_VIEW = 2, OP_CONST = 3 };

struct Opnd { int kind = OP_NODE; int index = -1; float cval = 0.f; };
// beside the fs_opkind / EwExtraOp values: a batched dot with a tiny contraction that produces
// the full tile (sum over k of a per-row scalar times a per-column vector), and a batched dot
// that contracts the full last dim into one value per row
// ... and the two dots of the block-composed template on the matrix unit: a producing dot
// a[B,M,K] . b[B,N,K]^T -> the group's full tile, and a consuming dot p[B,M,N] . v[B,N,D] -> [B,M,D]
enum RowExtraOp : int { ROP_DOT_OUTER = 200, ROP_DOT_REDUCE = 201, ROP_DOT_MMA_IN = 202, ROP_DOT_MMA_OUT = 203 };

struct RNode {
  int id = -1, op = 0, cls = CLS_NONE, nop = 1;
  Opnd o[2];
  std::vector<int> dot_row, dot_full;   // ROP_DOT_OUTER: view pairs per k; ROP_DOT_REDUCE: dot_full[0]
  float gelu[3] = {0.f, 0.f, 0.f};      // EW_OP_GELU_TANH: mul, a0, a1 of mul*h / (1 + exp2(h*(a0 + a1*h*h)))
  int out_ord = -1, out_dtype = FS_F32;
  bool over_dot_out = false;            // a row reduction over the [B, M, D] result of a consuming dot
};
struct RView {
  int param = -1, dtype = FS_F32, cls = CLS_FULL;
  int64_t stride[FS_MAX_RANK] = {0, 0, 0, 0};   // over the dims of the full shape (row views: last unused)
  int64_t offset = 0;                            // constant element offset (a slice of a dot operand)
};

struct Analysis {
  const Graph& g;
  std::string err;
  int rank = 0;
  int64_t S[FS_MAX_RANK] = {1, 1, 1, 1};
  int64_t rows = 1, cols = 1;
  std::vector<int> cls;
  std::vector<char> colv;        // a value of shape [C] computed in the group: one per column, the same for every row
  std::vector<RNode> nodes;
  std::vector<RView> views;
  int n_reduce = 0;
  int n_col = 0;                 // column reductions (over the rows), results are outputs only
  int64_t seg_rows = 0;          // 0: the column reductions run over all rows; else over each run of this many
                                 // consecutive rows (the innermost row dims: [B, S, H] summed over S -> [B, H])
  bool has_causal = false;       // a causal_mask op: the row's index in the second-to-last dim is needed
  // block composition around dots on the matrix unit (16-bit operands, contraction 16..128)
  int mma_in = -1, mma_out = -1;         // node ids of the producing and the consuming dot, -1 = none
  int mma_dtype = FS_F16;                // dtype of the dots' operands
  int64_t mma_k = 0, mma_d = 0;          // contraction length of the producing dot, result width of the consuming one
  int mma_va = -1, mma_vb = -1, mma_vv = -1;   // views (pointer only) of a, b and v
  bool mma_b_kn = false;                 // the producing dot's second operand is stored [B, K, N] (contraction along its rows)

  explicit Analysis(const Graph& gr) : g(gr) {}
  bool fail(const std::string& m) { err = m; return false; }

  static bool is_reduce(int k) { return k == FS_REDUCE_SUM || k == FS_REDUCE_MAX; }
  int canon(int n) const {
    while (g[n].kind == FS_CONVERT && g[n].dtype == FS_F32) n = g[n].operand[0];
    return n;
  }
  bool is_compute(int n) const {
    const int k = g[n].kind;
    return (is_binary(k) || is_unary(k) || k == FS_CONVERT || is_reduce(k) || k == FS_DOT || k == FS_CAUSAL_MASK) && canon(n) == n;
  }
  bool shape_is_full(const Node& x) const {
    if (x.rank != rank) return false;
    for (int d = 0; d < rank; ++d) if (x.shape[d] != S[d]) return false;
    return true;
  }
  // one value per row: the full shape without its last dim, or with it collapsed to 1
  bool shape_is_row(const Node& x) const {
    if (x.rank == rank && x.shape[rank - 1] == 1 && S[rank - 1] != 1) {
      for (int d = 0; d < rank - 1; ++d) if (x.shape[d] != S[d]) return false;
      return true;
    }
    if (x.rank != rank - 1) return false;
    for (int d = 0; d < rank - 1; ++d) if (x.shape[d] != S[d]) return false;
    return true;
  }

  // one value per column: [C] under a full shape of rank 2 or more (and not also the row shape)
  bool shape_is_column(const Node& x) const {
    return rank >= 2 && x.rank == 1 && x.shape[0] == S[rank - 1] && !shape_is_row(x);
  }

  // Leaf (parameter seen through broadcasts and widening converts, or constant) -> strides
  // over the dims of node n's own shape.  False if a computed value sits below a broadcast.
  bool leaf_strides(int n, int* base, int64_t* stride, bool* is_const, float* cval) {
    n = canon(n);
    const Node& x = g[n];
    *is_const = false;
    if (x.kind == FS_CONSTANT) { *is_const = true; *cval = (float)x.attr; return true; }
    if (x.kind == FS_BROADCAST) {
      int64_t inner[FS_MAX_RANK] = {0, 0, 0, 0};
      if (!leaf_strides(x.operand[0], base, inner, is_const, cval)) return false;
      if (*is_const) return true;
      const Node& a = g[x.operand[0]];
      for (int d = 0; d < x.rank; ++d) stride[d] = 0;
      for (int d = 0; d < a.rank; ++d) stride[x.axis + d] = a.shape[d] == 1 ? 0 : inner[d];
      return true;
    }
    if (x.kind != FS_PARAMETER) return fail("generated row schedule: a computed value is broadcast in a way other than per-row");
    *base = n;
    int64_t st = 1;
    for (int d = x.rank - 1; d >= 0; --d) { stride[d] = st; st *= x.shape[d]; }
    return true;
  }

  int view_index(int base, const int64_t* stride, int c, int64_t offset = 0) {
    for (size_t k = 0; k < views.size(); ++k) {
      bool same = views[k].param == g[base].ordinal && views[k].cls == c && views[k].offset == offset;
      for (int d = 0; d < FS_MAX_RANK && same; ++d) same = views[k].stride[d] == stride[d];
      if (same) return (int)k;
    }
    RView v;
    v.param = g[base].ordinal; v.dtype = g[base].dtype; v.cls = c; v.offset = offset;
    for (int d = 0; d < FS_MAX_RANK; ++d) v.stride[d] = stride[d];
    views.push_back(v);
    return (int)views.size() - 1;
  }

  // `as_column`: the consumer is a per-column value (shape [C]) kept as a full value whose rows are
  // all alike; its parameter operands have that shape too and are read with row stride 0.
  bool operand(int n, int consumer_cls, Opnd* o, bool as_column = false) {
    const int c = canon(n);
    if (is_compute(c)) {
      if (cls[c] != consumer_cls || (as_column && !colv[c])) return fail("generated row schedule: operand of the wrong shape class");
      o->kind = OP_NODE; o->index = c;
      return true;
    }
    // a per-row value broadcast along the last dim into a full op
    if (g[c].kind == FS_BROADCAST && consumer_cls == CLS_FULL && !as_column) {
      const int src = canon(g[c].operand[0]);
      if (is_compute(src) && colv[src]) {
        // a per-column value computed in the group, broadcast over the rows: it already is a full value here
        if (!shape_is_full(g[c]) || g[c].axis != rank - 1) return fail("generated row schedule: a per-column value broadcast along another dim");
        o->kind = OP_NODE; o->index = src;
        return true;
      }
      if (is_compute(src)) {
        if (cls[src] != CLS_ROW || !shape_is_full(g[c]) || (g[src].rank > 0 && g[c].axis != 0))  // leading dims line up
          return fail("generated row schedule: only per-row values may be broadcast back");
        o->kind = OP_ROWB; o->index = src;
        return true;
      }
    }
    int base = -1;
    int64_t st[FS_MAX_RANK] = {0, 0, 0, 0};
    bool is_const = false;
    float cv = 0.f;
    if (!leaf_strides(c, &base, st, &is_const, &cv)) return false;
    if (is_const) { o->kind = OP_CONST; o->cval = cv; return true; }
    const Node& shp = g[c];
    if (as_column) {
      if (!shape_is_column(shp)) return fail("generated row schedule: operand shape differs from its consumer's");
      const int64_t last = st[0];
      for (int d = 0; d < FS_MAX_RANK; ++d) st[d] = 0;
      st[rank - 1] = last;
      o->kind = OP_VIEW;
      o->index = view_index(base, st, CLS_FULL);
      return true;
    }
    if (consumer_cls == CLS_FULL ? !shape_is_full(shp) : !shape_is_row(shp))
      return fail("generated row schedule: operand shape differs from its consumer's");
    o->kind = OP_VIEW;
    o->index = view_index(base, st, consumer_cls);
    return true;
  }

  bool shape_is_dot_out(const Node& x) const {
    return mma_out >= 0 && rank == 3 && x.rank == 3 && x.shape[0] == S[0] && x.shape[1] == S[1] && x.shape[2] == mma_d;
  }
  // does op i work on the result of the consuming dot (the epilogue around the second dot)?
  bool reads_dot_out(int i) const {
    for (int j = 0; j < operand_count(g[i].kind); ++j) {
      const int c = canon(g[i].operand[j]);
      if (is_compute(c) && cls[c] == CLS_DOT_OUT) return true;
    }
    return false;
  }
  // Operand of an elementwise op on the consuming dot's result [B, M, D]: another such value, a per-row value
  // of the group broadcast along D, a constant, or an input seen as [B, M, D] (any strides over B and M;
  // contiguous or repeated along D).
  bool operand_dot_out(int n, Opnd* o) {
    const int c = canon(n);
    if (is_compute(c)) {
      if (cls[c] != CLS_DOT_OUT) return fail("generated row schedule: operand of the wrong shape class");
      o->kind = OP_NODE; o->index = c;
      return true;
    }
    if (g[c].kind == FS_BROADCAST) {
      const int src = canon(g[c].operand[0]);
      if (is_compute(src)) {
        if (cls[src] != CLS_ROW || !shape_is_dot_out(g[c]) || (g[src].rank > 0 && g[c].axis != 0))
          return fail("generated row schedule: only per-row values may be broadcast into the ops after a consuming dot");
        o->kind = OP_ROWB; o->index = src;
        return true;
      }
    }
    int base = -1;
    int64_t st[FS_MAX_RANK] = {0, 0, 0, 0};
    bool is_const = false;
    float cv = 0.f;
    if (!leaf_strides(c, &base, st, &is_const, &cv)) return false;
    if (is_const) { o->kind = OP_CONST; o->cval = cv; return true; }
    if (!shape_is_dot_out(g[c])) return fail("generated row schedule: operand shape differs from its consumer's");
    if (st[2] != 0 && st[2] != 1) return fail("generated row schedule: an operand strided along the last dim");
    if (st[2] == 1 && (st[0] % 4 || st[1] % 4)) return fail("generated row schedule: an operand of the ops after a consuming dot is not readable in pieces of 4 elements");
    o->kind = OP_VIEW;
    o->index = view_index(base, st, CLS_DOT_OUT);
    return true;
  }

  // A parameter behind widening converts, as a dense tensor: its node and dims.
  bool dense_param(int n, int* base) const {
    n = canon(n);
    if (g[n].kind != FS_PARAMETER) return false;
    *base = n;
    return true;
  }

  // Batched dots small enough to be arithmetic on the row's registers (no matrix unit: the
  // contraction is a handful of terms, or it is the row reduction itself):
  //   outer:  a[B,M,K] . b -> [B,M,N] = the group's full shape, K <= 8, a and b parameters,
  //           b contiguous along N (stored [B,K,N], or K == 1)
  //   reduce: p[B,M,N] . b -> [B,M,1], p a full value of the group, b a parameter contiguous
  //           along N (stored [B,1,N], or [B,N,1])
  bool dot_node(int i, RNode* r) {
    const Node& x = g[i];
    if (rank != 3 || x.rank != 3) return fail("generated row schedule: dot outside a rank-3 group");
    const int ia = canon(x.operand[0]), ib = canon(x.operand[1]);
    const Node& a = g[ia];
    const Node& b = g[ib];
    const bool bt = x.axis == 1;                       // b stored [B, N_out, K_contract]
    const int64_t Kc = a.shape[2], Nout = bt ? b.shape[1] : b.shape[2];
    r->id = i;
    int pb = -1;
    if (!dense_param(ib, &pb)) return fail("generated row schedule: second dot operand must be a group input");
    if (a.rank != 3 || b.rank != 3 || b.shape[0] != S[0] || (bt ? b.shape[2] : b.shape[1]) != Kc)
      return fail("generated row schedule: dot operand shapes do not fit the group");
    const int64_t none[FS_MAX_RANK] = {0, 0, 0, 0};
    if (is_compute(ia) && cls[ia] == CLS_FULL && x.shape[2] != 1) {
      // consuming dot on the matrix unit: p[B,M,N] . v[B,N,D] -> [B,M,D], p a 16-bit full value of the group
      if (mma_out >= 0) return fail("generated row schedule: more than one consuming dot");
      if (bt) return fail("generated row schedule: the second operand of a consuming dot must be stored [B, N, D]");
      if (Kc != S[2] || x.shape[0] != S[0] || x.shape[1] != S[1]) return fail("generated row schedule: consuming dot shape differs from the group's");
      if (a.dtype == FS_F32 || b.dtype != a.dtype) return fail("generated row schedule: a consuming dot needs 16-bit operands of one dtype");
      if (Nout != 32 && Nout != 64 && Nout != 128) return fail("generated row schedule: consuming dot result width must be 32, 64 or 128");
      if (x.dtype != FS_F32) return fail("generated row schedule: dots accumulate in f32");
      if (mma_in >= 0 && mma_dtype != a.dtype) return fail("generated row schedule: the two dots use different operand dtypes");
      r->op = ROP_DOT_MMA_OUT; r->cls = CLS_DOT_OUT; r->nop = 1;
      cls[i] = CLS_DOT_OUT;
      if (!operand(x.operand[0], CLS_FULL, &r->o[0])) return false;
      mma_out = i; mma_dtype = a.dtype; mma_d = Nout;
      mma_vv = view_index(pb, none, CLS_NONE);
      return true;
    }
    if (shape_is_full(x) && !(is_compute(ia) && cls[ia] == CLS_FULL) && Kc >= 16) {
      // producing dot on the matrix unit: a[B,M,K] . b[B,N,K]^T -> the full tile
      int pa = -1;
      if (!dense_param(ia, &pa)) return fail("generated row schedule: first operand of a producing dot must be a group input");
      if (mma_in >= 0) return fail("generated row schedule: more than one producing dot with a real contraction");
      if (a.dtype == FS_F32 || b.dtype != a.dtype) return fail("generated row schedule: a dot with contraction >= 16 needs 16-bit operands of one dtype (the matrix unit)");
      if (Kc % 8 != 0 || Kc > 128) return fail("generated row schedule: producing dot contraction must be a multiple of 8 up to 128");
      if (a.shape[0] != S[0] || a.shape[1] != S[1] || Nout != S[2]) return fail("generated row schedule: dot shape differs from the group's");
      if (x.dtype != FS_F32) return fail("generated row schedule: dots accumulate in f32");
      if (mma_out >= 0 && mma_dtype != a.dtype) return fail("generated row schedule: the two dots use different operand dtypes");
      r->op = ROP_DOT_MMA_IN; r->cls = CLS_FULL; r->nop = 0;
      cls[i] = CLS_FULL;
      mma_in = i; mma_dtype = a.dtype; mma_k = Kc; mma_b_kn = !bt;
      mma_va = view_index(pa, none, CLS_NONE);
      mma_vb = view_index(pb, none, CLS_NONE);
      return true;
    }
    if (shape_is_full(x) && !(is_compute(ia) && cls[ia] == CLS_FULL)) {
      // outer form
      int pa = -1;
      if (!dense_param(ia, &pa)) return fail("generated row schedule: first operand of a producing dot must be a group input");
      if (Kc > 8) return fail("generated row schedule: dot contraction longer than 8 (a matrix-unit schedule is needed)");
      if (bt && Kc != 1) return fail("generated row schedule: dot operand not contiguous along the row");
      if (a.shape[0] != S[0] || a.shape[1] != S[1] || Nout != S[2]) return fail("generated row schedule: dot shape differs from the group's");
      r->op = ROP_DOT_OUTER; r->cls = CLS_FULL; r->nop = 0;
      cls[i] = CLS_FULL;
      for (int64_t k = 0; k < Kc; ++k) {
        const int64_t sa[FS_MAX_RANK] = {S[1] * Kc, Kc, 0, 0};              // a[b, m, k]: one scalar per row
        const int64_t sb[FS_MAX_RANK] = {Kc * S[2], 0, 1, 0};               // b[b, k, :]: shared by the rows of a batch
        r->dot_row.push_back(view_index(pa, sa, CLS_ROW, k));
        r->dot_full.push_back(view_index(pb, sb, CLS_FULL, bt ? 0 : k * S[2]));
      }
      return true;
    }
    // reduce form
    if (!(x.shape[0] == S[0] && x.shape[1] == S[1] && x.shape[2] == 1))
      return fail("generated row schedule: a consuming dot must produce one value per row");
    if (Kc != S[2]) return fail("generated row schedule: dot contraction differs from the row length");
    r->op = ROP_DOT_REDUCE; r->cls = CLS_ROW; r->nop = 1;
    cls[i] = CLS_ROW;
    if (!operand(x.operand[0], CLS_FULL, &r->o[0])) return false;
    const int64_t sb[FS_MAX_RANK] = {S[2], 0, 1, 0};                         // b[b, :, 0] or b[b, 0, :]
    r->dot_full.push_back(view_index(pb, sb, CLS_FULL, 0));
    ++n_reduce;
    return true;
  }

  bool run() {
    const int n = g.size();
    // the full shape is the operand shape of the first reduction; without a reduction (full and
    // per-row arithmetic mixed, a per-row value broadcast into full ops) the largest shape computed
    int first = -1;
    for (int i = 0; i < n && first < 0; ++i) if (is_reduce(g[i].kind)) first = i;
    int shape_of = first >= 0 ? g[first].operand[0] : -1;
    // a dot of two group inputs with a real contraction fixes the shape: its result is the tile the
    // block-composed template is built around
    for (int i = 0; i < n; ++i) {
      if (g[i].kind != FS_DOT || g[i].rank != 3) continue;
      const int ia = canon(g[i].operand[0]), ib = canon(g[i].operand[1]);
      if (g[ia].kind == FS_PARAMETER && g[ib].kind == FS_PARAMETER && g[ia].rank == 3 && g[ia].shape[2] >= 16) { shape_of = i; break; }
    }
    if (shape_of < 0) {
      for (int i = 0; i < n; ++i) {
        const int k = g[i].kind;
        if (!(is_binary(k) || is_unary(k) || k == FS_CONVERT || k == FS_CAUSAL_MASK)) continue;
        if (shape_of < 0 || g[i].numel() > g[shape_of].numel() || (g[i].numel() == g[shape_of].numel() && g[i].rank > g[shape_of].rank))
          shape_of = i;
      }
      if (shape_of < 0) return fail("generated row schedule: the group computes nothing");
    }
    const Node& src = g[shape_of];
    rank = src.rank;
    if (rank < 1) return fail("generated row schedule: rank-0 group");
    for (int d = 0; d < rank; ++d) S[d] = src.shape[d];
    cols = S[rank - 1];
    rows = 1;
    for (int d = 0; d + 1 < rank; ++d) rows *= S[d];
    cls.assign(n, CLS_NONE);
    colv.assign(n, 0);
    std::vector<int> out_ord(n, -1), out_dtype(n, 0);
    std::vector<char> store_rounding(n, 0);    // a convert whose only job is the rounding of a consuming dot's result at its store
    for (int o : g.outputs) {
      int s = canon(g[o].operand[0]);
      if (g[s].kind == FS_CONVERT && g[canon(g[s].operand[0])].kind == FS_DOT && g[s].rank == 3 && rank == 3) {
        const int d = canon(g[s].operand[0]);
        const int da = canon(g[d].operand[0]);
        int users = 0;
        for (int i = 0; i < n; ++i) for (int j = 0; j < operand_count(g[i].kind); ++j) if (g[i].operand[j] == s) ++users;
        // (the dot is a consuming one if its first operand is computed in the group and is not a widening alias of an input)
        if (users == 1 && g[da].kind != FS_PARAMETER && g[d].shape[2] != 1) { store_rounding[s] = 1; s = d; }
      }
      if (!is_compute(s)) return fail("generated row schedule: an output that is a plain copy of an input");
      if (out_ord[s] >= 0) return fail("generated row schedule: one value feeds two outputs");
      out_ord[s] = g[o].ordinal;
      out_dtype[s] = g[o].dtype;
    }
    if (g.outputs.size() > 8) return fail("generated row schedule: more than 8 outputs");
    // A sum over the rows may be spelled as a chain of sums over the leading dim, one per
    // leading dim of the group's shape ([B, S, H] -> [S, H] -> [H]): the last one stands for the
    // whole chain, the ones before it (read by nothing else) compute nothing of their own.
    std::vector<int> col_base(n, -1);
    std::vector<char> col_mid(n, 0);
    {
      std::vector<int> n_users(n, 0);
      for (int i = 0; i < n; ++i) for (int j = 0; j < operand_count(g[i].kind); ++j) ++n_users[g[i].operand[j]];
      for (int i = 0; i < n; ++i) {
        const Node& x = g[i];
        if (!is_reduce(x.kind) || x.axis != 0 || x.rank != 1 || rank < 2 || x.shape[0] != S[rank - 1]) continue;
        int cur = x.operand[0], levels = 1;
        std::vector<int> mids;
        while (g[cur].kind == x.kind && g[cur].axis == 0 && n_users[cur] == 1 && out_ord[cur] < 0) {
          mids.push_back(cur);
          cur = g[cur].operand[0];
          ++levels;
        }
        cur = canon(cur);
        if (levels != rank - 1 || g[cur].rank != rank) continue;
        col_base[i] = cur;
        for (int m : mids) col_mid[m] = 1;
      }
    }
    // A sum over the innermost row dims only ([B, S, H] summed over S, or [B, N, S, H] over S and then
    // over N, each link over the dim before the last): column sums per run of consecutive rows.
    if (rank >= 3) {
      std::vector<int> n_users(n, 0);
      for (int i = 0; i < n; ++i) for (int j = 0; j < operand_count(g[i].kind); ++j) ++n_users[g[i].operand[j]];
      for (int i = 0; i < n; ++i) {
        const Node& x = g[i];
        if (!is_reduce(x.kind) || col_base[i] >= 0 || col_mid[i] || out_ord[i] < 0) continue;
        int cur = i, levels = 0;
        std::vector<int> mids;
        while (g[cur].kind == x.kind && g[g[cur].operand[0]].rank >= 3 && g[cur].axis == g[g[cur].operand[0]].rank - 2 &&
               (cur == i || (n_users[cur] == 1 && out_ord[cur] < 0))) {
          if (cur != i) mids.push_back(cur);
          cur = g[cur].operand[0];
          ++levels;
        }
        cur = canon(cur);
        if (levels < 1 || levels > rank - 2 || g[cur].rank != rank || !shape_is_full(g[cur])) continue;
        // the result keeps the outer row dims and the columns
        bool fits = x.rank == rank - levels && x.shape[x.rank - 1] == S[rank - 1];
        for (int d = 0; d + 1 < x.rank && fits; ++d) fits = x.shape[d] == S[d];
        if (!fits) continue;
        int64_t seg = 1;
        for (int d = rank - 1 - levels; d < rank - 1; ++d) seg *= S[d];
        if (seg == 0) continue;          // empty runs: left to the per-op form
        if (seg_rows != 0 && seg_rows != seg) return fail("generated row schedule: column sums over runs of rows of different lengths");
        seg_rows = seg;
        col_base[i] = cur;
        for (int m : mids) col_mid[m] = 1;
      }
      if (seg_rows != 0)
        for (int i = 0; i < n; ++i) if (col_base[i] >= 0 && g[i].rank == 1 && rank >= 2)
          return fail("generated row schedule: sums over all rows and sums over runs of rows in one group");
    }
    // the tanh-form GELU is computed as one op
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
    for (int i = 0; i < n; ++i) {
      const Node& x = g[i];
      const int k = x.kind;
      if (k == FS_PARAMETER || k == FS_CONSTANT || k == FS_BROADCAST || k == FS_OUTPUT) continue;
      if (inside_idiom[i] || col_mid[i] || store_rounding[i]) continue;
      if (idiom_of[i] >= 0) {
        const GeluIdiom& id = idioms[idiom_of[i]];
        RNode r;
        r.id = i; r.op = EW_OP_GELU_TANH; r.nop = 1;
        const int hc = canon(id.h);
        const bool after_dot = is_compute(hc) && cls[hc] == CLS_DOT_OUT;
        r.cls = after_dot ? CLS_DOT_OUT : shape_is_full(x) ? CLS_FULL : shape_is_row(x) ? CLS_ROW : CLS_NONE;
        if (r.cls == CLS_NONE) return fail("generated row schedule: an op whose shape is neither the group's nor its row shape");
        cls[i] = r.cls;
        if (after_dot ? !operand_dot_out(id.h, &r.o[0]) : !operand(id.h, r.cls, &r.o[0])) return false;
        gelu_constants(id, r.gelu);
        r.out_ord = out_ord[i];
        r.out_dtype = out_dtype[i];
        nodes.push_back(r);
        continue;
      }
      if (k == FS_DOT) {
        RNode r;
        if (!dot_node(i, &r)) return false;
        r.out_ord = out_ord[i];
        r.out_dtype = out_dtype[i];
        nodes.push_back(r);
        continue;
      }
      if (k == FS_CAUSAL_MASK) {
        // x[..., i, j] kept where j <= i: elementwise on a full value, with the row's own index
        if (!shape_is_full(x) || rank < 2) return fail("generated row schedule: causal_mask on something other than the group's full shape");
        RNode r;
        r.id = i; r.op = k; r.cls = CLS_FULL; r.nop = 1;
        cls[i] = CLS_FULL;
        if (!operand(x.operand[0], CLS_FULL, &r.o[0])) return false;
        r.o[1].cval = (float)x.attr;
        r.out_ord = out_ord[i];
        r.out_dtype = out_dtype[i];
        has_causal = true;
        nodes.push_back(r);
        continue;
      }
      if (!(is_binary(k) || is_unary(k) || k == FS_CONVERT || is_reduce(k)))
        return fail(std::string("generated row schedule: op ") + kind_name(k) + " is not elementwise, a reduction or a small dot");
      if (!is_compute(i)) continue;       // widening convert: alias
      RNode r;
      r.id = i;
      if (col_base[i] >= 0) {
        // a reduction over the rows: packed with the row work over the same register-resident rows
        if (out_ord[i] < 0) return fail("generated row schedule: a column-reduced value must be a group output");
        r.cls = CLS_COL; r.op = k; r.nop = 1;
        cls[i] = CLS_COL;
        if (!operand(col_base[i], CLS_FULL, &r.o[0])) return false;
        ++n_col;
      } else if (is_reduce(k)) {
        const bool after_dot = reads_dot_out(i);      // over the D columns of the consuming dot's result: one value per row all the same
        if (x.axis != rank - 1 || !shape_is_row(x)) return fail("generated row schedule: reduction not over the last dim of the group's shape");
        r.cls = CLS_ROW; r.op = k; r.nop = 1;
        r.over_dot_out = after_dot;
        cls[i] = CLS_ROW;
        if (after_dot ? !operand_dot_out(x.operand[0], &r.o[0]) : !operand(x.operand[0], CLS_FULL, &r.o[0])) return false;
        ++n_reduce;
      } else if (reads_dot_out(i)) {
        // the epilogue around the consuming dot: elementwise on its [B, M, D] result, in the accumulators' layout
        if (!shape_is_dot_out(x)) return fail("generated row schedule: an op on a consuming dot's result with another shape");
        r.cls = CLS_DOT_OUT;
        cls[i] = CLS_DOT_OUT;
        r.op = k == FS_CONVERT ? (x.dtype == FS_F16 ? (int)EW_OP_ROUND_F16 : (int)EW_OP_ROUND_BF16) : k;
        r.nop = is_binary(k) ? 2 : 1;
        for (int j = 0; j < r.nop; ++j) if (!operand_dot_out(x.operand[j], &r.o[j])) return false;
      } else {
        // arithmetic on per-column values (a scale vector prepared from parameters, say) is done as
        // full arithmetic whose rows are all alike: a few redundant ops per row, no kernel of its own
        const bool column = !shape_is_full(x) && !shape_is_row(x) && shape_is_column(x);
        r.cls = shape_is_full(x) || column ? CLS_FULL : shape_is_row(x) ? CLS_ROW : CLS_NONE;
        if (r.cls == CLS_NONE) return fail("generated row schedule: an op whose shape is neither the group's nor its row shape");
        if (column && out_ord[i] >= 0) return fail("generated row schedule: a per-column value computed in the group is a group output");
        cls[i] = r.cls;
        colv[i] = column;
        r.op = k == FS_CONVERT ? (x.dtype == FS_F16 ? (int)EW_OP_ROUND_F16 : (int)EW_OP_ROUND_BF16) : k;
        r.nop = is_binary(k) ? 2 : 1;
        for (int j = 0; j < r.nop; ++j) if (!operand(x.operand[j], r.cls, &r.o[j], column)) return false;
        if (r.nop == 2 && r.o[0].kind == OP_CONST && r.o[1].kind == OP_CONST) return fail("generated row schedule: op of two constants");
      }
      r.out_ord = out_ord[i];
      r.out_dtype = out_dtype[i];
      nodes.push_back(r);
    }
    if (views.size() > 24) return fail("generated row schedule: more than 24 distinct operand views");
    if (mma_out >= 0 && mma_in < 0) return fail("generated row schedule: a consuming dot without a producing one (the block-composed template is built around the first dot's tile)");
    if (mma_in >= 0) {
      if (n_col > 0) return fail("generated row schedule: column reductions beside dots on the matrix unit");
      if (S[1] > 128 || S[2] > 128) return fail("generated row schedule: dots on the matrix unit are fine-grained (tile up to 128 x 128)");
      if (S[1] == 0 || S[2] == 0) return fail("generated row schedule: empty tile of a matrix-unit dot");
      if (S[2] % 4 != 0) return fail("generated row schedule: the tile of a matrix-unit dot must be a multiple of 4 wide");
      for (const RNode& r : nodes) if (r.op == ROP_DOT_OUTER || r.op == ROP_DOT_REDUCE) return fail("generated row schedule: register dots beside dots on the matrix unit");
    }
    // a rounding read by nothing but the store of the same dtype is left to the store
    std::vector<char> read(n, 0);
    for (const RNode& r : nodes)
      for (int j = 0; j < r.nop; ++j) if (r.o[j].kind == OP_NODE || r.o[j].kind == OP_ROWB) read[r.o[j].index] = 1;
    for (const RNode& r : nodes)
      if (r.cls == CLS_DOT_OUT && r.out_ord < 0 && !read[r.id]) return fail("generated row schedule: a value computed after the consuming dot that nothing reads");
    for (RNode& r : nodes) {
      const bool rounds = (r.op == EW_OP_ROUND_F16 && r.out_dtype == FS_F16) || (r.op == EW_OP_ROUND_BF16 && r.out_dtype == FS_BF16);
      if (rounds && r.out_ord >= 0 && !read[r.id]) r.op = EW_OP_COPY;
    }
    // ... and one read by nothing but the consuming dot is left to the packing of the dot's operand
    if (mma_out >= 0) {
      std::vector<int> readers(n, 0), by_dot(n, 0);
      for (const RNode& r : nodes)
        for (int j = 0; j < r.nop; ++j) if (r.o[j].kind == OP_NODE || r.o[j].kind == OP_ROWB) {
          ++readers[r.o[j].index];
          if (r.op == ROP_DOT_MMA_OUT) ++by_dot[r.o[j].index];
        }
      for (RNode& r : nodes) {
        const bool rounds = (r.op == EW_OP_ROUND_F16 && mma_dtype == FS_F16) || (r.op == EW_OP_ROUND_BF16 && mma_dtype == FS_BF16);
        if (rounds && r.cls == CLS_FULL && r.out_ord < 0 && readers[r.id] > 0 && readers[r.id] == by_dot[r.id]) r.op = EW_OP_COPY;
      }
    }
    return true;
  }
};

struct Emitter {
  std::string s;
  void line(const char* fmt, ...) __attribute__((format(printf, 2, 3))) {
    char buf[1024];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    s += buf;
    s += '\n';
  }
};

// wave64 all-reduce over aligned groups of L lanes: DPP inside a 16-lane row, the gfx950
// permlane swaps across rows; every lane of the wavefront must be active
const char* kReducePreamble = R"SRC(
// the value of lane (own ^ mask) of a double, as two 32-bit permutes
static __device__ __forceinline__ double shfl_xor_f64(double v, int mask) {
  const int lane = __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
  const int addr = (lane ^ mask) << 2;
  const unsigned long long u = __builtin_bit_cast(unsigned long long, v);
  const unsigned lo = (unsigned)__builtin_amdgcn_ds_bpermute(addr, (int)(unsigned)u);
  const unsigned hi = (unsigned)__builtin_amdgcn_ds_bpermute(addr, (int)(unsigned)(u >> 32));
  return __builtin_bit_cast(double, ((unsigned long long)hi << 32) | lo);
}
template <int CTRL> static __device__ __forceinline__ float dpp_move(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, false));
}
struct std_true { static constexpr bool value = true; };      // compile-time switches handed to generic lambdas
struct std_false { static constexpr bool value = false; };
struct SumOp { static __device__ __forceinline__ float apply(float a, float b) { return a + b; } };
struct MaxOp { static __device__ __forceinline__ float apply(float a, float b) { return fmaxf(a, b); } };
template <class Op, int L> static __device__ __forceinline__ float lanes_allreduce(float v) {
  if (L >= 2) v = Op::apply(v, dpp_move<0xB1>(v));
  if (L >= 4) v = Op::apply(v, dpp_move<0x4E>(v));
  if (L >= 8) v = Op::apply(v, dpp_move<0x141>(v));
  if (L >= 16) v = Op::apply(v, dpp_move<0x140>(v));
  if (L >= 32) {
    const unsigned u = f32_bits(v);
    const auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    const unsigned lo = r[0], hi = r[1];
    v = Op::apply(bits_f32(lo), bits_f32(hi));
  }
  if (L >= 64) {
    const unsigned u = f32_bits(v);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    const unsigned lo = r[0], hi = r[1];
    v = Op::apply(bits_f32(lo), bits_f32(hi));
  }
  return v;
}
)SRC";

// what the block-composed template around matrix-unit dots adds: the MFMA wrappers (fp32 accumulate),
// the all-reduce over the four lanes that share an accumulator row, the transposing LDS read
const char* kMmaPreamble = R"SRC(
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
static __device__ __forceinline__ f32x4 mma_f16(u32x4 a, u32x4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}
static __device__ __forceinline__ f32x4 mma_bf16(u32x4 a, u32x4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}
// the value of lanes c, c+16, c+32, c+48 combined, in all four
template <class Op> static __device__ __forceinline__ float rows_allreduce(float v) {
  unsigned u = f32_bits(v);
  auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  unsigned lo = r[0], hi = r[1];
  v = Op::apply(bits_f32(lo), bits_f32(hi));
  u = f32_bits(v);
  r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  lo = r[0]; hi = r[1];
  return Op::apply(bits_f32(lo), bits_f32(hi));
}
// eight 16-bit values read through the transposing LDS read of gfx950, twice four: lane c of a 16-lane group
// receives column c of the 4 x 16 tile whose rows the group's lanes address in fours
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
static __device__ __forceinline__ u32x4 lds_read_transposed(const unsigned short* p, int second) {
  const u32x2 lo = __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p)));
  const u32x2 hi = __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + second)));
  return u32x4{lo[0], lo[1], hi[0], hi[1]};
}
)SRC";

std::string const_text(float c) {
  uint32_t u;
  memcpy(&u, &c, 4);
  char buf[40];
  snprintf(buf, sizeof buf, "bits_f32(0x%08xu)", u);
  return buf;
}


std::string op_text(int op, const std::string& a, const std::string& b, bool fast) {
  switch (op) {
    case FS_ADD: return a + " + " + b;
    case FS_SUBTRACT: return a + " - " + b;
    case FS_MULTIPLY: return a + " * " + b;
    case FS_DIVIDE: return a + " / " + b;
    case FS_MAXIMUM: return "fmaxf(" + a + ", " + b + ")";
    case FS_NEGATE: return "-" + a;
    case FS_EXP: return (fast ? "exp_fast(" : "expf(") + a + ")";
    case FS_LOG: return "logf(" + a + ")";
    case FS_TANH: return (fast ? "tanh_fast(" : "tanh_f32(") + a + ")";
    case FS_RSQRT: return "rsqrtf(" + a + ")";
    case FS_SQRT: return "sqrtf(" + a + ")";
    case FS_ERF: return (fast ? "erf_fast(" : "erff(") + a + ")";
    case FS_LOGISTIC: return "logistic(" + a + ")";
    case EW_OP_ROUND_F16: return "round_f16(" + a + ")";
    case EW_OP_ROUND_BF16: return "round_bf16(" + a + ")";
    default: return a;
  }
}

// Elements per 16-byte (or narrower) access of the full values, shared by the register and the
// streamed templates: 8 when every full tensor is 16-bit, else 4, narrower when the row length or
// an operand's strides and offset do not divide; 0 when an operand is strided along the last dim.
// *fast: some tensor of the group is 16-bit (the short forms of tanh and erf are accurate enough).
int chunk_elements(const Analysis& A, bool* fast) {
  bool any32 = false, any16 = false;
  for (const RView& v : A.views) {
    if (v.dtype != FS_F32) any16 = true;
    if (v.cls == CLS_FULL && v.stride[A.rank - 1] == 1 && v.dtype == FS_F32) any32 = true;
  }
  for (const RNode& n : A.nodes) if (n.out_ord >= 0) {
    if (n.out_dtype != FS_F32) any16 = true;
    if (n.cls == CLS_FULL && n.out_dtype == FS_F32) any32 = true;
  }
  *fast = any16;
  auto fits = [&](int w) {
    if (A.cols % w) return false;
    for (const RView& v : A.views) {
      if (v.cls != CLS_FULL) continue;
      const int64_t ls = v.stride[A.rank - 1];
      if (ls != 0 && ls != 1) return false;
      if (ls == 1) for (int d = 0; d + 1 < A.rank; ++d) if (v.stride[d] % w) return false;
      if (ls == 1 && v.offset % w) return false;
    }
    return true;
  };
  if (!any32 && fits(8)) return 8;
  if (fits(4)) return 4;
  if (fits(2)) return 2;
  if (fits(1)) return 1;
  return 0;
}

struct Gen {
  const Analysis& A;
  int L = 64, K = 1, W = 4;
  bool exact = true;          // K*L chunks cover the row exactly
  bool fast = false;          // 16-bit group: short tanh
  std::vector<int> splat;     // per view: 1 if one scalar per row (last stride 0 or row view)
  Emitter e;

  explicit Gen(const Analysis& a) : A(a) {}

  std::string opnd(const Opnd& o, int consumer_cls) const {
    char buf[64];
    if (consumer_cls == CLS_DOT_OUT) {
      // values after the consuming dot: D2 / 16 tiles of four consecutive columns per lane
      switch (o.kind) {
        case OP_NODE: snprintf(buf, sizeof buf, "d%d[dt][i]", o.index); return buf;
        case OP_ROWB: snprintf(buf, sizeof buf, "r%d", o.index); return buf;
        case OP_VIEW: snprintf(buf, sizeof buf, A.views[o.index].stride[2] == 0 ? "ws%d" : "w%d[dt][i]", o.index); return buf;
        default: return const_text(o.cval);
      }
    }
    switch (o.kind) {
      case OP_NODE: snprintf(buf, sizeof buf, consumer_cls == CLS_FULL ? "t%d[k][j]" : "r%d", o.index); return buf;
      case OP_ROWB: snprintf(buf, sizeof buf, "r%d", o.index); return buf;
      case OP_VIEW: snprintf(buf, sizeof buf, splat[o.index] ? "s%d" : "v%d[k][j]", o.index); return buf;
      default: return const_text(o.cval);
    }
  }
  std::string expr(const RNode& n) const {
    const std::string a = opnd(n.o[0], n.cls), b = n.nop == 2 ? opnd(n.o[1], n.cls) : std::string();
    // a full value divided by a per-row value: one reciprocal per row, then multiplies
    if (n.op == FS_DIVIDE && (n.cls == CLS_FULL || n.cls == CLS_DOT_OUT) && n.o[1].kind == OP_ROWB) return a + " * inv" + std::to_string(n.o[1].index);
    if (n.op == FS_CAUSAL_MASK) return "(col[k] + j <= irow) ? " + a + " : " + const_text(n.o[1].cval);
    if (n.op == EW_OP_GELU_TANH) return "gelu_tanh(" + a + ", " + const_text(n.gelu[0]) + ", " + const_text(n.gelu[1]) + ", " + const_text(n.gelu[2]) + ")";
    return op_text(n.op, a, b, fast);
  }

  // offset of the row's first element in a view: "row * c" if the row strides are those of
  // a dense tensor scaled by a constant, else from the row's coordinates
  std::string row_offset(const RView& v, bool* needs_coords, const char* rowvar = "row") const {
    const int nrow = A.rank - 1;
    char buf[160];
    if (nrow == 0) { snprintf(buf, sizeof buf, "%lldll", (long long)v.offset); return buf; }
    const int64_t unit = v.stride[nrow - 1];
    bool linear = true;
    int64_t mul = 1;
    for (int d = nrow - 1; d >= 0; --d) {
      if (A.S[d] != 1 && v.stride[d] != unit * mul) linear = false;
      mul *= A.S[d];
    }
    if (linear) {
      if (unit == 0) snprintf(buf, sizeof buf, "%lldll", (long long)v.offset);
      else snprintf(buf, sizeof buf, "%s * %lldll + %lldll", rowvar, (long long)unit, (long long)v.offset);
      return buf;
    }
    *needs_coords = true;
    std::string off;
    for (int d = 0; d < nrow; ++d) {
      if (v.stride[d] == 0 || A.S[d] == 1) continue;
      snprintf(buf, sizeof buf, "%si%d * %lldll", off.empty() ? "" : " + ", d, (long long)v.stride[d]);
      off += buf;
    }
    snprintf(buf, sizeof buf, "%s%lldll", off.empty() ? "" : " + ", (long long)v.offset);
    return off + buf;
  }

  int lanes_per_row = 0;      // 0: choose
  int wg = 256;               // workgroup size the kernel is generated for
  bool persistent = false;    // a fixed grid loops over the rows (groups with column reductions, or on request)
  bool want_persistent = false;
  int seg_groups = 0;         // column sums per run of rows: workgroups that share one run (1: results are stored directly)
  bool seg_per_wave = false;  // ... or every wavefront has a run of its own (many short runs): no LDS, no barrier
  bool stage = false;         // full outputs leave through an LDS staging tile (see emit)
  int64_t stage_bytes = 0;

  // Row steps requested ahead in the persistent form: one, or two (FS_ROW_PREFETCH=2): two row buffers per
  // streamed operand, the row loop unrolled twice so that each keeps its registers, and a buffer requested
  // again - for two steps ahead - as soon as its row has been taken out of it.  (Shifting the buffers down at
  // the end of an iteration instead makes the iteration wait for the request it has just issued.)
  int force_prefetch = 0;     // 1 or 2: the caller's choice
  int prefetch_depth(int n_prefetched) const {
    (void)n_prefetched;
    if (force_prefetch == 2 && A.seg_rows == 0 && L <= 64) return 2;
    return 1;
  }

  // ---- block composition around dots on the matrix unit (Section 5.1; DotGen of Section 5.3): one
  // workgroup per batch element, one wavefront per 16 rows of the tile.  The producing dot is computed
  // transposed (tile kt = b_kt . a^T), so lane (c, g) = (l % 16, l / 16) holds elements 16kt + 4g .. +3
  // of row c: in the terms of the register templates a row is spread over L = 4 lanes (g) with K = key
  // tiles chunks of W = 4 -- every elementwise op, reduction, load and store of those templates applies
  // unchanged, only the lanes of a row are 16 apart instead of adjacent.  The consuming dot takes the
  // lanes' values as its B fragments (keys inside a 32-step in the order the accumulators imply) and its
  // second operand transposed through LDS, in a buffer placed by the shared-memory planner.
  bool mma = false;
  int NQ = 1;                 // wavefronts = 16-row tiles of the tile's rows
  int64_t mma_lds_bytes = 0, mma_vt_offset = 0, mma_k_offset = 0;
  int mma_vp = 0, mma_kp = 0;              // padded row lengths (16-bit elements) of the two operands in LDS
  static int pow2_tiles(int64_t len) {
    const int need = (int)((len + 15) / 16);
    return need <= 1 ? 1 : need <= 2 ? 2 : need <= 4 ? 4 : 8;
  }
  bool geometry_mma(std::string* err) {
    mma = true;
    const int w = chunk_elements(A, &fast);
    if (w < 4) { *err = "generated row schedule: an operand of a matrix-unit group is not readable in 16-byte pieces of 4 elements"; return false; }
    fast = true;
    W = 4; L = 4;
    NQ = pow2_tiles(A.S[1]);
    K = pow2_tiles(A.S[2]);
    exact = (int64_t)K * 16 == A.cols;
    wg = 64 * NQ;
    if (A.mma_out >= 0) {
      // the LDS hand-off of the consuming dot (its second operand, transposed), placed by Algorithm 4
      const int NKP = K < 2 ? 2 : K;
      mma_vp = padded_row((int)A.mma_d, 8);
      const int n = (int)A.nodes.size();
      SharedPlanInput in;
      in.operands.resize(n);
      in.req_bytes.assign(n, 0);
      in.is_output.assign(n, 0);
      std::vector<int> idx_of(A.g.size(), -1);
      for (int i = 0; i < n; ++i) idx_of[A.nodes[i].id] = i;
      int at = -1;
      for (int i = 0; i < n; ++i) {
        const RNode& x = A.nodes[i];
        for (int j = 0; j < x.nop; ++j)
          if (x.o[j].kind == OP_NODE || x.o[j].kind == OP_ROWB) in.operands[i].push_back(idx_of[x.o[j].index]);
        if (x.out_ord >= 0) in.is_output[i] = 1;
        if (x.op == ROP_DOT_MMA_OUT) { in.req_bytes[i] = 2 * (int64_t)NKP * 16 * mma_vp; at = i; }
      }
      const SharedPlanResult r = shared_plan(in);
      mma_vt_offset = r.offset[at];
      mma_lds_bytes = r.total_bytes;
    }
    // the producing dot's second operand, shared by the workgroup's wavefronts: rows of whole 32-steps plus 8
    mma_k_offset = (mma_lds_bytes + 15) / 16 * 16;
    if (A.mma_b_kn) {
      // stored [K, N]: in LDS as stored, whole 32-steps of rows (zero beyond K), read back transposed like v
      mma_kp = padded_row(K * 16, 8);
      mma_lds_bytes = mma_k_offset + 2 * (int64_t)((A.mma_k + 31) / 32) * 32 * mma_kp;
    } else {
      mma_kp = ((int)((A.mma_k + 31) / 32)) * 32 + 8;
      mma_lds_bytes = mma_k_offset + 2 * (int64_t)K * 16 * mma_kp;
    }
    return true;
  }
  // Row length in 16-bit elements of an LDS tile that is read four rows at a time, `piece` bytes per lane and four
  // lanes per row (the transposing read): the shortest padding that is a multiple of 16 bytes and puts the four
  // rows of one access on different banks (64 banks of 4 bytes).
  static int padded_row(int width, int piece) {
    for (int pad = 8; pad <= 64; pad += 8) {
      const int banks = (width + pad) / 2, span = 4 * piece / 4;
      bool clash = false;
      for (int a = 0; a < 4 && !clash; ++a)
        for (int b = a + 1; b < 4 && !clash; ++b) {
          const int d = (((b - a) * banks) % 64 + 64) % 64;
          if (d < span || 64 - d < span) clash = true;
        }
      if (!clash) return width + pad;
    }
    return width + 8;
  }

  bool geometry(std::string* err) {
    if (A.mma_in >= 0) return geometry_mma(err);
    W = chunk_elements(A, &fast);
    if (W == 0) { *err = "generated row schedule: an operand strided along the last dim"; return false; }
    const int64_t nvec = A.cols / W;
    auto pow2_at_least = [](int64_t v) { int p = 1; while (p < v && p < 64) p *= 2; return p; };
    if (lanes_per_row > 0) {
      // the caller's template
      L = lanes_per_row;
    } else if (W == 1 && nvec <= 32) {
      // a short row that cannot be read in vectors: one thread per row, sequential reduction
      // (the THREAD template)
      L = 1;
    } else if (nvec <= 16) {
      // short rows: one chunk per lane, so that consecutive lanes read consecutive memory
      // across row boundaries
      L = pow2_at_least(nvec);
    } else {
      // the fewest lanes that keep at most 16 elements of a value per lane
      L = 2;
      while (L < 64 && (nvec + L - 1) / L > 16 / W) L *= 2;
      // ... unless that leaves a lane with fewer than four 16-byte loads in flight (one streamed operand of
      // 2-byte elements: two): then half the lanes with twice the pieces each (RMSNorm over 16384 x 1024
      // bf16: 13.1 -> 12.1 us)
      int streamed = 0;
      for (const RView& vw : A.views) {
        bool per_row = false;                        // (a per-column operand is a full view with zero row strides)
        for (int d = 0; d + 1 < A.rank; ++d) if (vw.stride[d] != 0) per_row = true;
        if (vw.cls == CLS_FULL && per_row) ++streamed;
      }
      const int64_t k0 = (nvec + L - 1) / L;
      if (fast && L >= 32 && streamed * k0 < 4 && 2 * k0 * W <= 32 && nvec % (L / 2) == 0) L /= 2;
    }
    K = (int)((nvec + L - 1) / L);
    // a row too long for one wavefront's registers goes to a team of wavefronts (one
    // workgroup per row)
    while (lanes_per_row == 0 && (int64_t)K * W > 32 && L < 1024) { L *= 2; K = (int)((nvec + L - 1) / L); }
    if ((int64_t)K * W > 32) {
      *err = lanes_per_row > 0 ? "generated row schedule: too few lanes per row for this row length"
                               : "generated row schedule: row longer than 32768 elements";
      return false;
    }
    exact = (int64_t)K * L == nvec;
    // Short rows that do not fill whole 128-byte lines: a workgroup's rows are contiguous in
    // memory, so its full outputs are first laid out in LDS and then stored as one dense run
    // of 16-byte accesses (stores of separate row pieces straddle lines and measured 2x slower).
    if (A.n_col > 0) {
      if (L > 64) {
        // a team of wavefronts per row: every lane's columns are its own in the workgroup, so the
        // running sums (two registers per column and reduction) stay few by spreading the row wider
        while ((int64_t)K * W * A.n_col > 16 && L < 1024) { L *= 2; K = (int)((nvec + L - 1) / L); }
        if ((int64_t)K * W * A.n_col > 16) { *err = "generated row schedule: column reductions over rows too long for their running sums to stay in registers"; return false; }
        exact = (int64_t)K * L == nvec;
      } else if ((int64_t)A.n_col * A.cols * 8 > 96 * 1024) {
        *err = "generated row schedule: column accumulators exceed the LDS";
        return false;
      }
      persistent = true;
    }
    if (L > 64) wg = L;                       // a team is one workgroup
    if (want_persistent && L <= 64) persistent = true;
    if (L <= 64 && !persistent) {
      int min_out = 4;
      bool full_out = false;
      for (const RNode& n : A.nodes) if (n.out_ord >= 0 && n.cls == CLS_FULL) { full_out = true; if (n.out_dtype != FS_F32) min_out = 2; }
      const int64_t row_bytes = A.cols * min_out;
      const int64_t tile = (int64_t)(wg / L) * A.cols * 4;
      // (the dense run starts 16-byte aligned when a workgroup's element count is a multiple of 4)
      stage = full_out && row_bytes % 128 != 0 && row_bytes < 2048 && tile <= 32 * 1024 && ((int64_t)(wg / L) * A.cols) % 4 == 0;
      stage_bytes = stage ? tile : 0;
    }
    return true;
  }

  // The consuming dot's second operand v[B, N, D]: every thread's 16-byte chunks are requested at the top
  // of the kernel, long before the LDS transpose needs them.
  void emit_mma_v_loads() {
    const int D2 = (int)A.mma_d, NKP = K < 2 ? 2 : K, CH = D2 / 8, VTOT = NKP * 16 * CH, NV = (VTOT + wg - 1) / wg;
    e.line("  constexpr int D2 = %d, NKP = %d, CH = %d, VTOT = %d, NV = %d, VP = %d;", D2, NKP, CH, VTOT, NV, mma_vp);
    e.line("  u32x4 vreg[NV];");
    e.line("  {");
    e.line("    const unsigned short* vb = static_cast<const unsigned short*>(a.in[%d]) + (long long)blockIdx.x * N * D2;", A.mma_vv);
    e.line("    UNROLL for (int i = 0; i < NV; ++i) {");
    e.line("      int ci = (int)threadIdx.x + i * %d; if (ci > VTOT - 1) ci = VTOT - 1;", wg);
    e.line("      int key = ci / CH; if (key > N - 1) key = N - 1;");
    e.line("      vreg[i] = *reinterpret_cast<const u32x4*>(vb + (long long)key * D2 + (ci %% CH) * 8);");
    e.line("    }");
    e.line("  }");
  }

  // The producing dot's second operand when it is stored [B, KC, N]: every thread's pieces of the batch element's
  // slab are requested at the top of the kernel (8 elements where rows start on 16 bytes, else 4).
  void emit_mma_b_loads() {
    const int KC = (int)A.mma_k, VE = A.S[2] % 8 == 0 ? 8 : 4, CHB = (int)((A.S[2] + VE - 1) / VE), BTOT = KC * CHB, NB = (BTOT + wg - 1) / wg;
    e.line("  constexpr int VE = %d, CHB = %d, BTOT = %d, NB = %d;", VE, CHB, BTOT, NB);
    e.line("  %s breg[NB];", VE == 8 ? "u32x4" : "u32x2");
    e.line("  {");
    e.line("    const unsigned short* bb = static_cast<const unsigned short*>(a.in[%d]) + (long long)blockIdx.x * %lldll;", A.mma_vb, (long long)(A.mma_k * A.S[2]));
    e.line("    UNROLL for (int i = 0; i < NB; ++i) {");
    e.line("      int ci = (int)threadIdx.x + i * %d; if (ci > BTOT - 1) ci = BTOT - 1;", wg);
    e.line("      breg[i] = *reinterpret_cast<const %s*>(bb + (long long)(ci / CHB) * N + (ci %% CHB) * VE);", VE == 8 ? "u32x4" : "u32x2");
    e.line("    }");
    e.line("  }");
  }

  // The producing dot, transposed: tile k = b_k(16 x KC) . a^T, so the lane holds t[k][j] = row `row`,
  // column 16k + 4*lane + j.  Fragments of a come straight from global memory in MFMA layout (8 consecutive
  // contraction indices of one row: one 16-byte load).  Every 16-row tile of b is loaded that way by ONE
  // wavefront and handed to the others through LDS; steps beyond KC are zero on both sides.  The consuming
  // dot's second operand goes to LDS as stored behind the same barrier.
  void emit_mma_in(const RNode& n) {
    const int KC = (int)A.mma_k, KS = (KC + 31) / 32, KT = (K + NQ - 1) / NQ;
    const bool kn = A.mma_b_kn;
    const char* mm = A.mma_dtype == FS_F16 ? "mma_f16" : "mma_bf16";
    e.line("  float t%d[K][W];", n.id);
    e.line("  {");
    e.line("    constexpr int KC = %d, KS = %d, KT = %d, KP = %d;", KC, KS, KT, mma_kp);
    e.line("    const int wv = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));");
    e.line("    const unsigned short* pa = static_cast<const unsigned short*>(a.in[%d]) + row * KC;", A.mma_va);
    if (!kn) e.line("    const unsigned short* pb = static_cast<const unsigned short*>(a.in[%d]) + (long long)blockIdx.x * N * KC;", A.mma_vb);
    e.line("    unsigned short* ksh = reinterpret_cast<unsigned short*>(lds_pool + %lld);   // %s", (long long)mma_k_offset,
           kn ? "[KS * 32][KP]: as stored, rows = contraction index" : "[K * 16][KP]");
    e.line("    u32x4 qf[KS];");
    e.line("    UNROLL for (int ks = 0; ks < KS; ++ks) {");
    e.line("      const int k0 = ks * 32 + 8 * lane;");
    e.line("      qf[ks] = k0 < KC ? *reinterpret_cast<const u32x4*>(pa + k0) : u32x4{0u, 0u, 0u, 0u};");
    e.line("    }");
    if (!kn) {
      e.line("    u32x4 kf[KT][KS];");
      e.line("    UNROLL for (int j = 0; j < KT; ++j) {");
      e.line("      const int kt = wv + j * %d;", NQ);
      e.line("      int nrow = 16 * kt + lane16; if (nrow > N - 1) nrow = N - 1;");
      e.line("      UNROLL for (int ks = 0; ks < KS; ++ks) {");
      e.line("        const int k0 = ks * 32 + 8 * lane;");
      e.line("        kf[j][ks] = u32x4{0u, 0u, 0u, 0u};");
      e.line("        if (kt < K && k0 < KC) kf[j][ks] = *reinterpret_cast<const u32x4*>(pb + (long long)nrow * KC + k0);");
      e.line("      }");
      e.line("    }");
      e.line("    asm volatile(\"\" ::: \"memory\");     // every request above is issued before the first wait below");
      e.line("    UNROLL for (int j = 0; j < KT; ++j) {");
      e.line("      const int kt = wv + j * %d;", NQ);
      e.line("      if (kt < K) { UNROLL for (int ks = 0; ks < KS; ++ks) *reinterpret_cast<u32x4*>(ksh + (16 * kt + lane16) * KP + ks * 32 + 8 * lane) = kf[j][ks]; }");
      e.line("    }");
    } else {
      e.line("    (void)wv;");
      e.line("    asm volatile(\"\" ::: \"memory\");     // every request above is issued before the first wait below");
      // the slab as stored; what the matrix instructions read beyond it (columns N .. 16 K of every row, rows KC .. 32 KS) is zero
      e.line("    UNROLL for (int i = 0; i < NB; ++i) {");
      e.line("      const int ci = (int)threadIdx.x + i * %d;", wg);
      e.line("      if (ci < BTOT) *reinterpret_cast<%s*>(ksh + (ci / CHB) * KP + (ci %% CHB) * VE) = breg[i];", A.S[2] % 8 == 0 ? "u32x4" : "u32x2");
      e.line("    }");
      e.line("    constexpr int PADC = (16 * K - N) / 4;         // 4-element pieces right of the slab, per row");
      e.line("    for (int i = threadIdx.x; i < KC * PADC; i += %d) *reinterpret_cast<u32x2*>(ksh + (i / (PADC > 0 ? PADC : 1)) * KP + N + 4 * (i %% (PADC > 0 ? PADC : 1))) = u32x2{0u, 0u};", wg);
      e.line("    for (int i = threadIdx.x; i < (32 * KS - KC) * 4 * K; i += %d) *reinterpret_cast<u32x2*>(ksh + (KC + i / (4 * K)) * KP + 4 * (i %% (4 * K))) = u32x2{0u, 0u};", wg);
    }
    if (A.mma_out >= 0) {
      e.line("    unsigned short* vsh = reinterpret_cast<unsigned short*>(lds_pool + %lld);   // [NKP * 16][VP], rows beyond N zero", (long long)mma_vt_offset);
      e.line("    UNROLL for (int i = 0; i < NV; ++i) {");
      e.line("      const int cu = (int)threadIdx.x + i * %d;", wg);
      e.line("      const int ci = cu < VTOT - 1 ? cu : VTOT - 1;");
      e.line("      const int key = ci / CH;");
      e.line("      const u32x4 tv = key < N ? vreg[i] : u32x4{0u, 0u, 0u, 0u};");
      e.line("      if (cu < VTOT) *reinterpret_cast<u32x4*>(vsh + key * VP + (ci %% CH) * 8) = tv;");
      e.line("    }");
    }
    e.line("    __syncthreads();");
    if (kn) e.line("    const unsigned short* blane = ksh + (8 * lane + (lane16 >> 2)) * KP + 4 * (lane16 & 3);   // the transposing read: rows 8 lane .. + 7 of a 32-step");
    e.line("    UNROLL for (int k = 0; k < K; ++k) {");
    e.line("      u32x4 kr[KS];");
    if (kn) e.line("      UNROLL for (int ks = 0; ks < KS; ++ks) kr[ks] = lds_read_transposed(blane + 32 * ks * KP + 16 * k, 4 * KP);");
    else e.line("      UNROLL for (int ks = 0; ks < KS; ++ks) kr[ks] = *reinterpret_cast<const u32x4*>(ksh + (16 * k + lane16) * KP + ks * 32 + 8 * lane);");
    e.line("      f32x4 acc = {0.f, 0.f, 0.f, 0.f};");
    e.line("      UNROLL for (int ks = 0; ks < KS; ++ks) acc = %s(kr[ks], qf[ks], acc);", mm);
    e.line("      UNROLL for (int j = 0; j < W; ++j) t%d[k][j] = acc[j];", n.id);
    e.line("    }");
    e.line("  }");
  }

  // The consuming dot, transposed: O^T(D2 x 16) = V^T(D2 x keys) . P^T.  P is the operand's registers packed
  // to the dot dtype (keys beyond N are zero); V sits in LDS as stored and is read transposed, the keys of a
  // 32-step in the order the accumulators of the producing dot imply (k-slot 4h+i of lane group g: key
  // 32kk + 16h + 4g + i).
  void emit_mma_out(const RNode& n) {
    const char* mm = A.mma_dtype == FS_F16 ? "mma_f16" : "mma_bf16";
    const char* pk = A.mma_dtype == FS_F16 ? "pack_to_f16" : "pack_to_bf16";
    const int src = n.o[0].index;
    e.line("  f32x4 d%d[D2 / 16];", n.id);
    e.line("  {");
    e.line("    u32x4 pb2[NKP / 2];");
    e.line("    UNROLL for (int kk = 0; kk < NKP / 2; ++kk) UNROLL for (int h = 0; h < 2; ++h) {");
    e.line("      const int kt = 2 * kk + h;");
    e.line("      float p[4] = {0.f, 0.f, 0.f, 0.f};");
    e.line("      if (kt < K) { UNROLL for (int i = 0; i < 4; ++i) p[i] = ok[kt < K ? kt : 0] ? t%d[kt < K ? kt : 0][i] : 0.f; }", src);
    e.line("      pb2[kk][2 * h] = %s(p[0], p[1]);", pk);
    e.line("      pb2[kk][2 * h + 1] = %s(p[2], p[3]);", pk);
    e.line("    }");
    e.line("    const unsigned short* vlane = reinterpret_cast<const unsigned short*>(lds_pool + %lld) + (4 * lane + (lane16 >> 2)) * VP + 4 * (lane16 & 3);", (long long)mma_vt_offset);
    e.line("    UNROLL for (int dt = 0; dt < D2 / 16; ++dt) d%d[dt] = f32x4{0.f, 0.f, 0.f, 0.f};", n.id);
    e.line("    UNROLL for (int kk = 0; kk < NKP / 2; ++kk) UNROLL for (int dt = 0; dt < D2 / 16; ++dt) {");
    e.line("      const u32x4 vf = lds_read_transposed(vlane + 32 * kk * VP + 16 * dt, 16 * VP);");
    e.line("      d%d[dt] = %s(vf, pb2[kk], d%d[dt]);", n.id, mm, n.id);
    e.line("    }");
    e.line("  }");
    if (n.out_ord >= 0) store_dot_out(n);
  }

  // A [B, M, D] value in the accumulators' layout (lane g of a row holds columns 16 dt + 4 g .. + 3 of every
  // 16-column tile dt) to its output.
  void store_dot_out(const RNode& n) {
    e.line("  {");
    if (n.out_dtype == FS_F32) {
      e.line("    float* orow = static_cast<float*>(a.out[%d]) + row * D2 + 4 * lane;", n.out_ord);
      e.line("    if (row_ok) { UNROLL for (int dt = 0; dt < D2 / 16; ++dt) __builtin_nontemporal_store(d%d[dt], reinterpret_cast<f32x4*>(orow + 16 * dt)); }", n.id);
    } else {
      const char* po = n.out_dtype == FS_F16 ? "pack_to_f16" : "pack_to_bf16";
      // 8 bytes per tile and lane; lanes g and g^1 trade one tile of a pair so that each stores 16 bytes
      e.line("    unsigned short* orow = static_cast<unsigned short*>(a.out[%d]) + row * D2 + 16 * (lane & 1) + 8 * (lane >> 1);", n.out_ord);
      e.line("    UNROLL for (int dp = 0; dp < D2 / 32; ++dp) {");
      e.line("      const unsigned a0 = %s(d%d[2 * dp][0], d%d[2 * dp][1]), a1 = %s(d%d[2 * dp][2], d%d[2 * dp][3]);", po, n.id, n.id, po, n.id, n.id);
      e.line("      const unsigned b0 = %s(d%d[2 * dp + 1][0], d%d[2 * dp + 1][1]), b1 = %s(d%d[2 * dp + 1][2], d%d[2 * dp + 1][3]);", po, n.id, n.id, po, n.id, n.id);
      e.line("      const auto r0 = __builtin_amdgcn_permlane16_swap(a0, b0, false, false);");
      e.line("      const auto r1 = __builtin_amdgcn_permlane16_swap(a1, b1, false, false);");
      e.line("      const unsigned x0 = r0[0], x1 = r1[0], x2 = r0[1], x3 = r1[1];");
      e.line("      if (row_ok) *reinterpret_cast<u32x4*>(orow + dp * 32) = u32x4{x0, x1, x2, x3};");
      e.line("    }");
    }
    e.line("  }");
  }

  // Inputs read by the ops after the consuming dot, in the accumulators' layout: requested at the top of the
  // kernel (they depend on nothing), used at the end.
  void emit_dot_out_view_loads() {
    for (size_t q = 0; q < A.views.size(); ++q) {
      const RView& v = A.views[q];
      if (v.cls != CLS_DOT_OUT) continue;
      const char* ty = v.dtype == FS_F32 ? "float" : "unsigned short";
      e.line("  const %s* wp%zu = static_cast<const %s*>(a.in[%zu]) + (long long)blockIdx.x * %lldll + (long long)(row_ok ? mrow : M - 1) * %lldll;",
             ty, q, ty, q, (long long)v.stride[0], (long long)v.stride[1]);
      if (v.stride[2] == 0) {
        e.line("  const float ws%zu = %s;", q, v.dtype == FS_F32 ? ("wp" + std::to_string(q) + "[0]").c_str()
                                                 : ((v.dtype == FS_F16 ? "f16_lo(wp" : "bf16_lo(wp") + std::to_string(q) + "[0])").c_str());
        continue;
      }
      e.line("  f32x4 w%zu[D2 / 16];", q);
      if (v.dtype == FS_F32) {
        e.line("  UNROLL for (int dt = 0; dt < D2 / 16; ++dt) w%zu[dt] = *reinterpret_cast<const f32x4*>(wp%zu + 16 * dt + 4 * lane);", q, q);
      } else {
        const char* lo = v.dtype == FS_F16 ? "f16_lo" : "bf16_lo";
        const char* hi = v.dtype == FS_F16 ? "f16_hi" : "bf16_hi";
        e.line("  UNROLL for (int dt = 0; dt < D2 / 16; ++dt) {");
        e.line("    const u32x2 x = *reinterpret_cast<const u32x2*>(wp%zu + 16 * dt + 4 * lane);", q);
        e.line("    w%zu[dt] = f32x4{%s(x[0]), %s(x[0]), %s(x[1]), %s(x[1])};", q, lo, hi, lo, hi);
        e.line("  }");
      }
    }
  }

  void emit(std::string* kernel_name) {
    const int rank = A.rank, nrow = rank - 1;
    std::string advance;        // persistent form: hand the prefetched vectors to the next iteration
    bool rotating = false;      // persistent form whose row buffers take turns (row loop unrolled over them)
    int rot_buffers = 2;        // ... how many
    std::string pro_req;        // ... the requests of the rows the loop starts with
    std::string deferred_head;  // ... and the text that goes between what is loaded once and the loop
    std::string loop_anchor = "  for (long long row0 = ";   // the text the row loop starts with: what is loaded once goes before it
    e.s = ew_preamble();
    e.s += kReducePreamble;
    if (mma) e.s += kMmaPreamble;
    const int T = L > 64 ? L / 64 : 1;      // wavefronts per row
    // (matrix-unit kernels: two wavefronts per SIMD asked for, so that the register budget is the 256 ordinary
    // registers and the compiler keeps the accumulators there instead of copying through the accumulation file)
    e.line("extern \"C\" __global__ %s__launch_bounds__(%d) void FS_ROW_NAME(const Args a) {", mma ? "__attribute__((amdgpu_waves_per_eu(2))) " : "",
           mma ? wg : L > 256 ? L : wg > 256 ? wg : 256);
    e.line("  constexpr int L = %d, K = %d, W = %d;", L, K, W);
    if (mma) {
      e.line("  constexpr int M = %lld, N = %lld;             // the tile of one batch element", (long long)A.S[1], (long long)A.S[2]);
      e.line("  const int lane = (threadIdx.x & 63) >> 4;      // the lane's place among the four that share a row (accumulator layout)");
      e.line("  const int lane16 = threadIdx.x & 15;           // the row inside the wavefront's 16");
      e.line("  const int mrow = 16 * (int)(threadIdx.x >> 6) + lane16;");
      e.line("  const bool row_ok = mrow < M;");
      e.line("  long long row = (long long)blockIdx.x * M + (row_ok ? mrow : M - 1);   // idle lanes redo the last row and store nothing");
    } else if (T > 1) {
      // one workgroup of T wavefronts per row; every reduction has its own exchange slots, so one
      // barrier per reduction is enough
      e.line("  constexpr int T = %d;", T);
      if (A.n_reduce > 0) e.line("  __shared__ float exch[%d][T];", A.n_reduce);
      e.line("  const int lane = threadIdx.x;");
      if (!persistent) e.line("  long long row = blockIdx.x;");
    } else {
      e.line("  const int lane = threadIdx.x & (L - 1);");
      if (!persistent) e.line("  long long row = ((long long)blockIdx.x * blockDim.x + threadIdx.x) / L;");
    }
    if (stage) {
      e.line("  constexpr int RPW = %d, N = %lld;            // rows per workgroup, row length", wg / L, (long long)A.cols);
      e.line("  __shared__ float stage[RPW * N];");
      e.line("  const int row_local = threadIdx.x / L;");
      e.line("  const long long wg_row0 = (long long)blockIdx.x * RPW;");
      e.line("  const long long left = %lldll - wg_row0;", (long long)A.rows);
      e.line("  const int wg_count = (int)(left < RPW ? left : RPW) * N;   // elements this workgroup owns");
    }
    e.line("  int col[K]; bool ok[K];");
    e.line("  UNROLL for (int k = 0; k < K; ++k) { const int c = k * L + lane; ok[k] = c < %lld; col[k] = (ok[k] ? c : 0) * W; }",
           (long long)(A.cols / W));
    if (persistent) {
      // Column reductions: every lane keeps a double-precision running sum for each of its
      // columns while the workgroups loop over the rows; the sums of a workgroup meet in LDS
      // and leave as one partial row per workgroup (a second, tiny kernel adds the partial rows).
      for (const RNode& n : A.nodes) if (n.cls == CLS_COL) {
        e.line("  double ca%d[K][W];", n.id);
        e.line("  UNROLL for (int k = 0; k < K; ++k) UNROLL for (int j = 0; j < W; ++j) ca%d[k][j] = %s;", n.id, n.op == FS_REDUCE_MAX ? "-__builtin_inf()" : "0.0");
      }
      e.line("  constexpr int RPW = %d;                      // rows a workgroup handles at a time", wg / L);
      if (A.seg_rows > 0 && seg_per_wave) {
        // column sums per run of SEG consecutive rows, a run per wavefront (a wavefront past the last
        // run redoes the last one and stores nothing)
        e.line("  constexpr long long SEG = %lldll;", (long long)A.seg_rows);
        e.line("  long long seg = (long long)blockIdx.x * (blockDim.x / 64) + (threadIdx.x >> 6);");
        e.line("  const bool seg_ok = seg < %lldll;", (long long)(A.rows / A.seg_rows));
        e.line("  if (!seg_ok) seg = %lldll;", (long long)(A.rows / A.seg_rows) - 1);
        e.line("  const long long seg_lo = seg * SEG, seg_hi = seg_lo + SEG;");
        e.line("  const int rl = (threadIdx.x & 63) / L;          // the lane's row among those its wavefront covers at a time");
        e.line("  const long long first_row = seg_lo, row_step = 64 / L;");
        e.line("  for (long long row0 = first_row; row0 < seg_hi; row0 += row_step) {");
      } else if (A.seg_rows > 0) {
        // column sums per run of SEG consecutive rows: G consecutive workgroups share one run
        e.line("  constexpr long long SEG = %lldll; constexpr int G = %d;", (long long)A.seg_rows, seg_groups);
        e.line("  const long long seg = blockIdx.x / G, seg_lo = seg * SEG, seg_hi = seg_lo + SEG;");
        e.line("  const int rl = threadIdx.x / L;");
        e.line("  const long long first_row = seg_lo + (long long)(blockIdx.x %% G) * RPW, row_step = (long long)G * RPW;");
        e.line("  for (long long row0 = first_row; row0 < seg_hi; row0 += row_step) {");
      } else {
        e.line("  const int rl = threadIdx.x / L;");
        e.line("  const long long first_row = (long long)blockIdx.x * RPW, row_step = (long long)gridDim.x * RPW;");
        if (L <= 64) {
          // One step of the row loop as a function of the row buffer it works on (ph) and of whether every row
          // of the step exists (ALL): the loop below is unrolled over the buffers, which take turns without
          // ever being copied, and has a branch-free main part.
          rotating = true;
          loop_anchor = "  auto step = [&](auto all_c, const int ph, const long long row0) __attribute__((always_inline)) {";
          e.line("%s", loop_anchor.c_str());
          e.line("  constexpr bool ALL = decltype(all_c)::value;");
        } else {
          e.line("  for (long long row0 = first_row; row0 < %lldll; row0 += row_step) {", (long long)A.rows);
        }
      }
      e.line("  long long row = row0 + rl;");
    }
    char row_hi[32], row_last[40], row_any[32];     // end of the rows of this workgroup's loop, its last row, a row that is surely valid
    if (persistent && A.seg_rows > 0) {
      snprintf(row_hi, sizeof row_hi, "seg_hi"); snprintf(row_last, sizeof row_last, "(seg_hi - 1)"); snprintf(row_any, sizeof row_any, "seg_lo");
    } else {
      snprintf(row_hi, sizeof row_hi, "%lldll", (long long)A.rows); snprintf(row_last, sizeof row_last, "%lldll", (long long)A.rows - 1); snprintf(row_any, sizeof row_any, "0");
    }
    if (!mma) {
      e.line("  const bool row_ok = %srow < %s%s;", rotating ? "ALL || " : "", row_hi, persistent && A.seg_rows > 0 && seg_per_wave ? " && seg_ok" : "");
      e.line("  if (!row_ok) row = %s;   // idle lanes redo the last row and store nothing: cross-lane steps need every lane", row_last);
    }
    if (mma) e.line("  __shared__ __attribute__((aligned(16))) unsigned char lds_pool[%lld];", (long long)mma_lds_bytes);
    if (mma && A.mma_b_kn) emit_mma_b_loads();
    if (mma && A.mma_out >= 0) { emit_mma_v_loads(); emit_dot_out_view_loads(); }
    // which views need the row's coordinates
    splat.assign(A.views.size(), 0);
    std::vector<std::string> roff(A.views.size());
    bool coords = false;
    for (size_t q = 0; q < A.views.size(); ++q) {
      const RView& v = A.views[q];
      roff[q] = row_offset(v, &coords);
      splat[q] = v.cls == CLS_ROW || v.stride[rank - 1] == 0;
    }
    if (A.has_causal) coords = true;
    if (coords) {
      const bool small = A.rows <= 0x7fffffffLL;
      const char* ty = small ? "unsigned" : "unsigned long long";
      const char* sfx = small ? "u" : "ull";
      e.line("  %s rr = (%s)row;", ty, ty);
      for (int d = nrow - 1; d >= 0; --d) {
        if (A.S[d] == 1) { e.line("  const long long i%d = 0;", d); continue; }
        e.line("  const long long i%d = rr %% %lld%s; rr /= %lld%s;", d, (long long)A.S[d], sfx, (long long)A.S[d], sfx);
      }
      if (A.has_causal) e.line("  const long long irow = i%d;      // the row's index in the second-to-last dim", nrow - 1);
    }
    // ---- loads
    // In the persistent form the next row's vectors are requested before the current row is
    // worked on (raw, still packed) and unpacked one iteration later: with few wavefronts per
    // CU that is what keeps HBM requests in flight.
    auto raw_type = [&](const RView& v) -> const char* {
      if (v.dtype == FS_F32) return W == 4 ? "f32x4" : nullptr;
      return W == 8 ? "u32x4" : W == 4 ? "u32x2" : nullptr;
    };
    std::vector<char> prefetched(A.views.size(), 0);
    std::vector<char> scalar_prefetched(A.views.size(), 0);    // per-row scalars (one value per row) requested ahead like the rows
    if (persistent) {
      for (size_t q = 0; q < A.views.size(); ++q) {
        const RView& v = A.views[q];
        bool dense = true, needs_coords = false, varies = false;
        for (int d = 0; d < nrow; ++d) if (A.S[d] != 1 && v.stride[d] == 0) dense = false;
        for (int d = 0; d < nrow; ++d) if (A.S[d] != 1 && v.stride[d] != 0) varies = true;
        (void)row_offset(v, &needs_coords);
        prefetched[q] = !splat[q] && dense && !needs_coords && raw_type(v) != nullptr;
        scalar_prefetched[q] = splat[q] && varies && !needs_coords;
      }
    }
    if (persistent) {
      // Rows are requested ahead of the one being worked on.  Rotating form: `depth` steps ahead into
      // depth + 1 buffers raw<q>x[..] that take turns - step ph works on buffer ph and first requests the row
      // `depth` steps ahead into the buffer the step before it has finished with; no buffer is ever copied (a
      // copy of a buffer requested one step ago would wait for it).  Otherwise: one step ahead into nraw<q>,
      // handed to raw<q> at the end of the iteration.
      std::string pro, nxt, adv;
      char buf[640];
      int n_pref = 0;
      for (size_t q = 0; q < A.views.size(); ++q) n_pref += prefetched[q] ? 1 : 0;
      const int depth = rotating ? prefetch_depth(n_pref) : 1;
      const int nb = depth + 1;
      rot_buffers = nb;
      // A per-row scalar loaded where it is used would make every iteration wait for all requests issued
      // before it, the rows requested ahead included (loads complete in order): it is requested with them,
      // and first, because it is needed first.
      for (size_t q = 0; q < A.views.size(); ++q) if (scalar_prefetched[q]) {
        const RView& v = A.views[q];
        const char* ty = v.dtype == FS_F32 ? "float" : "unsigned short";
        const char* cv = v.dtype == FS_F32 ? "" : v.dtype == FS_F16 ? "f16_lo" : "bf16_lo";
        bool dummy = false;
        const std::string offp = row_offset(v, &dummy, "rowp"), offn = row_offset(v, &dummy, "rown");
        if (rotating) {
          snprintf(buf, sizeof buf, "  float sraw%zux[%d];\n", q, nb);
          pro += buf;
          snprintf(buf, sizeof buf, "    sraw%zux[pp] = %s((static_cast<const %s*>(a.in[%zu]) + (%s))[0]);\n", q, cv, ty, q, offp.c_str());
          pro_req += buf;
          snprintf(buf, sizeof buf, "  sraw%zux[(ph + %d) %% %d] = %s((static_cast<const %s*>(a.in[%zu]) + (%s))[0]);\n", q, depth, nb, cv, ty, q, offn.c_str());
          nxt += buf;
        } else {
          snprintf(buf, sizeof buf, "  float sraw%zu = %s((static_cast<const %s*>(a.in[%zu]) + (%s))[0]);\n", q, cv, ty, q, offp.c_str());
          pro += buf;
          snprintf(buf, sizeof buf, "  const float nsraw%zu = %s((static_cast<const %s*>(a.in[%zu]) + (%s))[0]);\n", q, cv, ty, q, offn.c_str());
          nxt += buf;
          snprintf(buf, sizeof buf, "  sraw%zu = nsraw%zu;\n", q, q);
          adv += buf;
        }
      }
      for (size_t q = 0; q < A.views.size(); ++q) if (prefetched[q]) {
        const RView& v = A.views[q];
        const char* ty = v.dtype == FS_F32 ? "float" : "unsigned short";
        const char* rt = raw_type(v);
        bool dummy = false;
        const std::string offp = row_offset(v, &dummy, "rowp"), offn = row_offset(v, &dummy, "rown");
        if (rotating) {
          snprintf(buf, sizeof buf, "  %s raw%zux[%d][K];\n", rt, q, nb);
          pro += buf;
          snprintf(buf, sizeof buf, "    UNROLL for (int k = 0; k < K; ++k) raw%zux[pp][k] = __builtin_nontemporal_load(reinterpret_cast<const %s*>(static_cast<const %s*>(a.in[%zu]) + (%s) + col[k]));\n",
                   q, rt, ty, q, offp.c_str());
          pro_req += buf;
          snprintf(buf, sizeof buf, "  UNROLL for (int k = 0; k < K; ++k) raw%zux[(ph + %d) %% %d][k] = __builtin_nontemporal_load(reinterpret_cast<const %s*>(static_cast<const %s*>(a.in[%zu]) + (%s) + col[k]));\n",
                   q, depth, nb, rt, ty, q, offn.c_str());
          nxt += buf;
        } else {
          snprintf(buf, sizeof buf, "  %s raw%zu[K];\n  UNROLL for (int k = 0; k < K; ++k) raw%zu[k] = __builtin_nontemporal_load(reinterpret_cast<const %s*>(static_cast<const %s*>(a.in[%zu]) + (%s) + col[k]));\n",
                   rt, q, q, rt, ty, q, offp.c_str());
          pro += buf;
          snprintf(buf, sizeof buf, "  %s nraw%zu[K];\n  UNROLL for (int k = 0; k < K; ++k) nraw%zu[k] = __builtin_nontemporal_load(reinterpret_cast<const %s*>(static_cast<const %s*>(a.in[%zu]) + (%s) + col[k]));\n",
                   rt, q, q, rt, ty, q, offn.c_str());
          nxt += buf;
          snprintf(buf, sizeof buf, "  UNROLL for (int k = 0; k < K; ++k) raw%zu[k] = nraw%zu[k];\n", q, q);
          adv += buf;
        }
      }
      if (!pro.empty()) {
        // the prologue goes before the row loop: find the loop header emitted above
        const size_t at = e.s.rfind(loop_anchor);
        std::string head;
        if (rotating) {
          // what is loaded once has arrived before the first row is requested: a load still pending at the top
          // of the row loop would put a wait into the loop that, trip after trip, also waits for the rows
          // requested ahead
          head = "  __builtin_amdgcn_s_waitcnt(0);\n" + pro;
          snprintf(buf, sizeof buf, "  UNROLL for (int pp = 0; pp < %d; ++pp) {\n    long long rowp = first_row + pp * row_step + rl;\n    if (rowp >= %s) rowp = %s;\n", depth, row_hi, row_last);
          head += buf;
          head += pro_req + "  }\n";
          deferred_head = head;      // placed when the loop is closed: behind everything that is loaded once
          (void)at;
          e.line("  long long rown = row0 + %d * row_step + rl;", depth);
        } else {
          snprintf(buf, sizeof buf, "  long long rowp = first_row + rl;\n  if (rowp >= %s) rowp = %s;\n", row_hi, row_last);
          head = buf;
          e.s.insert(at, head + pro);
          e.line("  long long rown = row0 + row_step + rl;");
        }
        e.line("  if (rown >= %s) rown = %s;          // past the end: any valid row (one that is cached by then)", row_hi, row_any);
        e.s += nxt;
        e.line("  __builtin_amdgcn_sched_barrier(0);     // keep the requests above the work below");
        advance = adv.empty() ? std::string(" ") : adv;      // (non-empty: the operands are served from the buffers)
      }
    }
    for (size_t q = 0; q < A.views.size(); ++q) {
      const RView& v = A.views[q];
      const char* ty = v.dtype == FS_F32 ? "float" : "unsigned short";
      const char* one = v.dtype == FS_F32 ? "p[0]" : v.dtype == FS_F16 ? "f16_lo(p[0])" : "bf16_lo(p[0])";
      if (v.cls == CLS_NONE) continue;     // an operand of a matrix-unit dot: read by the dot's own code
      if (v.cls == CLS_DOT_OUT) continue;  // read in the accumulators' layout, at the top of the kernel
      // persistent form: an operand that does not depend on the row (a per-column vector, a
      // scalar) is loaded once, before the row loop
      bool invariant = persistent && !prefetched[q];      // (what is requested ahead is unpacked inside the loop, also when there is only one row)
      for (int d = 0; d < nrow; ++d) if (A.S[d] != 1 && v.stride[d] != 0) invariant = false;
      const size_t text_from = e.s.size();
      struct Hoist {
        Emitter& e; bool on; size_t from; const std::string& anchor;
        ~Hoist() {
          if (!on) return;
          const std::string text = e.s.substr(from);
          e.s.erase(from);
          e.s.insert(e.s.rfind(anchor), text);
        }
      } hoist{e, invariant, text_from, loop_anchor};
      if (splat[q] && scalar_prefetched[q] && !advance.empty()) {
        hoist.on = false;
        e.line("  const float s%zu = sraw%zu%s;", q, q, rotating ? "x[ph]" : "");
        continue;
      }
      if (splat[q]) {
        e.line("  float s%zu;", q);
        e.line("  { const %s* p = static_cast<const %s*>(a.in[%zu]) + (%s); s%zu = %s; }", ty, ty, q, roff[q].c_str(), q, one);
        continue;
      }
      if (prefetched[q]) {
        // unpack what was requested one iteration ago
        e.line("  float v%zu[K][W];", q);
        e.line("  UNROLL for (int k = 0; k < K; ++k) {");
        const char* ix = rotating ? "x[ph]" : "";
        if (v.dtype == FS_F32) e.line("    UNROLL for (int j = 0; j < 4; ++j) v%zu[k][j] = raw%zu%s[k][j];", q, q, ix);
        else e.line("    UNROLL for (int j = 0; j < W / 2; ++j) { v%zu[k][2 * j] = %s(raw%zu%s[k][j]); v%zu[k][2 * j + 1] = %s(raw%zu%s[k][j]); }",
                    q, v.dtype == FS_F16 ? "f16_lo" : "bf16_lo", q, ix, q, v.dtype == FS_F16 ? "f16_hi" : "bf16_hi", q, ix);
        e.line("  }");
        continue;
      }
      // tensors of the group's own shape stream through once; per-column operands are shared by all rows
      bool dense = true;
      for (int d = 0; d < nrow; ++d) if (A.S[d] != 1 && v.stride[d] == 0) dense = false;
      const char* ld = dense ? "__builtin_nontemporal_load" : "*";
      e.line("  float v%zu[K][W];", q);
      e.line("  UNROLL for (int k = 0; k < K; ++k) {");
      e.line("    const %s* p = static_cast<const %s*>(a.in[%zu]) + (%s) + col[k];", ty, ty, q, roff[q].c_str());
      if (W == 1) {
        e.line("    v%zu[k][0] = %s;", q, one);
      } else if (v.dtype == FS_F32 && W == 2) {
        e.line("    const f32x2 x = %s(reinterpret_cast<const f32x2*>(p));", ld);
        e.line("    v%zu[k][0] = x[0]; v%zu[k][1] = x[1];", q, q);
      } else if (v.dtype == FS_F32) {
        for (int h = 0; h < W / 4; ++h) {
          e.line("    { const f32x4 x = %s(reinterpret_cast<const f32x4*>(p) + %d);", ld, h);
          e.line("      UNROLL for (int j = 0; j < 4; ++j) v%zu[k][%d + j] = x[j]; }", q, 4 * h);
        }
      } else {
        const char* lo = v.dtype == FS_F16 ? "f16_lo" : "bf16_lo";
        const char* hi = v.dtype == FS_F16 ? "f16_hi" : "bf16_hi";
        if (W == 2) {
          e.line("    const unsigned x1 = %s(reinterpret_cast<const unsigned*>(p));", ld);
          e.line("    const unsigned x[1] = {x1};");
        } else {
          e.line("    const %s x = %s(reinterpret_cast<const %s*>(p));", W == 8 ? "u32x4" : "u32x2", ld, W == 8 ? "u32x4" : "u32x2");
        }
        e.line("    UNROLL for (int j = 0; j < W / 2; ++j) { v%zu[k][2 * j] = %s(x[j]); v%zu[k][2 * j + 1] = %s(x[j]); }", q, lo, q, hi);
      }
      e.line("  }");
    }
    // ---- ops in order
    std::vector<char> inv_done(A.g.size(), 0);
    int red_index = 0;
    for (const RNode& n : A.nodes) {
      const bool reduce = n.op == FS_REDUCE_SUM || n.op == FS_REDUCE_MAX;
      // combine the lanes' partial results of reduction r<id> (wavefront steps, then LDS across wavefronts)
      auto combine = [&](int id, bool sum) {
        const char* op = sum ? "SumOp" : "MaxOp";
        if (T > 1) {
          e.line("  r%d = lanes_allreduce<%s, 64>(r%d);", id, op, id);
          e.line("  if ((threadIdx.x & 63) == 0) exch[%d][threadIdx.x >> 6] = r%d;", red_index, id);
          e.line("  __syncthreads();");
          e.line("  r%d = exch[%d][0];", id, red_index);
          e.line("  UNROLL for (int w = 1; w < T; ++w) r%d = %s::apply(r%d, exch[%d][w]);", id, op, id, red_index);
          ++red_index;
        } else if (mma) {
          e.line("  r%d = rows_allreduce<%s>(r%d);", id, op, id);
        } else if (L > 1) {
          e.line("  r%d = lanes_allreduce<%s, L>(r%d);", id, op, id);
        }
      };
      if (n.cls == CLS_COL) {
        const std::string x = opnd(n.o[0], CLS_FULL);
        if (n.op == FS_REDUCE_MAX)
          e.line("  if (row_ok) UNROLL for (int k = 0; k < K; ++k) UNROLL for (int j = 0; j < W; ++j) ca%d[k][j] = fmax(ca%d[k][j], (double)%s);", n.id, n.id, x.c_str());
        else
          e.line("  if (row_ok) UNROLL for (int k = 0; k < K; ++k) UNROLL for (int j = 0; j < W; ++j) ca%d[k][j] += (double)%s;", n.id, x.c_str());
        continue;
      }
      if (reduce && n.over_dot_out) {
        const bool sum = n.op == FS_REDUCE_SUM;
        const std::string x = opnd(n.o[0], CLS_DOT_OUT);
        e.line("  float r%d = %s;", n.id, sum ? "0.0f" : "-__builtin_inff()");
        e.line("  UNROLL for (int dt = 0; dt < D2 / 16; ++dt) UNROLL for (int i = 0; i < 4; ++i) r%d = %s;", n.id,
               sum ? ("r" + std::to_string(n.id) + " + " + x).c_str() : ("fmaxf(r" + std::to_string(n.id) + ", " + x + ")").c_str());
        combine(n.id, sum);
      } else if (reduce) {
        const bool sum = n.op == FS_REDUCE_SUM;
        const std::string x = opnd(n.o[0], CLS_FULL);
        e.line("  float r%d = %s;", n.id, sum ? "0.0f" : "-__builtin_inff()");
        e.line("  UNROLL for (int k = 0; k < K; ++k) {");
        if (!exact) e.line("    if (!ok[k]) continue;");
        e.line("    UNROLL for (int j = 0; j < W; ++j) r%d = %s;", n.id,
               sum ? ("r" + std::to_string(n.id) + " + " + x).c_str() : ("fmaxf(r" + std::to_string(n.id) + ", " + x + ")").c_str());
        e.line("  }");
        combine(n.id, sum);
      } else if (n.op == ROP_DOT_REDUCE) {
        // one value per row: sum over the row of p[n] * b[n]
        const std::string x = opnd(n.o[0], CLS_FULL);
        e.line("  float r%d = 0.0f;", n.id);
        e.line("  UNROLL for (int k = 0; k < K; ++k) {");
        if (!exact) e.line("    if (!ok[k]) continue;");
        e.line("    UNROLL for (int j = 0; j < W; ++j) r%d = fmaf(%s, v%d[k][j], r%d);", n.id, x.c_str(), n.dot_full[0], n.id);
        e.line("  }");
        combine(n.id, true);
      } else if (n.op == ROP_DOT_MMA_IN) {
        emit_mma_in(n);
      } else if (n.op == ROP_DOT_MMA_OUT) {
        emit_mma_out(n);
        continue;                          // stores its result itself
      } else if (n.cls == CLS_DOT_OUT) {
        if (n.op == FS_DIVIDE && n.o[1].kind == OP_ROWB && !inv_done[n.o[1].index]) {
          e.line("  const float inv%d = 1.0f / r%d;", n.o[1].index, n.o[1].index);
          inv_done[n.o[1].index] = 1;
        }
        e.line("  f32x4 d%d[D2 / 16];", n.id);
        e.line("  UNROLL for (int dt = 0; dt < D2 / 16; ++dt) UNROLL for (int i = 0; i < 4; ++i) d%d[dt][i] = %s;", n.id, expr(n).c_str());
        if (n.out_ord >= 0) store_dot_out(n);
        continue;
      } else if (n.op == ROP_DOT_OUTER) {
        // the full tile from a tiny contraction: sum over k of (row scalar) * (column vector)
        e.line("  float t%d[K][W];", n.id);
        std::string ex;
        for (size_t k = 0; k < n.dot_row.size(); ++k) {
          char buf[96];
          if (k == 0) snprintf(buf, sizeof buf, "s%d * v%d[k][j]", n.dot_row[k], n.dot_full[k]);
          else snprintf(buf, sizeof buf, "fmaf(s%d, v%d[k][j], ", n.dot_row[k], n.dot_full[k]);
          ex = k == 0 ? std::string(buf) : std::string(buf) + ex + ")";
        }
        e.line("  UNROLL for (int k = 0; k < K; ++k) UNROLL for (int j = 0; j < W; ++j) t%d[k][j] = %s;", n.id, ex.c_str());
      } else if (n.cls == CLS_ROW) {
        e.line("  const float r%d = %s;", n.id, expr(n).c_str());
      } else {
        if (n.op == FS_DIVIDE && n.o[1].kind == OP_ROWB && !inv_done[n.o[1].index]) {
          e.line("  const float inv%d = 1.0f / r%d;", n.o[1].index, n.o[1].index);
          inv_done[n.o[1].index] = 1;
        }
        e.line("  float t%d[K][W];", n.id);
        e.line("  UNROLL for (int k = 0; k < K; ++k) UNROLL for (int j = 0; j < W; ++j) t%d[k][j] = %s;", n.id, expr(n).c_str());
      }
      if (n.out_ord < 0) continue;
      if (n.cls == CLS_ROW) {
        if (n.out_dtype == FS_F32) e.line("  if (lane == 0 && row_ok) static_cast<float*>(a.out[%d])[row] = r%d;", n.out_ord, n.id);
        else e.line("  if (lane == 0 && row_ok) static_cast<unsigned short*>(a.out[%d])[row] = (unsigned short)%s(r%d);", n.out_ord,
                    n.out_dtype == FS_F16 ? "to_f16" : "to_bf16", n.id);
        continue;
      }
      if (stage) {
        e.line("  __syncthreads();                             // the tile's previous use is over");
        e.line("  UNROLL for (int k = 0; k < K; ++k) {");
        e.line("    if (!ok[k]) continue;");
        e.line("    UNROLL for (int j = 0; j < W; ++j) stage[row_local * N + col[k] + j] = t%d[k][j];", n.id);
        e.line("  }");
        e.line("  __syncthreads();");
        if (n.out_dtype == FS_F32) {
          e.line("  {");
          e.line("    float* o = static_cast<float*>(a.out[%d]) + wg_row0 * N;", n.out_ord);
          e.line("    for (int i = threadIdx.x * 4; i + 4 <= wg_count; i += %d * 4)", wg);
          e.line("      __builtin_nontemporal_store(f32x4{stage[i], stage[i + 1], stage[i + 2], stage[i + 3]}, reinterpret_cast<f32x4*>(o + i));");
          e.line("    for (int i = (wg_count & ~3) + threadIdx.x; i < wg_count; i += %d) o[i] = stage[i];", wg);
          e.line("  }");
        } else {
          const char* cv = n.out_dtype == FS_F16 ? "to_f16" : "to_bf16";
          // 8 values per 16-byte store where the workgroup's first element is 16-byte aligned, else 4
          const int V = ((int64_t)(wg / L) * A.cols) % 8 == 0 ? 8 : 4;
          e.line("  {");
          e.line("    unsigned short* o = static_cast<unsigned short*>(a.out[%d]) + wg_row0 * N;", n.out_ord);
          e.line("    for (int i = threadIdx.x * %d; i + %d <= wg_count; i += %d * %d) {", V, V, wg, V);
          e.line("      unsigned w[%d];", V / 2);
          e.line("      UNROLL for (int j = 0; j < %d; ++j) w[j] = pack_%s(stage[i + 2 * j], stage[i + 2 * j + 1]);", V / 2, cv);
          if (V == 8) e.line("      __builtin_nontemporal_store(u32x4{w[0], w[1], w[2], w[3]}, reinterpret_cast<u32x4*>(o + i));");
          else e.line("      __builtin_nontemporal_store(u32x2{w[0], w[1]}, reinterpret_cast<u32x2*>(o + i));");
          e.line("    }");
          e.line("    for (int i = wg_count / %d * %d + threadIdx.x; i < wg_count; i += %d) o[i] = (unsigned short)%s(stage[i]);", V, V, wg, cv);
          e.line("  }");
        }
        continue;
      }
      e.line("  UNROLL for (int k = 0; k < K; ++k) {");
      e.line("    if (!(row_ok && ok[k])) continue;");
      if (n.out_dtype == FS_F32) {
        e.line("    float* p = static_cast<float*>(a.out[%d]) + row * %lldll + col[k];", n.out_ord, (long long)A.cols);
        if (W == 1) e.line("    p[0] = t%d[k][0];", n.id);
        else if (W == 2) e.line("    __builtin_nontemporal_store(f32x2{t%d[k][0], t%d[k][1]}, reinterpret_cast<f32x2*>(p));", n.id, n.id);
        else for (int h = 0; h < W / 4; ++h)
          e.line("    __builtin_nontemporal_store(f32x4{t%d[k][%d], t%d[k][%d], t%d[k][%d], t%d[k][%d]}, reinterpret_cast<f32x4*>(p) + %d);",
                 n.id, 4 * h, n.id, 4 * h + 1, n.id, 4 * h + 2, n.id, 4 * h + 3, h);
      } else {
        const char* cv = n.out_dtype == FS_F16 ? "to_f16" : "to_bf16";
        e.line("    unsigned short* p = static_cast<unsigned short*>(a.out[%d]) + row * %lldll + col[k];", n.out_ord, (long long)A.cols);
        if (W == 1) e.line("    p[0] = (unsigned short)%s(t%d[k][0]);", cv, n.id);
        else {
          e.line("    unsigned w[W / 2];");
          e.line("    UNROLL for (int j = 0; j < W / 2; ++j) w[j] = pack_%s(t%d[k][2 * j], t%d[k][2 * j + 1]);", cv, n.id, n.id);
          if (W == 8) e.line("    __builtin_nontemporal_store(u32x4{w[0], w[1], w[2], w[3]}, reinterpret_cast<u32x4*>(p));");
          else if (W == 4) e.line("    __builtin_nontemporal_store(u32x2{w[0], w[1]}, reinterpret_cast<u32x2*>(p));");
          else e.line("    __builtin_nontemporal_store(w[0], reinterpret_cast<unsigned*>(p));");
        }
      }
      e.line("  }");
    }
    if (persistent && rotating) {
      e.line("  };");
      e.s.insert(e.s.rfind(loop_anchor), deferred_head);
      // whole trips over the buffers without a branch inside (one path through the loop: the waits on the
      // requests count exactly), then the last, partial trip
      e.line("  long long trip0 = first_row;");
      e.line("  for (; trip0 + %d * row_step + RPW <= %s; trip0 += %d * row_step) {", rot_buffers - 1, row_hi, rot_buffers);
      e.line("    UNROLL for (int ph = 0; ph < %d; ++ph) step(std_true{}, ph, trip0 + ph * row_step);", rot_buffers);
      e.line("  }");
      e.line("  for (; trip0 < %s; trip0 += %d * row_step) {", row_hi, rot_buffers);
      e.line("    UNROLL for (int ph = 0; ph < %d; ++ph) if (trip0 + ph * row_step < %s) step(std_false{}, ph, trip0 + ph * row_step);", rot_buffers, row_hi);
      e.line("  }");
    } else if (persistent) {
      e.s += advance;
      if (T > 1 && A.n_reduce > 0) e.line("  __syncthreads();                             // the exchange slots are written again in the next row");
      e.line("  }");
    }
    // a run of rows that one workgroup sums alone: its sums are the results, stored as they are
    const bool direct = A.seg_rows > 0 && (seg_groups == 1 || seg_per_wave);
    auto direct_store = [&](const RNode& n, const char* index, const char* value) {
      char buf[256];
      if (n.out_dtype == FS_F32) snprintf(buf, sizeof buf, "static_cast<float*>(a.out[%d])[seg * %lldll + %s] = (float)%s;", n.out_ord, (long long)A.cols, index, value);
      else snprintf(buf, sizeof buf, "static_cast<unsigned short*>(a.out[%d])[seg * %lldll + %s] = (unsigned short)%s((float)%s);", n.out_ord, (long long)A.cols, index,
                    n.out_dtype == FS_F16 ? "to_f16" : "to_bf16", value);
      return std::string(buf);
    };
    if (persistent && A.n_col > 0 && T > 1) {
      // one row per workgroup at a time: no two lanes of the workgroup hold the same column
      if (!direct) e.line("  double* ws = static_cast<double*>(a.ws);");
      int ci = 0;
      for (const RNode& n : A.nodes) if (n.cls == CLS_COL) {
        char val[32];
        snprintf(val, sizeof val, "ca%d[k][j]", n.id);
        e.line("  UNROLL for (int k = 0; k < K; ++k) {");
        e.line("    if (!ok[k]) continue;");
        if (direct) e.line("    UNROLL for (int j = 0; j < W; ++j) %s", direct_store(n, "col[k] + j", val).c_str());
        else e.line("    UNROLL for (int j = 0; j < W; ++j) ws[((long long)%d * gridDim.x + blockIdx.x) * %lldll + col[k] + j] = ca%d[k][j];", ci, (long long)A.cols, n.id);
        e.line("  }");
        ++ci;
      }
    } else if (persistent && A.n_col > 0 && seg_per_wave) {
      // the wavefront's row groups hold the same columns: an xor butterfly adds them (fixed order), the
      // first row group stores
      if (L < 64) {
        for (const RNode& n : A.nodes) if (n.cls == CLS_COL)
          e.line(n.op == FS_REDUCE_MAX
                     ? "  for (int m = L; m < 64; m <<= 1) UNROLL for (int k = 0; k < K; ++k) UNROLL for (int j = 0; j < W; ++j) ca%d[k][j] = fmax(ca%d[k][j], shfl_xor_f64(ca%d[k][j], m));"
                     : "  for (int m = L; m < 64; m <<= 1) UNROLL for (int k = 0; k < K; ++k) UNROLL for (int j = 0; j < W; ++j) ca%d[k][j] += shfl_xor_f64(ca%d[k][j], m);", n.id, n.id, n.id);
      }
      e.line("  if (seg_ok && (int)(threadIdx.x & 63) < L) {");
      for (const RNode& n : A.nodes) if (n.cls == CLS_COL) {
        char val[32];
        snprintf(val, sizeof val, "ca%d[k][j]", n.id);
        e.line("    UNROLL for (int k = 0; k < K; ++k) {");
        e.line("      if (!ok[k]) continue;");
        e.line("      UNROLL for (int j = 0; j < W; ++j) %s", direct_store(n, "col[k] + j", val).c_str());
        e.line("    }");
      }
      e.line("  }");
    } else if (persistent && A.n_col > 0) {
      e.line("  __shared__ double colacc[%d][%lld];", A.n_col, (long long)A.cols);
      {
        unsigned max_mask = 0;      // a maximum starts from -inf (one loop: each element is initialised by one thread)
        int r = 0;
        for (const RNode& n : A.nodes) if (n.cls == CLS_COL) { if (n.op == FS_REDUCE_MAX) max_mask |= 1u << r; ++r; }
        if (max_mask == 0)
          e.line("  for (int i = threadIdx.x; i < %lld; i += blockDim.x) (&colacc[0][0])[i] = 0.0;", (long long)A.n_col * A.cols);
        else
          e.line("  for (int i = threadIdx.x; i < %lld; i += blockDim.x) (&colacc[0][0])[i] = ((0x%xu >> (i / %lld)) & 1u) ? -__builtin_inf() : 0.0;",
                 (long long)A.n_col * A.cols, max_mask, (long long)A.cols);
      }
      e.line("  __syncthreads();");
      // fixed summation order (results are bit-reproducible): first the row groups of a wavefront
      // (lanes that hold the same columns) by an xor butterfly, then the wavefronts one after the other
      if (L < 64) {
        for (const RNode& n : A.nodes) if (n.cls == CLS_COL)
          e.line(n.op == FS_REDUCE_MAX
                     ? "  for (int m = L; m < 64; m <<= 1) UNROLL for (int k = 0; k < K; ++k) UNROLL for (int j = 0; j < W; ++j) ca%d[k][j] = fmax(ca%d[k][j], shfl_xor_f64(ca%d[k][j], m));"
                     : "  for (int m = L; m < 64; m <<= 1) UNROLL for (int k = 0; k < K; ++k) UNROLL for (int j = 0; j < W; ++j) ca%d[k][j] += shfl_xor_f64(ca%d[k][j], m);", n.id, n.id, n.id);
      }
      e.line("  for (int w = 0; w < (int)blockDim.x / 64; ++w) {");
      e.line("    if ((int)(threadIdx.x >> 6) == w && (int)(threadIdx.x & 63) < L) {");
      int ci = 0;
      for (const RNode& n : A.nodes) if (n.cls == CLS_COL) {
        e.line("      UNROLL for (int k = 0; k < K; ++k) {");
        e.line("        if (!ok[k]) continue;");
        if (n.op == FS_REDUCE_MAX) e.line("        UNROLL for (int j = 0; j < W; ++j) colacc[%d][col[k] + j] = fmax(colacc[%d][col[k] + j], ca%d[k][j]);", ci, ci, n.id);
        else e.line("        UNROLL for (int j = 0; j < W; ++j) colacc[%d][col[k] + j] += ca%d[k][j];", ci, n.id);
        e.line("      }");
        ++ci;
      }
      e.line("    }");
      e.line("    __syncthreads();");
      e.line("  }");
      if (direct) {
        int r = 0;
        for (const RNode& n : A.nodes) if (n.cls == CLS_COL) {
          char val[32];
          snprintf(val, sizeof val, "colacc[%d][i]", r++);
          e.line("  for (int i = threadIdx.x; i < %lld; i += blockDim.x) %s", (long long)A.cols, direct_store(n, "i", val).c_str());
        }
      } else {
        e.line("  double* ws = static_cast<double*>(a.ws);");
        e.line("  for (int r = 0; r < %d; ++r)", A.n_col);
        e.line("    for (int i = threadIdx.x; i < %lld; i += blockDim.x) ws[((long long)r * gridDim.x + blockIdx.x) * %lldll + i] = colacc[r][i];",
               (long long)A.cols, (long long)A.cols);
      }
    }
    e.line("}");
    uint64_t h = 1469598103934665603ull;
    for (unsigned char c : e.s) { h ^= c; h *= 1099511628211ull; }
    char name[32];
    snprintf(name, sizeof name, "fs_row_%08x", (unsigned)(h ^ (h >> 32)));
    *kernel_name = name;
    const std::string tag = "FS_ROW_NAME";
    e.s.replace(e.s.find(tag), tag.size(), name);
  }
};


// ---------------------------------------------------------------------------------------------
// Streamed block template: one workgroup walks a row in passes (block composition with
// intermediates in shared memory, Section 5.1, for rows that do not fit registers).  The
// reductions split the group into passes: pass p holds everything that needs the results of
// p rounds of reductions.  A full value computed in one pass and read in a later one is
// either kept in an LDS row buffer or recomputed from the group's inputs (re-read from HBM);
// the row buffers are laid out by the shared-memory optimisation (Algorithm 4), which lets a
// value take over the buffer of a value it dominates -- softmax of a 40 000-element row
// needs one buffer, not three.  If even the shared layout exceeds the LDS, nothing is kept
// and every pass streams from HBM: any row length runs.
struct Stream {
  const Analysis& A;
  int W = 4, wg = 512;
  bool fast = false, cached = true, cache_views = true;
  std::vector<int> idx_of;            // node id -> index into A.nodes
  std::vector<int> ready;             // full value: first pass it can be computed in; per-row value: passes that must be over
  std::vector<int> phase;             // reductions: the pass that accumulates them
  int n_loops = 1;
  std::vector<char> cut_node, cut_view;     // kept in a row buffer
  std::vector<int> first_use;               // per view: the first pass that reads it
  std::vector<int64_t> off_node, off_view;  // float offset of the buffer
  std::vector<int> share_node;              // planner's report: index (planner numbering) taken over, -1
  int64_t lds_floats = 0;
  int n_buffers = 0, n_shared = 0;
  std::vector<char> splat;
  std::vector<std::string> roff;
  bool coords = false;
  Emitter e;

  explicit Stream(const Analysis& a) : A(a) {}

  static bool is_col(const RNode& n) { return n.cls == CLS_COL; }     // a reduction over the rows: running values per thread and column
  static bool is_red(const RNode& n) { return !is_col(n) && (n.op == FS_REDUCE_SUM || n.op == FS_REDUCE_MAX || n.op == ROP_DOT_REDUCE); }
  int n_iter() const { return (int)((A.cols / W + wg - 1) / wg); }   // chunks of a row per thread

  void schedule() {
    const int n = (int)A.nodes.size();
    idx_of.assign(A.g.size(), -1);
    for (int i = 0; i < n; ++i) idx_of[A.nodes[i].id] = i;
    ready.assign(n, 0);
    phase.assign(n, -1);
    int last = 0;
    for (int i = 0; i < n; ++i) {
      const RNode& x = A.nodes[i];
      int r = 0;
      for (int j = 0; j < x.nop; ++j)
        if (x.o[j].kind == OP_NODE || x.o[j].kind == OP_ROWB) r = std::max(r, ready[idx_of[x.o[j].index]]);
      if (is_red(x)) { phase[i] = r; ready[i] = r + 1; last = std::max(last, r); }
      else if (is_col(x)) { phase[i] = r; ready[i] = r; last = std::max(last, r); }    // accumulated in the pass that has its operand
      else {
        ready[i] = r;
        if (x.cls == CLS_FULL && x.out_ord >= 0) last = std::max(last, r);
      }
    }
    n_loops = last + 1;
  }

  // which values cross from one pass to a later one
  void find_cuts(std::vector<std::vector<int>>* targets) {
    const int n = (int)A.nodes.size();
    cut_node.assign(n, 0);
    cut_view.assign(A.views.size(), 0);
    targets->assign(n_loops, {});
    for (int i = 0; i < n; ++i) {
      const RNode& x = A.nodes[i];
      if (is_red(x) || is_col(x)) (*targets)[phase[i]].push_back(i);
      else if (x.cls == CLS_FULL && x.out_ord >= 0) (*targets)[ready[i]].push_back(i);
    }
    first_use.assign(A.views.size(), -1);
    if (!cached) return;
    // An input read in two or more passes is kept after its first read; one read in a single
    // pass (a per-column operand of the epilogue, say) is not worth a buffer.
    std::vector<std::vector<char>> view_pass(A.views.size(), std::vector<char>(n_loops, 0));
    for (int p = n_loops - 1; p >= 0; --p) {
      std::vector<char> seen(n, 0);
      std::vector<int> stack;
      auto use_view = [&](int v) { if (!splat_view(v)) view_pass[v][p] = 1; };
      auto use_full = [&](const Opnd& o) {
        if (o.kind == OP_VIEW) { use_view(o.index); return; }
        if (o.kind != OP_NODE) return;
        const int k = idx_of[o.index];
        if (A.nodes[k].cls != CLS_FULL) return;
        if (ready[k] < p) { cut_node[k] = 1; return; }
        if (!seen[k]) { seen[k] = 1; stack.push_back(k); }
      };
      for (int t : (*targets)[p]) {
        if (is_red(A.nodes[t]) || is_col(A.nodes[t])) {
          use_full(A.nodes[t].o[0]);
          for (int v : A.nodes[t].dot_full) use_view(v);
        } else if (!seen[t]) { seen[t] = 1; stack.push_back(t); }
      }
      for (int k = 0; k < n; ++k)        // values kept for later passes are produced in their own pass
        if (cut_node[k] && ready[k] == p && !seen[k]) { seen[k] = 1; stack.push_back(k); (*targets)[p].push_back(k); }
      while (!stack.empty()) {
        const int k = stack.back();
        stack.pop_back();
        const RNode& x = A.nodes[k];
        for (int j = 0; j < x.nop; ++j) use_full(x.o[j]);
        for (int v : x.dot_full) use_view(v);
      }
    }
    for (size_t v = 0; v < A.views.size(); ++v) {
      int uses = 0;
      for (int p = 0; p < n_loops; ++p) if (view_pass[v][p]) { if (first_use[v] < 0) first_use[v] = p; ++uses; }
      cut_view[v] = cache_views && uses >= 2;
    }
  }
  bool splat_view(int v) const { return A.views[v].cls == CLS_ROW || A.views[v].stride[A.rank - 1] == 0; }

  // Algorithm 4 over the kept values: ops = views, then nodes in execution order (pass, then list order)
  void plan_buffers() {
    const int n = (int)A.nodes.size(), nv = (int)A.views.size();
    std::vector<int> order(n);
    for (int i = 0; i < n; ++i) order[i] = i;
    auto time_of = [&](int i) { return is_red(A.nodes[i]) || is_col(A.nodes[i]) ? phase[i] : ready[i]; };
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return time_of(a) < time_of(b); });
    std::vector<int> pos(n);
    for (int k = 0; k < n; ++k) pos[order[k]] = nv + k;
    SharedPlanInput in;
    in.operands.resize(nv + n);
    in.req_bytes.assign(nv + n, 0);
    in.is_output.assign(nv + n, 0);
    const int64_t row_bytes = A.cols * 4;
    for (int v = 0; v < nv; ++v) if (cut_view[v]) in.req_bytes[v] = row_bytes;
    for (int i = 0; i < n; ++i) {
      const RNode& x = A.nodes[i];
      std::vector<int>& ops = in.operands[pos[i]];
      for (int j = 0; j < x.nop; ++j) {
        if (x.o[j].kind == OP_NODE || x.o[j].kind == OP_ROWB) ops.push_back(pos[idx_of[x.o[j].index]]);
        else if (x.o[j].kind == OP_VIEW) ops.push_back(x.o[j].index);
      }
      for (int v : x.dot_row) ops.push_back(v);
      for (int v : x.dot_full) ops.push_back(v);
      if (cut_node[i]) in.req_bytes[pos[i]] = row_bytes;
      if (x.out_ord >= 0) in.is_output[pos[i]] = 1;
    }
    const SharedPlanResult r = shared_plan(in);
    off_view.assign(nv, -1);
    off_node.assign(n, -1);
    n_buffers = 0; n_shared = 0;
    for (int v = 0; v < nv; ++v) if (cut_view[v]) { off_view[v] = r.offset[v] / 4; ++n_buffers; }
    for (int i = 0; i < n; ++i) if (cut_node[i]) {
      off_node[i] = r.offset[pos[i]] / 4;
      ++n_buffers;
      if (r.shares_with[pos[i]] >= 0) ++n_shared;
    }
    lds_floats = r.total_bytes / 4;
  }

  bool geometry(int want_wg, std::string* err) {
    W = chunk_elements(A, &fast);
    if (W == 0) { *err = "generated row schedule: an operand strided along the last dim"; return false; }
    const int64_t nvec = A.cols / W;
    wg = want_wg ? want_wg : nvec <= 2048 ? 256 : nvec <= 8192 ? 512 : 1024;
    return true;
  }

  // ---- emission helpers
  std::string opnd(const Opnd& o, int consumer_cls) const {
    char buf[64];
    switch (o.kind) {
      case OP_NODE: snprintf(buf, sizeof buf, consumer_cls == CLS_FULL ? "t%d[j]" : "r%d", o.index); return buf;
      case OP_ROWB: snprintf(buf, sizeof buf, "r%d", o.index); return buf;
      case OP_VIEW: snprintf(buf, sizeof buf, splat[o.index] ? "s%d" : "v%d[j]", o.index); return buf;
      default: return const_text(o.cval);
    }
  }
  std::string expr(const RNode& n) const {
    const std::string a = opnd(n.o[0], n.cls), b = n.nop == 2 ? opnd(n.o[1], n.cls) : std::string();
    if (n.op == FS_DIVIDE && n.cls == CLS_FULL && n.o[1].kind == OP_ROWB) return a + " * inv" + std::to_string(n.o[1].index);
    if (n.op == FS_CAUSAL_MASK) return "(col + j <= irow) ? " + a + " : " + const_text(n.o[1].cval);
    if (n.op == EW_OP_GELU_TANH) return "gelu_tanh(" + a + ", " + const_text(n.gelu[0]) + ", " + const_text(n.gelu[1]) + ", " + const_text(n.gelu[2]) + ")";
    return op_text(n.op, a, b, fast);
  }

  void load_global(const std::string& name, int q) {
    const RView& v = A.views[q];
    const char* ty = v.dtype == FS_F32 ? "float" : "unsigned short";
    e.line("        float %s[W];", name.c_str());
    e.line("        {");
    e.line("          const %s* p = static_cast<const %s*>(a.in[%d]) + (%s) + col;", ty, ty, q, roff[q].c_str());
    if (W == 1) {
      e.line("          %s[0] = %s;", name.c_str(), v.dtype == FS_F32 ? "p[0]" : v.dtype == FS_F16 ? "f16_lo(p[0])" : "bf16_lo(p[0])");
    } else if (v.dtype == FS_F32 && W == 2) {
      e.line("          const f32x2 x = *reinterpret_cast<const f32x2*>(p); %s[0] = x[0]; %s[1] = x[1];", name.c_str(), name.c_str());
    } else if (v.dtype == FS_F32) {
      for (int h = 0; h < W / 4; ++h)
        e.line("          { const f32x4 x = *(reinterpret_cast<const f32x4*>(p) + %d); UNROLL for (int j = 0; j < 4; ++j) %s[%d + j] = x[j]; }", h, name.c_str(), 4 * h);
    } else {
      const char* lo = v.dtype == FS_F16 ? "f16_lo" : "bf16_lo";
      const char* hi = v.dtype == FS_F16 ? "f16_hi" : "bf16_hi";
      if (W == 2) e.line("          const unsigned x[1] = {*reinterpret_cast<const unsigned*>(p)};");
      else e.line("          const %s x = *reinterpret_cast<const %s*>(p);", W == 8 ? "u32x4" : "u32x2", W == 8 ? "u32x4" : "u32x2");
      e.line("          UNROLL for (int j = 0; j < W / 2; ++j) { %s[2 * j] = %s(x[j]); %s[2 * j + 1] = %s(x[j]); }", name.c_str(), lo, name.c_str(), hi);
    }
    e.line("        }");
  }
  void store_global(const RNode& n) {
    e.line("        {");
    if (n.out_dtype == FS_F32) {
      e.line("          float* p = static_cast<float*>(a.out[%d]) + row * %lldll + col;", n.out_ord, (long long)A.cols);
      if (W == 1) e.line("          p[0] = t%d[0];", n.id);
      else if (W == 2) e.line("          __builtin_nontemporal_store(f32x2{t%d[0], t%d[1]}, reinterpret_cast<f32x2*>(p));", n.id, n.id);
      else for (int h = 0; h < W / 4; ++h)
        e.line("          __builtin_nontemporal_store(f32x4{t%d[%d], t%d[%d], t%d[%d], t%d[%d]}, reinterpret_cast<f32x4*>(p) + %d);",
               n.id, 4 * h, n.id, 4 * h + 1, n.id, 4 * h + 2, n.id, 4 * h + 3, h);
    } else {
      const char* cv = n.out_dtype == FS_F16 ? "to_f16" : "to_bf16";
      e.line("          unsigned short* p = static_cast<unsigned short*>(a.out[%d]) + row * %lldll + col;", n.out_ord, (long long)A.cols);
      if (W == 1) e.line("          p[0] = (unsigned short)%s(t%d[0]);", cv, n.id);
      else {
        e.line("          unsigned w[W / 2];");
        e.line("          UNROLL for (int j = 0; j < W / 2; ++j) w[j] = pack_%s(t%d[2 * j], t%d[2 * j + 1]);", cv, n.id, n.id);
        if (W == 8) e.line("          __builtin_nontemporal_store(u32x4{w[0], w[1], w[2], w[3]}, reinterpret_cast<u32x4*>(p));");
        else if (W == 4) e.line("          __builtin_nontemporal_store(u32x2{w[0], w[1]}, reinterpret_cast<u32x2*>(p));");
        else e.line("          __builtin_nontemporal_store(w[0], reinterpret_cast<unsigned*>(p));");
      }
    }
    e.line("        }");
  }

  void emit(const std::vector<std::vector<int>>& targets, std::string* kernel_name) {
    const int n = (int)A.nodes.size(), nv = (int)A.views.size(), nrow = A.rank - 1, T = wg / 64;
    splat.assign(nv, 0);
    roff.assign(nv, "");
    // row offsets reuse the register templates' logic
    Gen helper(A);
    for (int q = 0; q < nv; ++q) { splat[q] = splat_view(q); roff[q] = helper.row_offset(A.views[q], &coords); }
    if (A.has_causal) coords = true;
    std::vector<char> is_divisor(A.g.size(), 0);
    for (const RNode& x : A.nodes) if (x.op == FS_DIVIDE && x.cls == CLS_FULL && x.o[1].kind == OP_ROWB) is_divisor[x.o[1].index] = 1;
    int n_red = 0;
    std::vector<int> red_slot(n, -1);
    for (int i = 0; i < n; ++i) if (is_red(A.nodes[i])) red_slot[i] = n_red++;

    e.s = ew_preamble();
    e.s += kReducePreamble;
    e.line("extern \"C\" __global__ __launch_bounds__(%d) void FS_ROW_NAME(const Args a) {", wg);
    e.line("  constexpr int W = %d, NVEC = %lld, WG = %d, T = %d;", W, (long long)(A.cols / W), wg, T);
    if (lds_floats > 0) e.line("  __shared__ float rowbuf[%lld];", (long long)lds_floats);
    if (n_red > 0) e.line("  __shared__ float exch[%d][T];", n_red);
    const bool cols_red = A.n_col > 0;
    if (cols_red) {
      // Reductions over the rows: a thread works on the same chunks of every row (chunk threadIdx.x + it * WG),
      // so it keeps a double-precision running value per element of its chunks across the row loop, in
      // registers; the loops over a row are unrolled so that the chunk number is a constant.
      e.line("  constexpr int NIT = %d;", n_iter());
      for (const RNode& x : A.nodes) if (is_col(x)) {
        e.line("  double ca%d[NIT][W];", x.id);
        e.line("  UNROLL for (int it = 0; it < NIT; ++it) UNROLL for (int j = 0; j < W; ++j) ca%d[it][j] = %s;", x.id, x.op == FS_REDUCE_MAX ? "-__builtin_inf()" : "0.0");
      }
    }
    e.line("  for (long long row = blockIdx.x; row < %lldll; row += gridDim.x) {", (long long)A.rows);
    if (coords) {
      e.line("    unsigned long long rr = (unsigned long long)row;");
      for (int d = nrow - 1; d >= 0; --d) {
        if (A.S[d] == 1) { e.line("    const long long i%d = 0;", d); continue; }
        e.line("    const long long i%d = rr %% %lldull; rr /= %lldull;", d, (long long)A.S[d], (long long)A.S[d]);
      }
      if (A.has_causal) e.line("    const long long irow = i%d;", nrow - 1);
    }
    for (int q = 0; q < nv; ++q) if (splat[q]) {
      const RView& v = A.views[q];
      const char* ty = v.dtype == FS_F32 ? "float" : "unsigned short";
      const char* one = v.dtype == FS_F32 ? "p[0]" : v.dtype == FS_F16 ? "f16_lo(p[0])" : "bf16_lo(p[0])";
      e.line("    float s%d;", q);
      e.line("    { const %s* p = static_cast<const %s*>(a.in[%d]) + (%s); s%d = %s; }", ty, ty, q, roff[q].c_str(), q, one);
    }
    // per-row values that need no pass at all, then pass by pass
    auto row_ops = [&](int avail) {
      for (int i = 0; i < n; ++i) {
        const RNode& x = A.nodes[i];
        if (x.cls != CLS_ROW || is_red(x) || ready[i] != avail) continue;
        e.line("    const float r%d = %s;", x.id, expr(x).c_str());
        if (is_divisor[x.id]) e.line("    const float inv%d = 1.0f / r%d;", x.id, x.id);
        row_out(x);
      }
    };
    row_ops(0);
    for (int p = 0; p < n_loops; ++p) {
      for (int t : targets[p]) if (is_red(A.nodes[t]))
        e.line("    float r%d = %s;", A.nodes[t].id, A.nodes[t].op == FS_REDUCE_MAX ? "-__builtin_inff()" : "0.0f");
      if (cols_red) {
        e.line("    UNROLL for (int it = 0; it < NIT; ++it) {      // pass %d", p);
        e.line("      const int c = (int)threadIdx.x + it * WG;");
        e.line("      const int col = c * W;");
        e.line("      if (c < NVEC) {");
      } else {
        e.line("    for (int c = threadIdx.x; c < NVEC; c += WG) {      // pass %d", p);
        e.line("      const int col = c * W;");
        e.line("      {");
      }
      std::vector<char> have_node(n, 0), have_view(nv, 0);
      std::function<void(int)> need_view = [&](int q) {
        if (splat[q] || have_view[q]) return;
        have_view[q] = 1;
        char name[16];
        snprintf(name, sizeof name, "v%d", q);
        if (cached && cut_view[q] && p > first_use[q]) {
          e.line("        float %s[W];", name);
          e.line("        UNROLL for (int j = 0; j < W; ++j) %s[j] = rowbuf[%lld + col + j];", name, (long long)off_view[q]);
        } else {
          load_global(name, q);
        }
      };
      std::function<void(int)> need_node = [&](int k) {
        if (have_node[k]) return;
        have_node[k] = 1;
        const RNode& x = A.nodes[k];
        if (cached && cut_node[k] && ready[k] < p) {
          e.line("        float t%d[W];", x.id);
          e.line("        UNROLL for (int j = 0; j < W; ++j) t%d[j] = rowbuf[%lld + col + j];", x.id, (long long)off_node[k]);
          return;
        }
        for (int j = 0; j < x.nop; ++j) {
          if (x.o[j].kind == OP_VIEW) need_view(x.o[j].index);
          else if (x.o[j].kind == OP_NODE && A.nodes[idx_of[x.o[j].index]].cls == CLS_FULL) need_node(idx_of[x.o[j].index]);
        }
        for (int v : x.dot_full) need_view(v);
        e.line("        float t%d[W];", x.id);
        if (x.op == ROP_DOT_OUTER) {
          std::string ex;
          for (size_t k2 = 0; k2 < x.dot_row.size(); ++k2) {
            char buf[96];
            if (k2 == 0) snprintf(buf, sizeof buf, "s%d * v%d[j]", x.dot_row[k2], x.dot_full[k2]);
            else snprintf(buf, sizeof buf, "fmaf(s%d, v%d[j], ", x.dot_row[k2], x.dot_full[k2]);
            ex = k2 == 0 ? std::string(buf) : std::string(buf) + ex + ")";
          }
          e.line("        UNROLL for (int j = 0; j < W; ++j) t%d[j] = %s;", x.id, ex.c_str());
        } else {
          e.line("        UNROLL for (int j = 0; j < W; ++j) t%d[j] = %s;", x.id, expr(x).c_str());
        }
      };
      // everything this pass reads is loaded before anything it writes is stored: a value may
      // take over the buffer of the value it was computed from
      for (int t : targets[p]) {
        const RNode& x = A.nodes[t];
        if (is_red(x) || is_col(x)) {
          if (x.o[0].kind == OP_VIEW) need_view(x.o[0].index);
          else if (x.o[0].kind == OP_NODE) need_node(idx_of[x.o[0].index]);
          for (int v : x.dot_full) need_view(v);
        } else need_node(t);
      }
      for (int t : targets[p]) {
        const RNode& x = A.nodes[t];
        if (!is_col(x)) continue;
        const std::string v = opnd(x.o[0], CLS_FULL);
        if (x.op == FS_REDUCE_MAX) e.line("        UNROLL for (int j = 0; j < W; ++j) ca%d[it][j] = fmax(ca%d[it][j], (double)%s);", x.id, x.id, v.c_str());
        else e.line("        UNROLL for (int j = 0; j < W; ++j) ca%d[it][j] += (double)%s;", x.id, v.c_str());
      }
      if (cached) for (int q = 0; q < nv; ++q) if (cut_view[q] && first_use[q] == p) need_view(q);
      for (int t : targets[p]) {
        const RNode& x = A.nodes[t];
        if (!is_red(x)) continue;
        const std::string v = opnd(x.o[0], CLS_FULL);
        if (x.op == FS_REDUCE_SUM) e.line("        UNROLL for (int j = 0; j < W; ++j) r%d = r%d + %s;", x.id, x.id, v.c_str());
        else if (x.op == FS_REDUCE_MAX) e.line("        UNROLL for (int j = 0; j < W; ++j) r%d = fmaxf(r%d, %s);", x.id, x.id, v.c_str());
        else e.line("        UNROLL for (int j = 0; j < W; ++j) r%d = fmaf(%s, v%d[j], r%d);", x.id, v.c_str(), x.dot_full[0], x.id);
      }
      if (cached) {
        for (int q = 0; q < nv; ++q) if (cut_view[q] && first_use[q] == p)
          e.line("        UNROLL for (int j = 0; j < W; ++j) rowbuf[%lld + col + j] = v%d[j];", (long long)off_view[q], q);
        for (int k = 0; k < n; ++k) if (cut_node[k] && ready[k] == p)
          e.line("        UNROLL for (int j = 0; j < W; ++j) rowbuf[%lld + col + j] = t%d[j];", (long long)off_node[k], A.nodes[k].id);
      }
      for (int t : targets[p]) {
        const RNode& x = A.nodes[t];
        if (!is_red(x) && !is_col(x) && x.out_ord >= 0) store_global(x);
      }
      e.line("      }");
      e.line("    }");
      // combine this pass's reductions: wavefront steps, one LDS slot per wavefront, one barrier
      bool any = false;
      for (int t : targets[p]) if (is_red(A.nodes[t])) {
        const RNode& x = A.nodes[t];
        const char* op = x.op == FS_REDUCE_MAX ? "MaxOp" : "SumOp";
        e.line("    r%d = lanes_allreduce<%s, 64>(r%d);", x.id, op, x.id);
        if (T > 1) e.line("    if ((threadIdx.x & 63) == 0) exch[%d][threadIdx.x >> 6] = r%d;", red_slot[t], x.id);
        any = true;
      }
      if (any && T > 1) {
        e.line("    __syncthreads();");
        for (int t : targets[p]) if (is_red(A.nodes[t])) {
          const RNode& x = A.nodes[t];
          const char* op = x.op == FS_REDUCE_MAX ? "MaxOp" : "SumOp";
          e.line("    r%d = exch[%d][0];", x.id, red_slot[t]);
          e.line("    UNROLL for (int w = 1; w < T; ++w) r%d = %s::apply(r%d, exch[%d][w]);", x.id, op, x.id, red_slot[t]);
        }
      }
      for (int t : targets[p]) if (is_red(A.nodes[t])) {
        const RNode& x = A.nodes[t];
        if (is_divisor[x.id]) e.line("    const float inv%d = 1.0f / r%d;", x.id, x.id);
        row_out(x);
      }
      row_ops(p + 1);
    }
    if (n_red > 0 && T > 1) e.line("    __syncthreads();      // the exchange slots are reused by the next row");
    e.line("  }");
    if (cols_red) {
      // every thread's columns are its own in the workgroup: one partial row per workgroup and reduction,
      // straight from the registers (a second kernel adds the partial rows)
      e.line("  double* ws = static_cast<double*>(a.ws);");
      int ci = 0;
      for (const RNode& x : A.nodes) if (is_col(x)) {
        e.line("  UNROLL for (int it = 0; it < NIT; ++it) {");
        e.line("    const int c = (int)threadIdx.x + it * WG;");
        e.line("    if (c < NVEC) { UNROLL for (int j = 0; j < W; ++j) ws[((long long)%d * gridDim.x + blockIdx.x) * %lldll + c * W + j] = ca%d[it][j]; }", ci, (long long)A.cols, x.id);
        e.line("  }");
        ++ci;
      }
    }
    e.line("}");
    uint64_t h = 1469598103934665603ull;
    for (unsigned char c : e.s) { h ^= c; h *= 1099511628211ull; }
    char name[32];
    snprintf(name, sizeof name, "fs_row_%08x", (unsigned)(h ^ (h >> 32)));
    *kernel_name = name;
    const std::string tag = "FS_ROW_NAME";
    e.s.replace(e.s.find(tag), tag.size(), name);
  }
  void row_out(const RNode& x) {
    if (x.out_ord < 0) return;
    if (x.out_dtype == FS_F32) e.line("    if (threadIdx.x == 0) static_cast<float*>(a.out[%d])[row] = r%d;", x.out_ord, x.id);
    else e.line("    if (threadIdx.x == 0) static_cast<unsigned short*>(a.out[%d])[row] = (unsigned short)%s(r%d);", x.out_ord,
                x.out_dtype == FS_F16 ? "to_f16" : "to_bf16", x.id);
  }
};

struct GenArgs { const void* in[64]; void* out[16]; void* ws; };   // mirrors Args of the generated source

}  // namespace

static void dump_source(const std::string& src) {
  if (const char* dump = getenv("FS_DUMP_SOURCE")) {        // debugging aid: append what was generated
    if (FILE* f = fopen(dump, "a")) { fputs(src.c_str(), f); fputs("\n// ----\n", f); fclose(f); }
  }
}

bool row_gen_plan(const Graph& g, const LaunchOpts& opt, RowGenLaunch* out, int* status, std::string* err) {
  *status = FS_ERR_UNSUPPORTED;
  Analysis A(g);
  if (!A.run()) { *err = A.err; return false; }
  Gen gen(A);
  RowGenLaunch l;
  // A fixed number of workgroups that loop over the rows: with the lanes per row given too, the
  // register templates in their persistent form (the next row is requested while the current
  // one is worked on); without, the streamed template.
  const bool want_persistent = opt.grid > 0 && opt.rows_per_wave > 0 && A.n_col == 0;
  const bool want_stream = opt.grid > 0 && A.n_col == 0 && !want_persistent;
  if (opt.wg_size && (opt.wg_size < 64 || opt.wg_size > 1024 || opt.wg_size % 64 || (!want_stream && A.n_col == 0 && opt.wg_size > 256))) {
    *status = FS_ERR_INVALID;
    *err = "generated row schedule: wg_size must be 64, 128, 192 or 256 (a multiple of 64 up to 1024 with a fixed grid)";
    return false;
  }
  if (opt.rows_per_wave) {
    // rows one wavefront covers at a time = 64 / lanes per row
    const int r = opt.rows_per_wave;
    if (r < 1 || r > 64 || (r & (r - 1))) {
      *status = FS_ERR_INVALID;
      *err = "generated row schedule: rows_per_wave must be a power of two in 1..64 (lanes per row = 64 / rows_per_wave)";
      return false;
    }
    gen.lanes_per_row = 64 / r;
  }
  l.rows = A.rows; l.cols = A.cols;
  l.n_ops = (int)A.nodes.size();
  l.n_reduce = A.n_reduce;
  for (const RView& v : A.views) {
    l.view_param.push_back(v.param);
    bool dense = v.cls == CLS_FULL && v.offset == 0;
    int64_t st = 1;
    for (int d = A.rank - 1; d >= 0 && dense; --d) { if (A.S[d] != 1 && v.stride[d] != st) dense = false; st *= A.S[d]; }
    l.view_dense.push_back(dense ? 1 : 0);
  }
  gen.want_persistent = want_persistent;
  if (const char* pf = getenv("FS_ROW_PREFETCH")) gen.force_prefetch = atoi(pf);   // measurement aid: 1 or 2 row steps requested ahead
  gen.wg = opt.wg_size && (opt.wg_size <= 256 || A.n_col > 0) ? opt.wg_size : 256;
  if (gen.wg & (gen.wg - 1)) gen.wg = gen.wg > 512 ? 512 : gen.wg > 256 ? 256 : 128;   // lanes per row divide the workgroup
  std::string gerr;
  if (!want_stream && gen.geometry(&gerr)) {
    // the row lives in registers
    int64_t n_seg = 0;
    if (A.seg_rows > 0) {
      // column sums per run of rows: a run belongs to one workgroup where there are runs enough to fill
      // the chip; fewer, longer runs are shared by as many workgroups as leave each at least four rounds of rows
      n_seg = A.rows / A.seg_rows;
      const int64_t per_round = gen.L > 64 ? 1 : gen.wg / gen.L;
      int64_t share = n_seg >= 512 ? 1 : (512 + n_seg - 1) / n_seg;
      const int64_t most = A.seg_rows / (4 * per_round);
      if (share > most) share = most;
      if (share < 1) share = 1;
      if (share > 4096) share = 4096;
      gen.seg_groups = (int)share;
      if (n_seg * share > 0x7fffffffLL) { *err = "generated row schedule: too many runs of rows for one grid"; return false; }
      // Many short runs in a group that only reads full-size tensors: a run per wavefront, where a run
      // fills a workgroup's rounds of rows badly (below 90%) or a row takes a whole wavefront anyway --
      // nothing goes through LDS then.  Measured on [16384, 50, 128] fp32: 72 against 96 us; with a
      // full-size output packed in, the workgroup form is the faster one (139 against 158 us).
      bool full_out = false;
      for (const RNode& n : A.nodes) if (n.out_ord >= 0 && n.cls == CLS_FULL) full_out = true;
      const int64_t rounds = (A.seg_rows + per_round - 1) / per_round;
      const bool fills_badly = A.seg_rows * 10 < rounds * per_round * 9;
      gen.seg_per_wave = share == 1 && gen.L <= 64 && n_seg >= 2048 && A.seg_rows <= 512 && !full_out && (fills_badly || gen.L == 64);
    }
    gen.emit(&l.kernel_name);
    dump_source(gen.e.s);
    std::string cerr;
    if (!ew_compile_source(gen.e.s, &l.code_object, &cerr)) { *err = "generated row schedule: " + cerr; return false; }
    l.L = gen.L; l.K = gen.K; l.W = gen.W;
    l.rows_read_before_written = true;
    for (const RNode& n : A.nodes) if (n.op == ROP_DOT_OUTER || n.op == ROP_DOT_REDUCE) l.rows_read_before_written = false;
    l.lds_bytes = gen.L > 64 ? (int64_t)A.n_reduce * (gen.L / 64) * 4 : gen.stage_bytes;
    l.wg = l.L > 64 ? l.L : gen.wg;     // a team is one workgroup per row
    const int64_t rows_per_wg = l.L > 64 ? 1 : l.wg / l.L;
    int64_t grid = (A.rows + rows_per_wg - 1) / rows_per_wg;
    if (gen.persistent) {
      // a fixed grid loops over the rows: one partial row per workgroup and column reduction
      // (teams: as many workgroups as keep 2048 threads on every CU, but at least sixteen rows each, so
      // that the partial rows stay small beside the rows themselves)
      int64_t want = opt.grid > 0 ? opt.grid : l.L > 64 ? 256 * (2048 / l.L) / 2 : 256;
      if (l.L > 64 && opt.grid <= 0 && want > (A.rows + 15) / 16) want = (A.rows + 15) / 16;
      if (want < grid) grid = want;
      if (n_seg > 0) grid = gen.seg_per_wave ? (n_seg + l.wg / 64 - 1) / (l.wg / 64) : n_seg * gen.seg_groups;      // the runs of rows fix the grid
      l.segmented = A.seg_rows > 0;
      l.seg_count = n_seg;
      l.seg_groups = gen.seg_groups;
      l.persistent = true;
      for (const RNode& n : A.nodes) if (n.cls == CLS_COL) {
        l.col_out[l.n_col] = n.out_ord;
        l.col_dtype[l.n_col] = n.out_dtype;
        l.col_is_max[l.n_col] = n.op == FS_REDUCE_MAX ? 1 : 0;
        ++l.n_col;
      }
      if (A.n_col > 0 && l.L <= 64 && !gen.seg_per_wave) l.lds_bytes = (int64_t)A.n_col * A.cols * 8;
      l.seg_per_wave = gen.seg_per_wave;
      l.workspace_bytes = (n_seg > 0 && gen.seg_groups == 1) ? 0 : (int64_t)A.n_col * grid * A.cols * 8;
      l.n_kernels = A.n_col > 0 && l.workspace_bytes > 0 ? 2 : 1;
    }
    if (gen.mma) {
      // one workgroup per batch element, one wavefront per 16 rows of the tile
      l.mma = true;
      l.mma_dots = A.mma_out >= 0 ? 2 : 1;
      l.mma_k = (int)A.mma_k; l.mma_d = (int)A.mma_d;
      l.wg = gen.wg;
      l.lds_bytes = gen.mma_lds_bytes;
      l.rows_read_before_written = false;
      grid = A.S[0];
      if (opt.wg_size && opt.wg_size != l.wg) {
        *status = FS_ERR_INVALID;
        *err = "generated row schedule: wg_size of a matrix-unit group is fixed at 64 per 16 rows of the tile";
        return false;
      }
    }
    if (grid > 0x7fffffffLL) { *err = "generated row schedule: too many rows for one grid"; return false; }
    l.grid = (int)(grid < 1 ? 1 : grid);
    *out = l;
    *status = FS_OK;
    return true;
  }
  const bool too_long = gerr.find("row longer") != std::string::npos || gerr.find("running sums to stay in registers") != std::string::npos;
  if (!want_stream && (opt.rows_per_wave || !too_long)) { *err = gerr; return false; }
  if (A.mma_in >= 0) { *err = gerr.empty() ? "generated row schedule: dots on the matrix unit have no streamed form" : gerr; return false; }
  if (A.n_col > 0 && A.seg_rows > 0) { *err = "generated row schedule: column reductions per run of rows over rows longer than the register templates hold"; return false; }

  // the row is streamed in passes by one workgroup
  Stream st(A);
  if (A.n_col > 0) {
    // Running values of the column reductions: two registers each, beside about 48 for the rest of the kernel.  A
    // workgroup of 1024 threads has 128 registers per thread, one of 512 has 256, one of 256 has 512: the largest
    // workgroup whose threads can hold their share (rounded up to whole passes) is taken.
    const int sizes[3] = {1024, 512, 256};
    bool fits = false;
    for (int k = 0; k < 3 && !fits; ++k) {
      if (opt.wg_size && k > 0) break;
      if (!st.geometry(opt.wg_size ? opt.wg_size : sizes[k], err)) return false;
      const int64_t per_thread = (int64_t)st.n_iter() * st.W * A.n_col;
      fits = per_thread <= (st.wg > 512 ? 40 : st.wg > 256 ? 104 : 232);
    }
    if (!fits) {
      *err = "generated row schedule: column reductions over rows too long for their running values to stay in registers";
      return false;
    }
  } else if (!st.geometry(opt.wg_size, err)) {
    return false;
  }
  st.schedule();
  std::vector<std::vector<int>> targets;
  const int64_t kLdsLimit = 160 * 1024 - 512;
  st.cached = true;
  st.splat.assign(A.views.size(), 0);
  st.find_cuts(&targets);
  st.plan_buffers();
  const int64_t exch_bytes = (int64_t)A.n_reduce * (st.wg / 64) * 4;
  if (st.lds_floats * 4 + exch_bytes > kLdsLimit) {
    // the shared layout does not fit: keep computed values only and re-read the inputs ...
    st.cache_views = false;
    st.find_cuts(&targets);
    st.plan_buffers();
  }
  if (st.lds_floats * 4 + exch_bytes > kLdsLimit) {
    // ... or keep nothing: every pass recomputes from the inputs
    st.cached = false;
    st.find_cuts(&targets);
    st.lds_floats = 0; st.n_buffers = 0; st.n_shared = 0;
  }
  st.emit(targets, &l.kernel_name);
  dump_source(st.e.s);
  std::string cerr;
  if (!ew_compile_source(st.e.s, &l.code_object, &cerr)) { *err = "generated row schedule: " + cerr; return false; }
  l.streamed = true;
  l.passes = st.n_loops;
  l.row_buffers = st.n_buffers;
  l.buffers_shared = st.n_shared;
  l.inputs_cached = st.cached && st.cache_views;
  l.W = st.W; l.L = st.wg; l.K = 0;
  l.wg = st.wg;
  l.lds_bytes = st.lds_floats * 4 + (int64_t)A.n_reduce * (st.wg / 64) * 4;
  int64_t grid = A.rows;
  if (opt.grid > 0 && opt.grid < grid) grid = opt.grid;
  if (grid > (1 << 22)) grid = 1 << 22;
  if (A.n_col > 0) {
    // a fixed grid walks the rows: workgroups that fill 2048 threads per CU, one partial row each
    const int64_t want = opt.grid > 0 ? opt.grid : 256 * (2048 / st.wg);
    if (grid > want) grid = want;
    for (const RNode& n : A.nodes) if (n.cls == CLS_COL) {
      l.col_out[l.n_col] = n.out_ord;
      l.col_dtype[l.n_col] = n.out_dtype;
      l.col_is_max[l.n_col] = n.op == FS_REDUCE_MAX ? 1 : 0;
      ++l.n_col;
    }
    l.persistent = true;
    if (grid < 1) grid = 1;
    l.workspace_bytes = (int64_t)A.n_col * grid * A.cols * 8;
    l.n_kernels = 2;
  }
  l.grid = (int)(grid < 1 ? 1 : grid);
  *out = l;
  *status = FS_OK;
  return true;
}

std::string row_gen_describe(const RowGenLaunch& l) {
  char buf[720];
  if (l.streamed) {
    char cols[96] = "";
    if (l.n_col > 0) snprintf(cols, sizeof cols, " + column reduce x%d[GRID-THREAD,CTA] (%d partial rows, then a combine kernel)", l.n_col, l.grid);
    snprintf(buf, sizeof buf, "reduce x%d[GRID,CTA-S] + elementwise x%d[GRID,CTA-THREAD_%d]%s streamed in %d passes, %d row buffers in LDS (%d taken over from dominated values)%s (generated kernel %s, %zu bytes of code); cta_num=%d, cta_size=%d, lds=%lld",
             l.n_reduce, l.n_ops - l.n_reduce - l.n_col, l.W, cols, l.passes, l.row_buffers, l.buffers_shared,
             l.passes > 1 && !l.inputs_cached ? ", inputs re-read per pass" : "",
             l.kernel_name.c_str(), l.code_object.size(), l.grid, l.wg, (long long)l.lds_bytes);
    return buf;
  }
  if (l.mma) {
    char tail[160] = "";
    if (l.mma_dots == 2) snprintf(tail, sizeof tail, " + dot_2[GRID,WARP_16,CTA]S (contraction over the tile's %lld columns, %d wide, on MFMA)", (long long)l.cols, l.mma_d);
    snprintf(buf, sizeof buf, "dot_1[GRID,WARP_16,CTA] (contraction %d on MFMA) + reduce x%d[GRID,WARP_16,WARP] + elementwise x%d[GRID,WARP_16,WARP-THREAD_%d]%s block-composed (generated kernel %s, %zu bytes of code); cta_num=%d, cta_size=%d, lds=%lld",
             l.mma_k, l.n_reduce, l.n_ops - l.n_reduce - l.mma_dots, l.K * l.W, tail, l.kernel_name.c_str(), l.code_object.size(), l.grid, l.wg, (long long)l.lds_bytes);
    return buf;
  }
  if (l.persistent && l.n_col == 0) {
    snprintf(buf, sizeof buf, "reduce x%d[GRID,%s] + elementwise x%d[GRID,%s-THREAD_%d] persistent, next row prefetched (generated kernel %s, %zu bytes of code); cta_num=%d, cta_size=%d, lds=%lld",
             l.n_reduce, l.L == 1 ? "THREAD" : "WARP", l.n_ops - l.n_reduce, l.L == 1 ? "CTA" : "WARP", l.K * l.W,
             l.kernel_name.c_str(), l.code_object.size(), l.grid, l.wg, (long long)l.lds_bytes);
    return buf;
  }
  if (l.n_col > 0) {
    char how[160];
    if (l.segmented && l.n_kernels == 1)
      snprintf(how, sizeof how, "column reductions per run of %lld rows, one %s per run", (long long)(l.seg_count ? l.rows / l.seg_count : 0), l.seg_per_wave ? "wavefront" : "workgroup");
    else if (l.segmented)
      snprintf(how, sizeof how, "column reductions per run of %lld rows, %d partial rows per run, then a combine kernel", (long long)(l.seg_count ? l.rows / l.seg_count : 0), l.seg_groups);
    else
      snprintf(how, sizeof how, "%d partial rows, then a combine kernel", l.grid);
    snprintf(buf, sizeof buf, "reduce x%d[GRID,%s] + column reduce x%d[GRID-S,CTA] + elementwise x%d[GRID,%s-THREAD_%d] packed (generated kernel %s, %zu bytes of code; %s); cta_num=%d, cta_size=%d, lds=%lld",
             l.n_reduce, l.L > 64 ? "CTA-S" : "WARP", l.n_col, l.n_ops - l.n_reduce - l.n_col, l.L > 64 ? "CTA" : "WARP", l.K * l.W, l.kernel_name.c_str(), l.code_object.size(), how, l.grid, l.wg,
             (long long)l.lds_bytes);
    return buf;
  }
  snprintf(buf, sizeof buf, "reduce x%d[GRID,%s] + elementwise x%d[GRID,%s-THREAD_%d] (generated kernel %s, %zu bytes of code); cta_num=%d, cta_size=%d, lds=%lld",
           l.n_reduce, l.L == 1 ? "THREAD" : l.L > 64 ? "CTA-S" : "WARP", l.n_ops - l.n_reduce, l.L == 1 ? "CTA" : l.L > 64 ? "CTA" : "WARP", l.K * l.W,
           l.kernel_name.c_str(), l.code_object.size(), l.grid, l.wg, (long long)l.lds_bytes);
  return buf;
}

int row_gen_launch(RowGenLaunch& l, const void* const* in, void* const* out, int n_out, void* workspace, void* stream,
                   std::string* err) {
  if (l.rows == 0 || l.cols == 0) {
    // no rows: the column sums are zero (the combine kernel over zero partial rows writes them)
    if (l.n_col > 0 && l.cols > 0 && !l.segmented) {      // (no rows and sums per run of rows: no run, nothing to write)
      void* col_out[8];
      for (int r = 0; r < l.n_col; ++r) col_out[r] = out[l.col_out[r]];
      return col_combine_launch(nullptr, 0, l.cols, l.n_col, col_out, l.col_dtype, stream, err);
    }
    return 0;
  }
  GenArgs args{};
  for (size_t k = 0; k < l.view_param.size(); ++k) args.in[k] = in[l.view_param[k]];
  for (int k = 0; k < n_out && k < 8; ++k) args.out[k] = out[k];
  args.ws = workspace;
  const int rc = ew_module_launch(&l.loaded, l.code_object, l.kernel_name, &args, sizeof args, l.grid, l.wg, stream, err);
  if (rc != 0 || l.n_col == 0 || l.n_kernels == 1) return rc;
  void* col_out[8];
  for (int r = 0; r < l.n_col; ++r) col_out[r] = out[l.col_out[r]];
  if (l.seg_count > 0) return col_combine_launch(workspace, l.seg_groups, l.cols, l.n_col, col_out, l.col_dtype, stream, err, l.seg_count, l.col_is_max);
  return col_combine_launch(workspace, l.grid, l.cols, l.n_col, col_out, l.col_dtype, stream, err, 1, l.col_is_max);
}

void row_gen_release(RowGenLaunch& l) { ew_module_release(&l.loaded); }

}  // namespace fs
