// Validation of a fusion group: topological order, operand counts, shapes and dtypes of
// every op of the vocabulary in fs.h.  Pure host code.
#include "graph.h"

#include <cstdio>

namespace fs {

const char* kind_name(int k) {
  static const char* names[FS_NUM_OPKINDS] = {
      "parameter", "constant", "add", "subtract", "multiply", "divide", "maximum", "negate", "exp",
      "log", "tanh", "rsqrt", "sqrt", "convert", "broadcast", "reduce_sum", "reduce_max", "dot",
      "causal_mask", "output", "erf", "logistic"};
  return (k >= 0 && k < FS_NUM_OPKINDS) ? names[k] : "?";
}

int64_t Graph::algorithmic_bytes() const {
  int64_t total = 0;
  for (int i : params) total += nodes[i].numel() * (nodes[i].dtype == FS_F32 ? 4 : 2);
  for (int i : outputs) total += nodes[i].numel() * (nodes[i].dtype == FS_F32 ? 4 : 2);
  return total;
}

namespace {

struct Fail {
  std::string* err;
  int index;
  bool operator()(const char* what) const {
    char buf[256];
    snprintf(buf, sizeof buf, "op %d: %s", index, what);
    *err = buf;
    return false;
  }
};

}  // namespace

bool build_graph(const fs_op_desc* ops, int32_t n_ops, Graph* g, std::string* err) {
  if (!ops) { *err = "ops is NULL"; return false; }
  if (n_ops < 1 || n_ops > 4096) { *err = "n_ops out of range [1,4096]"; return false; }
  g->nodes.clear(); g->params.clear(); g->outputs.clear();
  g->nodes.reserve(n_ops);
  std::vector<char> consumed_output(n_ops, 0);
  for (int i = 0; i < n_ops; ++i) {
    const fs_op_desc& d = ops[i];
    Fail fail{err, i};
    if (d.kind < 0 || d.kind >= FS_NUM_OPKINDS) return fail("unknown op kind");
    if (d.dtype < FS_F32 || d.dtype > FS_BF16) return fail("unknown dtype");
    if (d.rank < 0 || d.rank > FS_MAX_RANK) return fail("rank out of range");
    if (d.reserved != 0) return fail("reserved field must be 0");
    Node n;
    n.kind = d.kind; n.dtype = d.dtype; n.rank = d.rank; n.axis = d.axis; n.attr = d.attr;
    // every extent and the running product stay below 2^40, so the product cannot wrap; an extent of 0
    // makes the tensor empty whatever the other extents are
    bool empty = false;
    for (int k = 0; k < d.rank; ++k) empty = empty || d.shape[k] == 0;
    int64_t running = 1;
    for (int k = 0; k < d.rank; ++k) {
      if (d.shape[k] < 0) return fail("negative extent");
      if (d.shape[k] >= ((int64_t)1 << 40)) return fail("tensor too large");
      if (!empty) {
        running *= d.shape[k];
        if (running >= ((int64_t)1 << 40)) return fail("tensor too large");
      }
      n.shape[k] = d.shape[k];
    }
    const int nop = operand_count(d.kind);
    for (int k = 0; k < 3; ++k) {
      if (k < nop) {
        if (d.operand[k] < 0 || d.operand[k] >= i) return fail("operand must refer to an earlier op");
        if (g->nodes[d.operand[k]].kind == FS_OUTPUT) return fail("an output op cannot be consumed");
        n.operand[k] = d.operand[k];
      } else if (d.operand[k] != -1) {
        return fail("unused operand slot must be -1");
      }
    }
    const Node* a = nop > 0 ? &g->nodes[n.operand[0]] : nullptr;
    const Node* b = nop > 1 ? &g->nodes[n.operand[1]] : nullptr;
    switch (d.kind) {
      case FS_PARAMETER:
        n.ordinal = (int)g->params.size();
        g->params.push_back(i);
        break;
      case FS_CONSTANT:
        if (n.rank != 0) return fail("constant must have rank 0");
        break;
      case FS_ADD: case FS_SUBTRACT: case FS_MULTIPLY: case FS_DIVIDE: case FS_MAXIMUM: {
        const bool ca = a->kind == FS_CONSTANT, cb = b->kind == FS_CONSTANT;
        if (ca && cb) return fail("binary op of two constants");
        if (!ca && !(a->same_shape(n) && a->dtype == n.dtype)) return fail("operand 0 shape/dtype differs from result");
        if (!cb && !(b->same_shape(n) && b->dtype == n.dtype)) return fail("operand 1 shape/dtype differs from result");
        break;
      }
      case FS_NEGATE: case FS_EXP: case FS_LOG: case FS_TANH: case FS_RSQRT: case FS_SQRT: case FS_ERF: case FS_LOGISTIC:
        if (!(a->same_shape(n) && a->dtype == n.dtype)) return fail("operand shape/dtype differs from result");
        break;
      case FS_CONVERT:
        if (!a->same_shape(n)) return fail("convert changes the shape");
        break;
      case FS_BROADCAST: {
        if (a->dtype != n.dtype) return fail("broadcast changes the dtype");
        if (a->kind == FS_CONSTANT) return fail("broadcast of a rank-0 constant: use the constant directly");
        if (n.axis < 0 || n.axis + a->rank > n.rank) return fail("broadcast axis out of range");
        for (int k = 0; k < a->rank; ++k)
          if (a->shape[k] != 1 && a->shape[k] != n.shape[n.axis + k]) return fail("broadcast extent mismatch");
        break;
      }
      case FS_REDUCE_SUM: case FS_REDUCE_MAX: {
        if (a->dtype != n.dtype) return fail("reduce changes the dtype");
        if (a->rank < 1 || n.axis < 0 || n.axis >= a->rank) return fail("reduce axis out of range");
        if (n.rank != a->rank - 1) return fail("reduce result must drop the reduced dim");
        for (int k = 0, j = 0; k < a->rank; ++k) {
          if (k == n.axis) continue;
          if (n.shape[j++] != a->shape[k]) return fail("reduce result extent mismatch");
        }
        if (d.kind == FS_REDUCE_MAX && a->shape[n.axis] == 0) return fail("reduce_max over an empty dim");
        break;
      }
      case FS_DOT: {
        if (a->rank != 3 || b->rank != 3 || n.rank != 3) return fail("dot operands and result must have rank 3");
        if (a->dtype != b->dtype) return fail("dot operands differ in dtype");
        if (n.axis != 0 && n.axis != 1) return fail("dot axis must be 0 or 1");
        const int64_t kb = n.axis ? b->shape[2] : b->shape[1], nb = n.axis ? b->shape[1] : b->shape[2];
        if (a->shape[0] != b->shape[0] || a->shape[2] != kb) return fail("dot operand extents mismatch");
        if (n.shape[0] != a->shape[0] || n.shape[1] != a->shape[1] || n.shape[2] != nb)
          return fail("dot result extents mismatch");
        break;
      }
      case FS_CAUSAL_MASK:
        if (n.rank < 2) return fail("causal_mask needs rank >= 2");
        if (!(a->same_shape(n) && a->dtype == n.dtype)) return fail("operand shape/dtype differs from result");
        break;
      case FS_OUTPUT:
        if (!(a->same_shape(n) && a->dtype == n.dtype)) return fail("output shape/dtype differs from its operand");
        if (a->kind == FS_CONSTANT) return fail("output of a constant");
        if (consumed_output[n.operand[0]]) return fail("value is already an output");
        consumed_output[n.operand[0]] = 1;
        n.ordinal = (int)g->outputs.size();
        g->outputs.push_back(i);
        break;
      default:
        return fail("unknown op kind");
    }
    g->nodes.push_back(n);
  }
  if (g->params.empty()) { *err = "group has no parameter"; return false; }
  if (g->outputs.empty()) { *err = "group has no output"; return false; }
  if (g->params.size() > 64 || g->outputs.size() > 16) { *err = "too many parameters or outputs"; return false; }
  return true;
}

// A reduction over the last dim whose only reader reduces the result over ITS last dim, by the same
// operator, is one reduction over the two trailing dims taken as one: tensors are dense, so [.., B, C]
// read as [.., B*C] is the same memory.  The rewritten list has one reduction less and its full
// values one dim less; every kernel schedule sees a plain reduction over the last dim.  Applies
// only where nothing else distinguishes the two trailing dims: every op of full rank has the full
// shape, every op one dim shorter is such an inner reduction, and what is broadcast into the full
// shape covers leading dims only.  At least one leading dim is kept (a reduction of everything to
// a scalar stays a chain: one row would leave the whole tensor to one workgroup).
bool collapse_trailing_reductions(const Graph& g, std::vector<fs_op_desc>* out) {
  const int n = g.size();
  std::vector<int> readers(n, 0), reader_of(n, -1);
  for (int i = 0; i < n; ++i)
    for (int j = 0; j < operand_count(g[i].kind); ++j) { ++readers[g[i].operand[j]]; reader_of[g[i].operand[j]] = i; }
  auto is_reduce = [](int k) { return k == FS_REDUCE_SUM || k == FS_REDUCE_MAX; };
  auto inner_of = [&](int i) {      // i is the inner reduction of a collapsible pair
    const Node& r1 = g[i];
    if (!is_reduce(r1.kind) || readers[i] != 1) return false;
    const Node& x = g[r1.operand[0]];
    const Node& r2 = g[reader_of[i]];
    return x.rank >= 3 && r1.axis == x.rank - 1 && r2.kind == r1.kind && r2.axis == r1.rank - 1;
  };
  int first = -1;
  for (int i = 0; i < n && first < 0; ++i) if (inner_of(i)) first = i;
  if (first < 0) return false;
  const Node& full = g[g[first].operand[0]];
  const int r = full.rank;
  for (int i = 0; i < n; ++i) {
    const Node& x = g[i];
    if (x.kind == FS_DOT || x.kind == FS_CAUSAL_MASK) return false;
    if (x.rank > r) return false;
    if (x.rank == r && !x.same_shape(full)) return false;
    if (x.rank == r - 1 && !(inner_of(i) && g[x.operand[0]].same_shape(full))) return false;
    if (x.kind == FS_BROADCAST && x.rank == r && x.axis + g[x.operand[0]].rank > r - 2) return false;
    if (x.kind == FS_BROADCAST && x.rank == r - 1) return false;
  }
  std::vector<int> remap(n, -1);
  out->clear();
  for (int i = 0; i < n; ++i) {
    const Node& x = g[i];
    if (x.rank == r - 1 && is_reduce(x.kind)) { remap[i] = remap[x.operand[0]]; continue; }   // the inner reduction: its reader reads the full value
    fs_op_desc d{};
    d.kind = x.kind; d.dtype = x.dtype; d.rank = x.rank; d.axis = x.axis; d.attr = x.attr;
    for (int k = 0; k < x.rank; ++k) d.shape[k] = x.shape[k];
    if (x.rank == r) {
      d.rank = r - 1;
      d.shape[r - 2] = full.shape[r - 2] * full.shape[r - 1];
      d.shape[r - 1] = 0;
    }
    const int nop = operand_count(x.kind);
    for (int k = 0; k < 3; ++k) d.operand[k] = k < nop ? remap[x.operand[k]] : -1;
    if (is_reduce(x.kind) && g[x.operand[0]].rank == r - 1) d.axis = r - 2;     // the outer reduction, now over the merged dim
    remap[i] = (int)out->size();
    out->push_back(d);
  }
  return true;
}

// A reduction over the leading dim that keeps all the others ([B, S, H] -> [S, H]) is a column reduction
// of the same memory read as [B, S*H] -> [S*H]: tensors are dense, so the kept dims merge into one.  The
// rewritten list has rank-2 full values and rank-1 kept values; the schedules then see sums (or maxima)
// over the rows of a matrix.  Applies where nothing tells the kept dims apart: every op has the full
// shape, the kept shape or rank 0, every reduction runs over the leading dim of a full value, and what is
// broadcast into the full shape is a kept-shape value or a scalar.
bool collapse_kept_dims_of_leading_reductions(const Graph& g, std::vector<fs_op_desc>* out) {
  const int n = g.size();
  auto is_reduce = [](int k) { return k == FS_REDUCE_SUM || k == FS_REDUCE_MAX; };
  int first = -1;
  for (int i = 0; i < n && first < 0; ++i)
    if (is_reduce(g[i].kind) && g[i].axis == 0 && g[g[i].operand[0]].rank >= 3) first = i;
  if (first < 0) return false;
  const Node& full = g[g[first].operand[0]];
  const int r = full.rank;
  auto is_kept = [&](const Node& x) {
    if (x.rank != r - 1) return false;
    for (int d = 0; d < r - 1; ++d) if (x.shape[d] != full.shape[d + 1]) return false;
    return true;
  };
  for (int i = 0; i < n; ++i) {
    const Node& x = g[i];
    if (x.kind == FS_DOT || x.kind == FS_CAUSAL_MASK) return false;
    if (!(x.rank == 0 || (x.rank == r && x.same_shape(full)) || is_kept(x))) return false;
    if (is_reduce(x.kind) && !(x.axis == 0 && g[x.operand[0]].rank == r)) return false;
    if (x.kind == FS_BROADCAST) {
      const Node& a = g[x.operand[0]];
      if (a.rank == 0) continue;
      if (!(x.rank == r && is_kept(a) && x.axis == 1)) return false;
    }
  }
  int64_t merged = 1;
  for (int d = 1; d < r; ++d) merged *= full.shape[d];
  out->clear();
  for (int i = 0; i < n; ++i) {
    const Node& x = g[i];
    fs_op_desc d{};
    d.kind = x.kind; d.dtype = x.dtype; d.rank = x.rank; d.axis = x.axis; d.attr = x.attr;
    if (x.rank == r) { d.rank = 2; d.shape[0] = full.shape[0]; d.shape[1] = merged; }
    else if (x.rank == r - 1) { d.rank = 1; d.shape[0] = merged; }
    if (x.kind == FS_BROADCAST) d.axis = g[x.operand[0]].rank == 0 ? 0 : 1;
    const int nop = operand_count(x.kind);
    for (int k = 0; k < 3; ++k) d.operand[k] = k < nop ? x.operand[k] : -1;
    out->push_back(d);
  }
  return true;
}

}  // namespace fs
