// Validated host copy of a fusion group (the op list handed to fs_plan_create).
#pragma once
#include <stdint.h>
#include <string>
#include <vector>
#include "../../include/fs.h"

namespace fs {

struct Node {
  int kind = 0, dtype = 0, rank = 0, axis = 0;
  int64_t shape[FS_MAX_RANK] = {0, 0, 0, 0};
  int operand[3] = {-1, -1, -1};
  double attr = 0.0;
  int ordinal = -1;   // parameter ordinal or output ordinal

  int64_t numel() const {
    int64_t n = 1;
    for (int d = 0; d < rank; ++d) n *= shape[d];
    return n;
  }
  bool same_shape(const Node& o) const {
    if (rank != o.rank) return false;
    for (int d = 0; d < rank; ++d) if (shape[d] != o.shape[d]) return false;
    return true;
  }
};

struct Graph {
  std::vector<Node> nodes;
  std::vector<int> params;    // node index of each parameter, in order
  std::vector<int> outputs;   // node index of each FS_OUTPUT op, in order
  const Node& operator[](int i) const { return nodes[i]; }
  int size() const { return (int)nodes.size(); }
  int64_t algorithmic_bytes() const;
};

// Copies and checks the list.  On failure returns false and sets *err.
bool build_graph(const fs_op_desc* ops, int32_t n_ops, Graph* g, std::string* err);

// One step of merging chained reductions over the two trailing dims into a reduction over one merged
// dim; true (and the rewritten op list) if the group allows it.  See graph.cpp.
bool collapse_trailing_reductions(const Graph& g, std::vector<fs_op_desc>* out);
// Reductions over the leading dim that keep all other dims ([B, S, H] -> [S, H]): the kept dims merged
// into one, so that the group is a matrix [B, S*H] with reductions over its rows.  See graph.cpp.
bool collapse_kept_dims_of_leading_reductions(const Graph& g, std::vector<fs_op_desc>* out);

inline bool is_binary(int k) { return k >= FS_ADD && k <= FS_MAXIMUM; }
inline bool is_unary(int k) { return (k >= FS_NEGATE && k <= FS_SQRT) || k == FS_ERF || k == FS_LOGISTIC; }
// how many entries of Node::operand an op of this kind reads
inline int operand_count(int k) { return k == FS_PARAMETER || k == FS_CONSTANT ? 0 : (is_binary(k) || k == FS_DOT) ? 2 : 1; }
const char* kind_name(int k);

}  // namespace fs
