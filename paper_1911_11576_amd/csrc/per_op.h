// Per-op baseline executor: every op of the group as its own kernel, intermediates as
// whole tensors in a plan-owned HBM workspace.  This is the unfused side of the paper's
// execution-based score (Section 4.3): sum_j K(Op_j) with N launches, against which the
// stitched kernel K(P) is measured.  Broadcasts and constants are folded into their
// consumers' indexing (as a framework with implicit broadcasting does), so they cost no
// launch; a column reduction costs two (partials, then combine).
#pragma once
#include <stdint.h>
#include <string>
#include <vector>
#include "graph.h"

namespace fs {

struct PerOpView {          // how a consumer reads one operand
  int base = -1;            // node that owns the memory (parameter or materialised op); -1: constant
  float cval = 0.f;
  bool full = true;         // same contiguous layout as the consumer's result
  int64_t stride[FS_MAX_RANK] = {0, 0, 0, 0};   // element strides along the consumer's dims
};

// how node `n` (a value of its consumer's shape) maps onto memory: broadcasts and outputs
// are looked through down to the parameter or materialised op that owns the bytes
PerOpView view_of(const Graph& g, int n);

struct PerOpStep {
  int node = -1;
  int kind = 0;             // fs_opkind of the node (FS_OUTPUT: plain copy)
  PerOpView a, b;
  bool vector_ok = false;   // 16-byte path usable
  int64_t outer = 1, red = 1, inner = 1;   // reduce geometry
  int launches = 1;
};

struct PerOpPlan {
  std::vector<PerOpStep> steps;
  std::vector<int64_t> offset;   // per node: workspace offset, -1 if not in the workspace
  std::vector<int> out_of;       // per node: output ordinal whose buffer holds it, or -1
  int64_t scratch_offset = 0, scratch_bytes = 0;   // column-reduce partials
  int n_kernels = 0;
  int64_t workspace_bytes = 0, moved_bytes = 0;
};

bool per_op_plan(const Graph& g, PerOpPlan* plan, std::string* err);
std::string per_op_describe(const PerOpPlan& plan);
int per_op_launch(const Graph& g, const PerOpPlan& plan, const void* const* in, void* const* out,
                  void* workspace, void* stream, std::string* err);

}  // namespace fs
