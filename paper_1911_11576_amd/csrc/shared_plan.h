// Shared-memory planning (paper Section 5.4, Algorithm 4): which ops of a fusion group may
// reuse the shared (LDS) space of an earlier op.  Pure host code.
#pragma once
#include <stdint.h>
#include <vector>

namespace fs {

struct SharedPlanInput {
  // ops in execution order (a topological order of the data-flow graph)
  std::vector<std::vector<int>> operands;   // per op: indices of earlier ops
  std::vector<int64_t> req_bytes;           // per op: shared space its result needs, 0 = none
  std::vector<char> is_output;              // per op: 1 if the group's root consumes it
};
struct SharedPlanResult {
  std::vector<int64_t> offset;              // per op: byte offset of its space, -1 = none
  std::vector<int> shares_with;             // per op: the op whose space it took over, -1 = fresh
  int64_t total_bytes = 0;                  // worst-case footprint
};

// Immediate dominators in the data-flow graph seen from the group's root (edges run from
// a user to its operands; a virtual root uses every output): idom[i] = -1 for ops whose
// immediate dominator is the root itself, -2 for ops the root does not reach.
std::vector<int> dataflow_idom(const SharedPlanInput& in);
// true if every path from the root to `b` passes through `a` (a != b)
bool dominates(const std::vector<int>& idom, int a, int b);

SharedPlanResult shared_plan(const SharedPlanInput& in);

}  // namespace fs
