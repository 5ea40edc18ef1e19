// Shared-memory planning (paper Section 5.4, Algorithm 4).
//
// Ops are visited in execution order.  An op that needs no shared space passes on the
// allocation information of its operands (which spaces its inputs still live in).  An op
// that needs space looks at the spaces reaching it through its operands: a space whose owner
// is dominated by the op (every path from the group's root to the owner runs through the
// op: once the op has produced its result nothing else will read the owner's value) can be
// taken over; the first such space is shared, the others are reclaimed for later ops.  If
// none can be taken over, a reclaimed space that is large enough is reused, else fresh
// space is allocated.  The goal, as in the paper, is to bound the worst-case footprint, not
// to find the minimum.
#include "shared_plan.h"

#include <algorithm>
#include <set>

namespace fs {

std::vector<int> dataflow_idom(const SharedPlanInput& in) {
  const int n = (int)in.operands.size();
  // Vertices 0..n-1 are the ops, vertex n is the virtual root.  In the graph seen from the
  // root, the predecessors of an op are its users (and the root, for outputs).  Execution
  // order reversed is a reverse postorder of that graph: every user comes after its operands.
  std::vector<std::vector<int>> users(n);
  std::vector<char> used(n, 0);
  for (int i = 0; i < n; ++i)
    for (int o : in.operands[i]) { users[o].push_back(i); used[o] = 1; }
  const int root = n;
  for (int i = 0; i < n; ++i) {
    const bool out = in.is_output.empty() ? !used[i] : in.is_output[i] != 0;
    if (out) users[i].push_back(root);
  }
  // Cooper-Harvey-Kennedy iteration; order number = position in the traversal from the root:
  // the root first, then ops from last to first.
  auto order_of = [&](int v) { return v == root ? 0 : n - v; };
  std::vector<int> idom(n + 1, -2);
  idom[root] = root;
  auto intersect = [&](int a, int b) {
    while (a != b) {
      while (order_of(a) > order_of(b)) a = idom[a];
      while (order_of(b) > order_of(a)) b = idom[b];
    }
    return a;
  };
  bool changed = true;
  while (changed) {
    changed = false;
    for (int v = n - 1; v >= 0; --v) {
      int cand = -2;
      for (int u : users[v]) {
        if (idom[u] == -2) continue;            // user not reached from the root (yet)
        cand = cand == -2 ? u : intersect(cand, u);
      }
      if (cand != -2 && idom[v] != cand) { idom[v] = cand; changed = true; }
    }
  }
  std::vector<int> res(n);
  for (int i = 0; i < n; ++i) res[i] = idom[i] == root ? -1 : idom[i];
  return res;
}

bool dominates(const std::vector<int>& idom, int a, int b) {
  if (a == b || idom[b] == -2) return false;
  for (int v = idom[b]; v >= 0; v = idom[v]) if (v == a) return true;
  return false;
}

SharedPlanResult shared_plan(const SharedPlanInput& in) {
  const int n = (int)in.operands.size();
  SharedPlanResult r;
  r.offset.assign(n, -1);
  r.shares_with.assign(n, -1);
  const std::vector<int> idom = dataflow_idom(in);
  struct Block { int64_t offset, bytes; };
  std::vector<Block> block_of(n, Block{-1, 0});     // the space an op currently owns
  std::vector<Block> reclaimed;                      // spaces free for later ops
  std::vector<std::set<int>> info(n);                // per op: owners of the spaces its value still depends on
  for (int i = 0; i < n; ++i) {
    std::set<int> prev;                              // CollectAllocInfo over the operands
    for (int o : in.operands[i]) prev.insert(info[o].begin(), info[o].end());
    if (in.req_bytes[i] <= 0) { info[i] = prev; continue; }   // PropagateAllocInfo
    const int64_t need = in.req_bytes[i];
    bool shared = false;
    std::set<int> still;
    for (int p : prev) {
      if (block_of[p].offset < 0) continue;          // already handed on
      if (dominates(idom, i, p)) {
        if (!shared && block_of[p].bytes >= need) {  // Share
          block_of[i] = block_of[p];
          r.shares_with[i] = p;
          shared = true;
        } else {                                     // Reclaim
          reclaimed.push_back(block_of[p]);
        }
        block_of[p] = Block{-1, 0};
      } else {
        still.insert(p);
      }
    }
    if (!shared) {                                   // Alloc: a reclaimed space that fits, else fresh space
      int best = -1;
      for (size_t k = 0; k < reclaimed.size(); ++k)
        if (reclaimed[k].bytes >= need && (best < 0 || reclaimed[k].bytes < reclaimed[best].bytes)) best = (int)k;
      if (best >= 0) {
        block_of[i] = reclaimed[best];
        reclaimed.erase(reclaimed.begin() + best);
      } else {
        block_of[i] = Block{r.total_bytes, need};
        r.total_bytes += need;
      }
    }
    r.offset[i] = block_of[i].offset;
    still.insert(i);
    info[i] = still;
  }
  return r;
}

}  // namespace fs
