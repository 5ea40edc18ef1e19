// Shared-memory planning (paper Section 5.4, Algorithm 4): an arena of LDS blocks, a dominance tree
// of the group's data-flow graph, and one walk over the ops in execution order that decides for every
// request whether it takes over the block of a value it dominates, reuses a freed block or grows the
// arena.  The goal, as in the paper, is to bound the worst-case footprint, not to find the minimum.
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

namespace {

// The LDS arena: blocks carved out of one growing range.  A block has an owner (the op whose value
// lives in it) or is free; a free block keeps its place and size and is handed to the next request it
// is large enough for.
struct Arena {
  struct Block { int64_t offset, bytes; int owner; };   // owner -1: free
  std::vector<Block> blocks;
  int64_t top = 0;
  int grow(int64_t bytes, int owner) {
    blocks.push_back(Block{top, bytes, owner});
    top += bytes;
    return (int)blocks.size() - 1;
  }
  // the smallest free block that holds `bytes`, or -1
  int best_free(int64_t bytes) const {
    int best = -1;
    for (size_t k = 0; k < blocks.size(); ++k)
      if (blocks[k].owner < 0 && blocks[k].bytes >= bytes && (best < 0 || blocks[k].bytes < blocks[best].bytes)) best = (int)k;
    return best;
  }
};

}  // namespace

// Every value carries the set of arena blocks it still depends on: its own block, if it has one, and the
// blocks of the values it was computed from, as long as those values may be read again.  A value that
// needs space may take the block of a value it dominates (Section 5.4: once the dominating op has
// produced its result, nothing reads the dominated value any more); the other blocks of dominated
// values in its set become free.
SharedPlanResult shared_plan(const SharedPlanInput& in) {
  const int n = (int)in.operands.size();
  SharedPlanResult r;
  r.offset.assign(n, -1);
  r.shares_with.assign(n, -1);
  const std::vector<int> idom = dataflow_idom(in);
  Arena arena;
  std::vector<std::vector<int>> depends(n);          // per op: arena blocks in use below it, ordered by owner
  auto by_owner = [&](int a, int b) { return arena.blocks[a].owner < arena.blocks[b].owner; };
  for (int i = 0; i < n; ++i) {
    std::vector<int>& mine = depends[i];
    for (int o : in.operands[i]) mine.insert(mine.end(), depends[o].begin(), depends[o].end());
    // blocks that changed hands since an operand recorded them no longer hold that operand's input
    mine.erase(std::remove_if(mine.begin(), mine.end(), [&](int k) { return arena.blocks[k].owner < 0 || arena.blocks[k].owner >= i; }), mine.end());
    std::sort(mine.begin(), mine.end(), by_owner);
    mine.erase(std::unique(mine.begin(), mine.end()), mine.end());
    const int64_t need = in.req_bytes[i];
    if (need <= 0) continue;
    int taken = -1;
    std::vector<int> kept;
    for (int k : mine) {
      Arena::Block& b = arena.blocks[k];
      if (!dominates(idom, i, b.owner)) { kept.push_back(k); continue; }
      if (taken < 0 && b.bytes >= need) { taken = k; r.shares_with[i] = b.owner; b.owner = i; }
      else b.owner = -1;
    }
    if (taken < 0) {
      taken = arena.best_free(need);
      if (taken >= 0) arena.blocks[taken].owner = i;
      else taken = arena.grow(need, i);
    }
    r.offset[i] = arena.blocks[taken].offset;
    kept.push_back(taken);
    mine = kept;
  }
  r.total_bytes = arena.top;
  return r;
}

}  // namespace fs
