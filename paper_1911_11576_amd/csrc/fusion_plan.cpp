// Fusion planning (paper Section 4).
//
//   patterns   substitution fusion (Algorithm 1) under a growing set of partition ops (large
//              dots; then every dot; then column reductions; then every reduction), each
//              segment also split into its connected parts; exploratory fusion (Algorithm 2)
//              from ops with large results, bounded by a visit budget
//   scores     model based (Section 4.3): f(P) = M(V) + (N-1)*phi, V the off-chip bytes the
//              fused kernel does not move, M from a measured bandwidth-vs-bytes table; negative
//              if the kernel generator / recogniser cannot take the pattern
//   selection  maximise the summed score over pairwise disjoint patterns (the ILP of Section
//              4.1, solved by branch and bound over at most 256 patterns per conflict component); if the chosen
//              patterns make the contracted graph cyclic, the patterns on the cycle are forbidden
//              as a set and the problem is solved again
//
// Constants and broadcasts own no kernel: they are copied into every group that reads them.
#include "fusion_plan.h"

#include <algorithm>
#include <cmath>
#include <functional>
#include <map>
#include <set>

#include "ew_ir.h"

namespace fs {

namespace {

bool is_free(const Node& x) { return x.kind == FS_CONSTANT || x.kind == FS_BROADCAST; }
bool is_reduce_kind(int k) { return k == FS_REDUCE_SUM || k == FS_REDUCE_MAX; }
int64_t value_bytes(const Node& x) { return x.numel() * (x.dtype == FS_F32 ? 4 : 2); }
int n_operands(const Node& x) {
  if (x.kind == FS_PARAMETER || x.kind == FS_CONSTANT) return 0;
  return (is_binary(x.kind) || x.kind == FS_DOT) ? 2 : 1;
}

// Data flow between kernel-owning ops, seen through the free nodes.
struct Flow {
  const Graph& g;
  std::vector<std::vector<int>> producers;   // per op: owned ops and parameters it reads (through free nodes)
  std::vector<std::vector<int>> consumers;   // per op / parameter: owned ops and output ops that read it
  explicit Flow(const Graph& gr) : g(gr), producers(gr.size()), consumers(gr.size()) {
    const int n = g.size();
    // sources[i]: the owned ops / parameters behind node i (i itself unless free)
    std::vector<std::vector<int>> sources(n);
    for (int i = 0; i < n; ++i) {
      const Node& x = g[i];
      std::vector<int> in;
      for (int j = 0; j < n_operands(x); ++j)
        for (int s : sources[x.operand[j]]) if (std::find(in.begin(), in.end(), s) == in.end()) in.push_back(s);
      if (is_free(x)) { sources[i] = in; continue; }
      sources[i] = {i};
      if (x.kind == FS_PARAMETER) continue;
      producers[i] = in;
      for (int s : in) consumers[s].push_back(i);
    }
  }
};

}  // namespace

bool fusion_owns_kernel(const Graph& g, int op) {
  const Node& x = g[op];
  return !(x.kind == FS_PARAMETER || x.kind == FS_OUTPUT || is_free(x));
}

bool fusion_is_convex(const Graph& g, const std::vector<int>& ops) {
  Flow f(g);
  std::vector<char> in(g.size(), 0), seen(g.size(), 0);
  for (int o : ops) in[o] = 1;
  std::vector<int> stack;
  for (int o : ops) for (int c : f.consumers[o]) if (!in[c] && !seen[c]) { seen[c] = 1; stack.push_back(c); }
  while (!stack.empty()) {
    const int v = stack.back();
    stack.pop_back();
    for (int c : f.consumers[v]) {
      if (in[c]) return false;                 // left the set and came back
      if (!seen[c]) { seen[c] = 1; stack.push_back(c); }
    }
  }
  return true;
}

int64_t fusion_saved_bytes(const Graph& g, const std::vector<int>& ops) {
  Flow f(g);
  std::vector<char> in(g.size(), 0);
  for (int o : ops) in[o] = 1;
  int64_t saved = 0;
  // values produced inside: reads by inside consumers disappear; the write too if nothing outside reads it
  for (int o : ops) {
    int inside = 0, outside = 0;
    for (int c : f.consumers[o]) (in[c] ? inside : outside)++;
    saved += (int64_t)inside * value_bytes(g[o]);
    if (outside == 0 && inside > 0) saved += value_bytes(g[o]);
  }
  // values from outside read by several ops of the pattern are read once
  std::map<int, int> reads;
  for (int o : ops) for (int p : f.producers[o]) if (!in[p]) reads[p]++;
  for (const auto& kv : reads) if (kv.second > 1) saved += (int64_t)(kv.second - 1) * value_bytes(g[kv.first]);
  return saved;
}

double fusion_model_us(const FusionConfig& cfg, int64_t bytes) {
  // measured on MI355X with the plain copy kernel (bytes moved, GB/s); used unless the caller brings a table
  static const std::pair<int64_t, double> kDefault[] = {
      {1 << 20, 400.0}, {4 << 20, 1500.0}, {16 << 20, 2600.0}, {32 << 20, 4600.0}, {64 << 20, 5300.0},
      {128 << 20, 5900.0}, {256 << 20, 6300.0}, {512 << 20, 6400.0}, {1024 << 20, 6500.0}};
  std::vector<std::pair<int64_t, double>> table = cfg.bandwidth;
  if (table.empty()) table.assign(kDefault, kDefault + sizeof kDefault / sizeof kDefault[0]);
  if (bytes <= 0) return 0.0;
  double gbs = table.back().second;
  if (bytes <= table.front().first) gbs = table.front().second;
  else for (size_t k = 1; k < table.size(); ++k) {
    if (bytes <= table[k].first) {      // interpolate in log(bytes)
      const double a = std::log((double)table[k - 1].first), b = std::log((double)table[k].first);
      const double t = (std::log((double)bytes) - a) / (b - a);
      gbs = table[k - 1].second + t * (table[k].second - table[k - 1].second);
      break;
    }
  }
  return (double)bytes / (gbs * 1e9) * 1e6;
}

namespace {

// The pattern as a stand-alone op list: parameters for what it reads from outside, its own
// ops with the free nodes they need, outputs for what is read outside.
void extract(const std::vector<fs_op_desc>& all, const Graph& g, const Flow& f, const std::vector<int>& ops,
             FusionGroup* out) {
  const int n = g.size();
  std::vector<char> in(n, 0), take(n, 0);
  for (int o : ops) in[o] = take[o] = 1;
  // free nodes needed, walking operands from the owned ops
  std::function<void(int)> need = [&](int i) {
    const Node& x = g[i];
    for (int j = 0; j < n_operands(x); ++j) {
      const int a = x.operand[j];
      if (is_free(g[a]) && !take[a]) { take[a] = 1; need(a); }
    }
  };
  for (int o : ops) need(o);
  std::vector<int> remap(n, -1);
  out->ops = ops;
  out->list.clear(); out->input_of.clear(); out->output_of.clear();
  auto param_for = [&](int src) {
    if (remap[src] >= 0) return;
    fs_op_desc d{};
    d.kind = FS_PARAMETER; d.dtype = g[src].dtype; d.rank = g[src].rank; d.axis = 0;
    for (int k = 0; k < FS_MAX_RANK; ++k) d.shape[k] = k < g[src].rank ? g[src].shape[k] : 0;
    d.operand[0] = d.operand[1] = d.operand[2] = -1;
    remap[src] = (int)out->list.size();
    out->list.push_back(d);
    out->input_of.push_back(src);
  };
  for (int i = 0; i < n; ++i) {
    if (!take[i]) continue;
    const Node& x = g[i];
    for (int j = 0; j < n_operands(x); ++j) if (!take[x.operand[j]]) param_for(x.operand[j]);
  }
  for (int i = 0; i < n; ++i) {
    if (!take[i]) continue;
    fs_op_desc d = all[i];
    for (int j = 0; j < 3; ++j) d.operand[j] = j < n_operands(g[i]) ? remap[g[i].operand[j]] : -1;
    remap[i] = (int)out->list.size();
    out->list.push_back(d);
  }
  for (int o : ops) {
    bool outside = false;
    for (int c : f.consumers[o]) if (!in[c]) outside = true;
    if (!outside) continue;
    fs_op_desc d{};
    d.kind = FS_OUTPUT; d.dtype = g[o].dtype; d.rank = g[o].rank;
    for (int k = 0; k < FS_MAX_RANK; ++k) d.shape[k] = k < g[o].rank ? g[o].shape[k] : 0;
    d.operand[0] = remap[o]; d.operand[1] = d.operand[2] = -1;
    out->list.push_back(d);
    out->output_of.push_back(o);
  }
}

}  // namespace

}  // namespace fs

// the public plan constructor, used in dry-run mode to ask whether a pattern can be generated
extern "C" fs_status fs_plan_create(const fs_op_desc* ops, int32_t n_ops, const fs_plan_options* opt, fs_plan** out);
extern "C" fs_status fs_destroy(fs_plan* plan);

namespace fs {

namespace {

bool generable(const FusionGroup& gr) {
  if (gr.list.empty() || gr.output_of.empty()) return false;
  fs_plan* p = nullptr;
  codegen_set_dry_run(true);
  const fs_status st = fs_plan_create(gr.list.data(), (int32_t)gr.list.size(), nullptr, &p);
  codegen_set_dry_run(false);
  if (st != FS_OK) return false;
  fs_destroy(p);
  return true;
}

struct Planner {
  const std::vector<fs_op_desc>& all;
  const Graph& g;
  const FusionConfig& cfg;
  Flow f;
  std::vector<int> owned;                      // kernel-owning ops in list order
  std::map<std::vector<int>, int> index_of;    // op set -> pattern number
  std::vector<FusionPattern> patterns;

  Planner(const std::vector<fs_op_desc>& a, const Graph& gr, const FusionConfig& c) : all(a), g(gr), cfg(c), f(gr) {
    for (int i = 0; i < g.size(); ++i) if (fusion_owns_kernel(g, i)) owned.push_back(i);
  }

  bool small_dot(const Node& x) const {
    if (x.kind != FS_DOT) return false;
    const Node& a = g[x.operand[0]];
    return a.shape[a.rank - 1] <= 8 || x.shape[x.rank - 1] == 1;     // arithmetic on a row's registers, no matrix unit
  }
  // a dot that a stitched kernel can hold: arithmetic on registers, or fine-grained enough for one workgroup's
  // matrix-unit tile (Section 5.1 composes batched GEMMs of that size with the ops around them); larger dots are
  // library calls and part the graph
  bool fine_dot(const Node& x) const {
    if (small_dot(x)) return true;
    if (x.kind != FS_DOT || x.rank != 3) return false;
    const Node& a = g[x.operand[0]];
    return a.rank == 3 && x.shape[1] <= 128 && x.shape[2] <= 128 && a.shape[2] <= 128;
  }
  bool row_reduce(const Node& x) const { return is_reduce_kind(x.kind) && x.axis == g[x.operand[0]].rank - 1; }

  void add(std::vector<int> ops, int origin) {
    std::sort(ops.begin(), ops.end());
    if (ops.size() < 2 || (int)ops.size() > cfg.max_pattern_ops) return;
    if (index_of.count(ops)) return;
    FusionPattern p;
    p.ops = ops;
    p.origin = origin;
    index_of[ops] = (int)patterns.size();
    patterns.push_back(p);
  }

  // Algorithm 1: all ops between adjacent partition ops (in list order) form one pattern
  void substitution(const std::function<bool(const Node&)>& is_partition) {
    std::vector<int> seg;
    auto flush = [&]() {
      if (seg.size() >= 2) {
        add(seg, 0);
        // a segment beyond the size a pattern may have: its consecutive stretches of that size, and of
        // half that size (any stretch of a topological order is convex)
        if ((int)seg.size() > cfg.max_pattern_ops)
          for (int len : {cfg.max_pattern_ops, cfg.max_pattern_ops / 2})
            for (size_t at = 0; len >= 2 && at < seg.size(); at += (size_t)len)
              add(std::vector<int>(seg.begin() + at, seg.begin() + std::min(seg.size(), at + (size_t)len)), 0);
        // its connected parts as patterns of their own (what the generator takes when the
        // whole segment mixes shapes)
        std::map<int, int> comp;
        for (int o : seg) comp[o] = o;
        std::function<int(int)> find = [&](int v) { return comp[v] == v ? v : comp[v] = find(comp[v]); };
        std::set<int> inseg(seg.begin(), seg.end());
        for (int o : seg) for (int p : f.producers[o]) if (inseg.count(p)) comp[find(o)] = find(p);
        std::map<int, std::vector<int>> parts;
        for (int o : seg) parts[find(o)].push_back(o);
        if (parts.size() > 1) for (auto& kv : parts) add(kv.second, 1);
        // and the connected parts of its ops of one shape: the scalar arithmetic behind full
        // reductions, the elementwise ops of one tensor among several -- candidates where the
        // segment as a whole mixes shapes that no single kernel iterates over
        for (int o : seg) comp[o] = o;
        auto plain = [&](int v) { return !is_reduce_kind(g[v].kind) && g[v].kind != FS_DOT; };
        for (int o : seg) for (int p : f.producers[o])
          if (inseg.count(p) && plain(o) && plain(p) && g[o].same_shape(g[p])) comp[find(o)] = find(p);
        std::map<int, std::vector<int>> same;
        for (int o : seg) same[find(o)].push_back(o);
        if (same.size() > 1) {
          for (auto& kv : same) add(kv.second, 1);
          // such a part together with the row reductions that read it (elementwise -> reduce, the
          // input fusion of a reduction)
          for (auto& kv : same) {
            std::vector<int> ext = kv.second;
            for (int o : seg)
              if (row_reduce(g[o]) && find(o) != kv.first)
                for (int p : f.producers[o]) if (inseg.count(p) && find(p) == kv.first) { ext.push_back(o); break; }
            if (ext.size() > kv.second.size()) add(ext, 1);
            // and with the reductions that continue those over the next dim (chains over the
            // trailing dims, which a plan merges into one reduction)
            for (bool grown = ext.size() > kv.second.size(); grown;) {
              grown = false;
              const std::set<int> have(ext.begin(), ext.end());
              for (int o : seg)
                if (row_reduce(g[o]) && !have.count(o))
                  for (int p : f.producers[o]) if (have.count(p) && is_reduce_kind(g[p].kind) && g[p].kind == g[o].kind) { ext.push_back(o); grown = true; break; }
              if (grown) add(ext, 1);          // one more link of every chain
            }
          }
          // what is left of the segment without one such part: ops that only met through it (the
          // tensors that a shared scalar factor scales are independent parts of one kernel once the
          // factor is computed elsewhere)
          if (same.size() <= 64) for (auto& kv : same) {
            if (kv.second.size() < 2) continue;
            std::vector<int> rest;
            for (int o : seg) if (find(o) != kv.first) rest.push_back(o);
            add(rest, 1);
          }
        }
      }
      seg.clear();
    };
    for (int o : owned) {
      if (is_partition(g[o])) { flush(); continue; }
      seg.push_back(o);
    }
    flush();
  }

  // Model-based score of a set of ops: negative if it is not convex or no stitched plan can be
  // built for it (asked of fs_plan_create itself, which stops before compilation).  Remembered per set.
  std::map<std::vector<int>, std::pair<double, int64_t>> evaluated;
  std::map<std::vector<int>, FusionGroup> lists;       // the stand-alone op lists of the generable sets
  double evaluate(const std::vector<int>& ops, int64_t* saved = nullptr) {
    auto it = evaluated.find(ops);
    if (it == evaluated.end()) {
      std::pair<double, int64_t> r{-1.0, 0};
      if (fusion_is_convex(g, ops)) {
        FusionGroup gr;
        extract(all, g, f, ops, &gr);
        if (generable(gr)) {
          r.second = fusion_saved_bytes(g, ops);
          r.first = fusion_model_us(cfg, r.second) + (double)(ops.size() - 1) * cfg.launch_us;
          lists.emplace(ops, std::move(gr));
        }
      }
      it = evaluated.emplace(ops, r).first;
    }
    if (saved) *saved = it->second.second;
    return it->second.first;
  }

  // Algorithm 2: a seed grows by one producer or consumer at a time as long as the grown set is
  // still a valid pattern (convex, a stitched plan exists); every set on the way is a pattern.
  // Depth first, so the maximal patterns around a seed come early; every seed has its share of
  // the visit budget.
  int visited = 0, seed_limit = 0;
  std::set<std::vector<int>> explored;
  bool fusible(const Node& x) const {
    return is_binary(x.kind) || is_unary(x.kind) || x.kind == FS_CONVERT || x.kind == FS_CAUSAL_MASK ||
           is_reduce_kind(x.kind) || fine_dot(x);
  }
  void explore(const std::vector<int>& seed) {
    if (visited >= seed_limit || (int)seed.size() >= cfg.max_pattern_ops) return;
    std::set<int> in(seed.begin(), seed.end()), cand;
    for (int o : seed) {
      for (int p : f.producers[o]) if (!in.count(p) && fusion_owns_kernel(g, p) && fusible(g[p])) cand.insert(p);
      for (int c : f.consumers[o]) if (!in.count(c) && fusion_owns_kernel(g, c) && fusible(g[c])) cand.insert(c);
    }
    for (int c : cand) {
      std::vector<int> next = seed;
      next.push_back(c);
      std::sort(next.begin(), next.end());
      if (!explored.insert(next).second) continue;
      if (!fusion_is_convex(g, next)) continue;          // would introduce a cyclic dependence
      if (++visited > seed_limit) return;
      if (evaluate(next) < 0.0) continue;                // no kernel for it: nothing grows from here
      add(next, 2);
      explore(next);
    }
  }

  void generate() {
    // the multi-step heuristic: partition ops grow from large dots to every reduction
    substitution([&](const Node& x) { return x.kind == FS_DOT && !fine_dot(x); });
    substitution([&](const Node& x) { return x.kind == FS_DOT; });
    substitution([&](const Node& x) { return x.kind == FS_DOT || (is_reduce_kind(x.kind) && !row_reduce(x)); });
    substitution([&](const Node& x) { return x.kind == FS_DOT || is_reduce_kind(x.kind); });
    // exploratory seeds: fusible ops with large results and few operands (all ops here have at most two)
    std::vector<int> seeds;
    for (int o : owned) if (fusible(g[o]) && value_bytes(g[o]) >= cfg.seed_bytes) seeds.push_back(o);
    for (size_t k = 0; k < seeds.size() && visited < cfg.explore_budget; ++k) {
      const int share = std::max(24, (cfg.explore_budget - visited) / (int)(seeds.size() - k));
      seed_limit = std::min(cfg.explore_budget, visited + share);
      explore(std::vector<int>{seeds[k]});
    }
    for (const std::vector<int>& p : cfg.extra_patterns) add(p, 3);
  }

  // The hybrid policy of Section 4.3: the model's score for every pattern; where the caller ran a
  // pattern and reports the time it saves, that figure stands instead (also when it says the
  // fused kernel loses: a negative score keeps the pattern out of the selection).
  void score() {
    std::map<std::vector<int>, double> reported;
    for (size_t k = 0; k < cfg.extra_patterns.size() && k < cfg.extra_scores.size(); ++k) {
      if (std::isnan(cfg.extra_scores[k])) continue;
      std::vector<int> key = cfg.extra_patterns[k];
      std::sort(key.begin(), key.end());
      reported[key] = cfg.extra_scores[k];
    }
    for (FusionPattern& p : patterns) {
      p.score = evaluate(p.ops, &p.saved_bytes);
      auto li = lists.find(p.ops);
      if (li != lists.end()) { p.list = li->second.list; p.input_of = li->second.input_of; p.output_of = li->second.output_of; }
      auto it = reported.find(p.ops);
      if (p.score >= 0.0 && it != reported.end()) { p.score = it->second; p.measured = true; }
    }
  }
};

// maximise sum of scores over pairwise disjoint patterns, none of the forbidden sets complete
// Maximum-weight selection of pairwise compatible patterns by branch and bound over up to 256
// patterns (heaviest first).  Exact unless the node budget runs out, in which case the best
// selection found so far stands (the first descent is the greedy one).
struct Mask {
  uint64_t w[4] = {0, 0, 0, 0};
  void set(int i) { w[i >> 6] |= 1ull << (i & 63); }
  bool test(int i) const { return (w[i >> 6] >> (i & 63)) & 1; }
  Mask operator|(const Mask& o) const { Mask r; for (int k = 0; k < 4; ++k) r.w[k] = w[k] | o.w[k]; return r; }
  bool contains(const Mask& o) const { for (int k = 0; k < 4; ++k) if ((w[k] & o.w[k]) != o.w[k]) return false; return true; }
};

struct Solver {
  std::vector<double> w;
  std::vector<Mask> conflict;
  std::vector<Mask> forbidden;
  Mask best_sel;
  double best = -1.0;
  long long nodes = 0;
  static constexpr long long kNodeBudget = 4000000;
  void rec(int i, const Mask& sel, const Mask& blocked, double val, double rest) {
    if (val > best) { best = val; best_sel = sel; }
    if (i == (int)w.size() || val + rest <= best || ++nodes > kNodeBudget) return;
    const double rest_after = rest - w[i];
    if (!blocked.test(i)) {
      Mask s2 = sel;
      s2.set(i);
      bool ok = true;
      for (const Mask& fset : forbidden) if (s2.contains(fset)) ok = false;
      if (ok) rec(i + 1, s2, blocked | conflict[i], val + w[i], rest_after);
    }
    rec(i + 1, sel, blocked, val, rest_after);
  }
  Mask solve() {
    double rest = 0;
    for (double x : w) rest += x;
    best = -1.0; best_sel = Mask(); nodes = 0;
    rec(0, Mask(), Mask(), 0.0, rest);
    return best_sel;
  }
};

}  // namespace

bool fusion_plan(const std::vector<fs_op_desc>& ops, const FusionConfig& cfg, FusionResult* out, std::string* err) {
  Graph g;
  if (!build_graph(ops.data(), (int32_t)ops.size(), &g, err)) return false;
  for (const std::vector<int>& p : cfg.extra_patterns)
    for (int o : p) if (!fusion_owns_kernel(g, o)) { *err = "fusion plan: a supplied pattern names an op that owns no kernel"; return false; }
  Planner pl(ops, g, cfg);
  pl.generate();
  pl.score();
  // Candidates: the patterns with non-negative scores.  Patterns that share no op with each
  // other never constrain each other, so the selection problem splits along the connected
  // components of the conflict graph; each component is solved exactly over its best
  // max_patterns (at most 256) patterns.
  std::vector<int> cand;
  for (size_t k = 0; k < pl.patterns.size(); ++k) if (pl.patterns[k].score >= 0.0) cand.push_back((int)k);
  std::stable_sort(cand.begin(), cand.end(), [&](int a, int b) { return pl.patterns[a].score > pl.patterns[b].score; });
  const int cap = std::min(cfg.max_patterns, 256);
  const int m = (int)cand.size();
  std::vector<std::set<int>> sets(m);
  for (int a = 0; a < m; ++a) sets[a].insert(pl.patterns[cand[a]].ops.begin(), pl.patterns[cand[a]].ops.end());
  // component of each candidate: union-find over shared ops
  std::vector<int> comp(m);
  for (int a = 0; a < m; ++a) comp[a] = a;
  std::function<int(int)> find = [&](int v) { return comp[v] == v ? v : comp[v] = find(comp[v]); };
  {
    std::map<int, int> first_with_op;
    for (int a = 0; a < m; ++a)
      for (int o : sets[a]) {
        auto it = first_with_op.find(o);
        if (it == first_with_op.end()) first_with_op[o] = a;
        else comp[find(a)] = find(it->second);
      }
  }
  std::vector<std::vector<int>> forbidden_sets;      // cycle repairs: candidate numbers that may not all be chosen
  // chosen[a] for every candidate, solving component by component
  auto solve_all = [&]() {
    std::vector<char> chosen(m, 0);
    std::map<int, std::vector<int>> by_comp;
    for (int a = 0; a < m; ++a) by_comp[find(a)].push_back(a);      // candidates are sorted by score already
    for (auto& kv : by_comp) {
      std::vector<int> ids = kv.second;
      if ((int)ids.size() > cap) {
        // More candidates than the solver takes: first the patterns of substitution fusion (few, and
        // the search's variants of a large pattern must not crowd out a small disjoint one), then the
        // two heaviest patterns that contain each op (so that no op loses its best cover to a crowd
        // of variants elsewhere), then the heaviest of the rest.
        std::map<int, int> covers;
        std::vector<char> keep(ids.size(), 0);
        int kept = 0;
        for (size_t q = 0; q < ids.size() && kept < cap; ++q) {
          if (pl.patterns[cand[ids[q]]].origin == 2) continue;
          keep[q] = 1;
          ++kept;
          for (int o : sets[ids[q]]) ++covers[o];
        }
        for (size_t q = 0; q < ids.size() && kept < cap; ++q) {
          if (keep[q]) continue;
          bool wanted = false;
          for (int o : sets[ids[q]]) if (covers[o] < 2) wanted = true;
          if (!wanted) continue;
          keep[q] = 1;
          ++kept;
          for (int o : sets[ids[q]]) ++covers[o];
        }
        for (size_t q = 0; q < ids.size() && kept < cap; ++q) if (!keep[q]) { keep[q] = 1; ++kept; }
        std::vector<int> chosen_ids;
        for (size_t q = 0; q < ids.size(); ++q) if (keep[q]) chosen_ids.push_back(ids[q]);
        ids.swap(chosen_ids);
      }
      Solver sv;
      const int k = (int)ids.size();
      sv.w.resize(k);
      sv.conflict.assign(k, Mask());
      std::map<int, int> local;
      for (int i = 0; i < k; ++i) { sv.w[i] = pl.patterns[cand[ids[i]]].score; local[ids[i]] = i; }
      for (int i = 0; i < k; ++i)
        for (int j = 0; j < k; ++j) {
          if (i == j) continue;
          bool meet = false;
          for (int o : sets[ids[i]]) if (sets[ids[j]].count(o)) { meet = true; break; }
          if (meet) sv.conflict[i].set(j);
        }
      for (const std::vector<int>& fs_ : forbidden_sets) {
        Mask mask;
        bool inside = true;
        for (int a : fs_) { auto it = local.find(a); if (it == local.end()) { inside = false; break; } mask.set(it->second); }
        if (inside) sv.forbidden.push_back(mask);
      }
      const Mask sel = sv.solve();
      for (int i = 0; i < k; ++i) if (sel.test(i)) chosen[ids[i]] = 1;
    }
    return chosen;
  };
  Flow& f = pl.f;
  const int n = g.size();
  std::vector<int> group_of(n, -1);
  std::vector<std::vector<int>> members;
  out->solver_rounds = 0;
  for (int round = 0; round < 32; ++round) {
    ++out->solver_rounds;
    const std::vector<char> chosen = solve_all();
    // contract: chosen patterns, then every other owned op on its own
    members.clear();
    std::fill(group_of.begin(), group_of.end(), -1);
    std::vector<int> chosen_cand;
    for (int a = 0; a < m; ++a) if (chosen[a]) {
      for (int o : sets[a]) group_of[o] = (int)members.size();
      members.emplace_back(sets[a].begin(), sets[a].end());
      chosen_cand.push_back(a);
    }
    const int n_chosen = (int)members.size();
    for (int o : pl.owned) if (group_of[o] < 0) { group_of[o] = (int)members.size(); members.push_back({o}); }
    const int ng = (int)members.size();
    std::vector<std::set<int>> succ(ng);
    std::vector<int> indeg(ng, 0);
    for (int o : pl.owned) for (int c : f.consumers[o]) {
      if (!fusion_owns_kernel(g, c)) continue;
      const int a = group_of[o], b = group_of[c];
      if (a != b && succ[a].insert(b).second) ++indeg[b];
    }
    // Kahn, smallest first op first
    std::vector<int> order;
    std::set<std::pair<int, int>> ready;
    for (int k = 0; k < ng; ++k) if (indeg[k] == 0) ready.insert({members[k][0], k});
    while (!ready.empty()) {
      const int k = ready.begin()->second;
      ready.erase(ready.begin());
      order.push_back(k);
      for (int b : succ[k]) if (--indeg[b] == 0) ready.insert({members[b][0], b});
    }
    if ((int)order.size() == ng) {
      // acyclic: this is the plan
      out->groups.clear();
      out->total_score = 0.0;
      for (int k : order) {
        FusionGroup gr;
        extract(ops, g, f, members[k], &gr);
        gr.score = k < n_chosen ? pl.patterns[cand[chosen_cand[k]]].score : 0.0;
        out->total_score += gr.score;
        out->groups.push_back(gr);
      }
      for (int a : chosen_cand) pl.patterns[cand[a]].chosen = true;
      out->patterns = pl.patterns;
      return true;
    }
    // a cycle: the chosen patterns among the groups Kahn could not schedule and that lie on a
    // cycle are forbidden as a set (the additional constraint of the iterative process)
    std::vector<char> stuck(ng, 1);
    for (int k : order) stuck[k] = 0;
    // shrink to groups that are on a cycle: repeatedly drop stuck groups without a stuck successor
    bool changed = true;
    while (changed) {
      changed = false;
      for (int k = 0; k < ng; ++k) if (stuck[k]) {
        bool has = false;
        for (int b : succ[k]) if (stuck[b]) has = true;
        if (!has) { stuck[k] = 0; changed = true; }
      }
    }
    std::vector<int> fset;
    for (int k = 0; k < n_chosen; ++k) if (stuck[k]) fset.push_back(chosen_cand[k]);
    if (fset.empty()) { *err = "fusion plan: cycle without a fused pattern on it"; return false; }
    // the patterns of a forbidden set must be decided together from now on
    for (size_t k = 1; k < fset.size(); ++k) comp[find(fset[k])] = find(fset[0]);
    forbidden_sets.push_back(fset);
  }
  *err = "fusion plan: cycle repair did not converge";
  return false;
}

}  // namespace fs
