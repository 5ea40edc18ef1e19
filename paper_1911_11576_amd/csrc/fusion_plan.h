// Fusion planning (paper Section 4): choose disjoint fusion patterns of a computation graph.
// Pure host code.
#pragma once
#include <stdint.h>
#include <string>
#include <utility>
#include <vector>
#include "graph.h"

namespace fs {

struct FusionConfig {
  double launch_us = 2.5;                 // phi: average launch latency of one kernel
  int max_patterns = 256;                 // patterns per conflict component handed to the solver (the best by score)
  int explore_budget = 400;               // patterns the exploratory search may visit
  int max_pattern_ops = 128;
  int64_t seed_bytes = 1 << 20;           // exploratory seeds: ops whose result is at least this large
  std::vector<std::pair<int64_t, double>> bandwidth;   // M(V) model: (bytes, GB/s), increasing bytes
  std::vector<std::vector<int>> extra_patterns;        // caller-supplied candidates
  std::vector<double> extra_scores;                    // per supplied candidate: its measured f(P) in microseconds,
                                                       // NaN (or no entry): the model's score
};

struct FusionPattern {
  std::vector<int> ops;                   // owned ops (op indices of the graph), increasing
  int origin = 0;                         // 0 substitution, 1 a connected part of a substitution segment, 2 exploratory, 3 caller
  int64_t saved_bytes = 0;                // V
  double score = -1.0;                    // f(P) in microseconds; negative: cannot be generated, or measured to lose
  bool measured = false;                  // the score is the caller's measurement, not the model's
  bool chosen = false;
  // the pattern as a stand-alone op list (filled for patterns a stitched plan exists for)
  std::vector<fs_op_desc> list;
  std::vector<int> input_of, output_of;
};

struct FusionGroup {
  std::vector<int> ops;                   // owned ops, increasing
  double score = 0.0;                     // 0 for an op left alone
  // the group as a stand-alone op list for plan creation
  std::vector<fs_op_desc> list;
  std::vector<int> input_of;              // per parameter of `list`: the op of the graph whose value it is
  std::vector<int> output_of;             // per output of `list`: the op of the graph whose value it is
};

struct FusionResult {
  std::vector<FusionPattern> patterns;    // every candidate that was scored
  std::vector<FusionGroup> groups;        // the plan, in an order that respects data flow
  double total_score = 0.0;
  int solver_rounds = 1;                  // 1 + number of cycle repairs
};

// true if the op owns a kernel when nothing is fused (constants, broadcasts, parameters and
// outputs do not)
bool fusion_owns_kernel(const Graph& g, int op);
// Fusing `ops` leaves the graph acyclic: no path leaves the set and comes back.
bool fusion_is_convex(const Graph& g, const std::vector<int>& ops);
// V: bytes of off-chip traffic the fused pattern saves against one kernel per op.
int64_t fusion_saved_bytes(const Graph& g, const std::vector<int>& ops);
// M(V) in microseconds from the bandwidth model.
double fusion_model_us(const FusionConfig& cfg, int64_t bytes);

bool fusion_plan(const std::vector<fs_op_desc>& ops, const FusionConfig& cfg, FusionResult* out, std::string* err);

}  // namespace fs
