// Result of recognising a fusion group (see match.cpp).
#pragma once
#include <string>
#include <vector>
#include "graph.h"
#include "specs.h"

namespace fs {

enum MatchKind : int { MATCH_NONE = 0, MATCH_ROW = 1, MATCH_LNBWD = 2, MATCH_ATTN = 3 };

struct Match {
  int kind = MATCH_NONE;
  RowSpec row;
  LnBwdSpec lnbwd;
  AttnSpec attn;
  std::string why;   // reason when nothing matches
};

// An activation idiom inside a group: out = half*h*(1 + tanh(k0*(h + k1*h^3))) in any association
// and operand order, where nothing outside the idiom reads a value computed between h and out
// (`interior`).  The kernel generators compute it as 2*half*h / (1 + exp2(h*(a0 + a1*h*h))): one exp2 and
// one reciprocal, against eleven arithmetic ops and a tanh spelled out.
struct GeluIdiom { int out = -1, h = -1; double half = 0, k0 = 0, k1 = 0; std::vector<int> interior; };
std::vector<GeluIdiom> find_gelu_idioms(const Graph& g);
// half*h*(1 + tanh(w)) == 2*half*h / (1 + exp(-2w)) with w = k0*(h + k1*h^3): the constants of
// mul*h / (1 + exp2(h*(a0 + a1*h*h)))
inline void gelu_constants(const GeluIdiom& id, float out[3]) {
  const double log2e = 1.4426950408889634;
  out[0] = (float)(2.0 * id.half);
  out[1] = (float)(-2.0 * id.k0 * log2e);
  out[2] = (float)(-2.0 * id.k0 * id.k1 * log2e);
}

// True if a stitched schedule covers the group; fills the matching spec.
bool recognise(const Graph& g, Match* m);

}  // namespace fs
