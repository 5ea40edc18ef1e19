// Result of recognising a fusion group (see match.cpp).
#pragma once
#include <string>
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

// True if a stitched schedule covers the group; fills the matching spec.
bool recognise(const Graph& g, Match* m);

}  // namespace fs
