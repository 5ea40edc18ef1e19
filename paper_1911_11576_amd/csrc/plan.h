// The plan object behind the C ABI's opaque fs_plan, and the two steps every launch entry point shares.
#pragma once
#include <string>

#include "../../include/fs.h"
#include "graph.h"
#include "launchers.h"
#include "match.h"
#include "per_op.h"
#include "row_codegen.h"

struct fs_plan {
  fs::Graph graph;
  int mode = FS_MODE_STITCHED;
  int schedule = FS_SCHED_PER_OP;
  fs::Match match;
  fs::RowLaunch row;
  fs::RowTeamLaunch row_team;
  fs::RowBlockLaunch row_block;
  fs::RowGenLaunch row_gen;
  int row_form = 0;   // 0 one wavefront per row group, 1 wavefront team, 2 row cached in LDS, 3 generated kernel
  fs::LnBwdLaunch lnbwd;
  fs::AttnLaunch attn;
  fs::EwLaunch ew;
  fs::PerOpPlan per_op;
  int n_kernels = 1;
  int64_t lds_bytes = 0, workspace_bytes = 0, moved_bytes = 0;
  void* workspace = nullptr;
  int device = -1;
  std::string description;
};

namespace fs {

// status + message of the calling thread (what fs_last_error returns)
fs_status set_error(fs_status st, const std::string& msg);
// Arguments of a launch checked against the plan: counts, NULL and alignment, identical pointers.
fs_status check_launch_args(fs_plan* p, const void* const* inputs, int32_t n_in, void* const* outputs, int32_t n_out);
// The plan's kernels enqueued with `workspace` as their scratch memory.
fs_status enqueue_plan(fs_plan* p, const void* const* inputs, void* const* outputs, int32_t n_out, void* workspace,
                       void* hip_stream);

}  // namespace fs
