// Host entry points of the stitched schedules: each schedule has a `plan` step (pure
// host: geometry, LDS budget; no GPU call), a `describe` step and a `launch` step.
#pragma once
#include <string>
#include <vector>
#include "ew_ir.h"
#include "specs.h"

namespace fs {

struct RowLaunch { int variant = 0, K = 1, L = 64, U = 1, wg = 256, grid = 1; };
bool row_stitch_plan(const RowSpec&, const LaunchOpts&, RowLaunch*, std::string* err);
std::string row_stitch_describe(const RowSpec&, const RowLaunch&);
int row_stitch_launch(const RowSpec&, const RowLaunch&, const void* const* in, void* const* out,
                      void* stream, std::string* err);

// Wavefront-team form of the row schedule: a register-resident row spread over the
// wavefronts of one workgroup (2049..32768 elements).
struct RowTeamLaunch { int variant = 0, K = 1, wg = 128, grid = 1; };
bool row_team_plan(const RowSpec&, const LaunchOpts&, RowTeamLaunch*, std::string* err);
std::string row_team_describe(const RowSpec&, const RowTeamLaunch&);
int row_team_launch(const RowSpec&, const RowTeamLaunch&, const void* const* in, void* const* out,
                    void* stream, std::string* err);

// Block-composed form of the row schedule for long or unaligned rows (row cached in LDS).
struct RowBlockLaunch { int variant = 0, wg = 256, grid = 1; bool vector = true; int64_t lds_bytes = 0; };
bool row_block_plan(const RowSpec&, const LaunchOpts&, RowBlockLaunch*, int* status, std::string* err);
std::string row_block_describe(const RowSpec&, const RowBlockLaunch&);
int row_block_launch(const RowSpec&, const RowBlockLaunch&, const void* const* in, void* const* out,
                     void* stream, std::string* err);

// LayerNorm backward: row path for dx packed with the column path for dgamma/dbeta.
struct LnBwdLaunch { int K = 1, wg = 256, grid = 1, n_kernels = 1; int64_t lds_bytes = 0, workspace_bytes = 0; };
bool lnbwd_stitch_plan(const LnBwdSpec&, const LaunchOpts&, LnBwdLaunch*, std::string* err);
std::string lnbwd_stitch_describe(const LnBwdSpec&, const LnBwdLaunch&);
int lnbwd_stitch_launch(const LnBwdSpec&, const LnBwdLaunch&, const void* const* in, void* const* out,
                        void* workspace, void* stream, std::string* err);

// Batched dot -> softmax -> batched dot on MFMA.
struct AttnLaunch { int wg = 256, grid = 1, nq = 4, nk = 4; int64_t lds_bytes = 0; };   // nq, nk: 16-row tiles of queries (= wavefronts) and of keys
bool attn_stitch_plan(const AttnSpec&, const LaunchOpts&, AttnLaunch*, int* status, std::string* err);
std::string attn_stitch_describe(const AttnSpec&, const AttnLaunch&);
int attn_stitch_launch(const AttnSpec&, const AttnLaunch&, const void* const* in, void* const* out,
                       void* stream, std::string* err);

// Generic elementwise stitching (ew_stitch.hip, ew_codegen.cpp): the group either as a
// generated kernel or as a register program for the interpreter kernel.
struct Graph;
struct EwLaunch {
  int wg = 256, grid = 1, n_ops = 0;
  std::vector<int> view_param;        // parameter ordinal behind each operand view
  std::vector<char> view_full;        // generated form: the view has the group's own dense layout (read once, by the thread that writes the same elements)
  // generated form
  bool generated = false;
  int width = 4;                      // elements per thread
  int parts = 1;                      // independent groups packed into the launch (each on its own run of workgroups)
  int64_t n = 0;
  std::vector<char> code_object;
  std::string kernel_name;
  EwModule loaded;                    // run-time state: the module once it is on a device
  std::string note;                   // why generation was not used, if it was tried
  // interpreted form
  int U = 1, n_slots = 0, n_ins = 0;  // U: chunks a thread carries in lock step
  bool vector = true;
  int64_t lds_bytes = 0;
  std::vector<char> blob;             // the compiled program (plain data)
};
bool ew_stitch_plan(const Graph&, const LaunchOpts&, EwLaunch*, int* status, std::string* err);
std::string ew_stitch_describe(const EwLaunch&);
int ew_stitch_launch(EwLaunch&, const void* const* in, void* const* out, int n_out, void* stream,
                     std::string* err);
void ew_stitch_release(EwLaunch&);

int stream_copy_launch(void* dst, const void* src, int64_t bytes, void* stream, std::string* err);
// out[r][s][c] = sum over g of partial[r][s * groups + g][c] (doubles), stored in dtype[r]; r < n_red <= 8;
// s < n_seg runs of rows (1: sums over all rows)
int col_combine_launch(const void* partial, int groups, int64_t cols, int n_red, void* const* out, const int* dtype,
                       void* stream, std::string* err, int64_t n_seg = 1, const int* is_max = nullptr);   // is_max[r]: a maximum, not a sum

}  // namespace fs
