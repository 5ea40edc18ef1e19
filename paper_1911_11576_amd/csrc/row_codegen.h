// Generated form of the row schedule (warp composition, paper Section 5.1, emitted as code,
// Section 5.3): any group of elementwise ops and reductions over the last dim, in any
// order and depth, with column reductions and small dots packed in; rows in the registers of
// 1 to 1024 lanes, or streamed through LDS.  See row_codegen.cpp.
#pragma once
#include <stdint.h>
#include <string>
#include <vector>
#include "ew_ir.h"
#include "graph.h"
#include "specs.h"

namespace fs {

struct RowGenLaunch {
  int wg = 256, grid = 1;
  int L = 64, K = 1, W = 4;           // lanes per row, chunks per lane, elements per chunk
  int n_ops = 0, n_reduce = 0;
  bool streamed = false;              // one workgroup walks the row in passes
  bool persistent = false;            // a fixed grid loops over register-resident rows
  int passes = 1, row_buffers = 0, buffers_shared = 0;
  bool inputs_cached = true;
  // column reductions: one double-precision partial row per workgroup in the plan's workspace,
  // then a second kernel adds them
  int n_col = 0;
  int col_out[8] = {0}, col_dtype[8] = {0}, col_is_max[8] = {0};   // output ordinal, dtype and operator of each
  // column sums per run of consecutive rows ([B, S, H] summed over S): number of runs (0: sums over all
  // rows) and workgroups per run; with one workgroup per run the kernel stores the results itself
  bool segmented = false, seg_per_wave = false;
  int64_t seg_count = 0;
  int seg_groups = 0;
  int n_kernels = 1;
  // block composition around dots on the matrix unit: one workgroup per batch element
  bool mma = false;
  int mma_dots = 0, mma_k = 0, mma_d = 0;   // dots on MFMA (1 or 2), contraction of the first, result width of the second
  int64_t workspace_bytes = 0;
  int64_t rows = 0, cols = 0, lds_bytes = 0;
  std::vector<int> view_param;        // parameter ordinal behind each operand view
  std::vector<char> view_dense;       // the view is the parameter as a dense tensor of the group's full shape
  bool rows_read_before_written = false;   // register templates without dots: a row is read completely, by the lanes that write it, before any of it is written
  std::vector<char> code_object;
  std::string kernel_name;
  EwModule loaded;                    // run-time state: the module once it is on a device
};
bool row_gen_plan(const Graph&, const LaunchOpts&, RowGenLaunch*, int* status, std::string* err);
std::string row_gen_describe(const RowGenLaunch&);
int row_gen_launch(RowGenLaunch&, const void* const* in, void* const* out, int n_out, void* workspace,
                   void* stream, std::string* err);
void row_gen_release(RowGenLaunch&);

}  // namespace fs
