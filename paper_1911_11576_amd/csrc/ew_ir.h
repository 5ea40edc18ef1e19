// An all-elementwise fusion group after analysis: the ops that compute something, in list
// order, with their operands resolved to earlier ops, parameter views (broadcasts folded
// into strides) or constants.  Written by the analysis in ew_stitch.hip; read by the
// register-program compiler there and by the kernel generator (ew_codegen.cpp).
#pragma once
#include <stdint.h>
#include <string>
#include <vector>
#include "../../include/fs.h"

namespace fs {

enum EwOperandKind : int { EW_FROM_NODE = 0, EW_FROM_VIEW = 1, EW_FROM_CONST = 2 };
// beside the fs_opkind values; EW_OP_COPY stands for a rounding whose only reader is the store of
// the same dtype, which rounds the same way
// EW_OP_GELU_TANH is the tanh-form GELU found as an idiom (see match.h), one operand and three constants
enum EwExtraOp : int { EW_OP_ROUND_F16 = 100, EW_OP_ROUND_BF16 = 101, EW_OP_COPY = 102, EW_OP_GELU_TANH = 103 };

struct EwIrOperand {
  int kind = EW_FROM_NODE;
  int index = -1;          // EW_FROM_NODE: id of the producing node; EW_FROM_VIEW: view number
  float cval = 0.f;        // EW_FROM_CONST
};
struct EwIrNode {
  int id = -1;             // op index in the group (names the value)
  int op = 0;              // fs_opkind of an elementwise op, or an EwExtraOp
  int n_operands = 1;
  EwIrOperand opnd[2];
  float gelu[3] = {0.f, 0.f, 0.f};   // EW_OP_GELU_TANH: mul, a0, a1 of mul*h / (1 + exp2(h*(a0 + a1*h*h)))
  int out_ordinal = -1;    // >= 0: the value is this group output ...
  int out_dtype = FS_F32;  // ... stored in this dtype
};
struct EwIrView {
  int param = -1;          // parameter ordinal
  int dtype = FS_F32;      // its storage dtype
  bool full = true;        // same dense layout as the group's shape
  int64_t stride[FS_MAX_RANK] = {0, 0, 0, 0};   // element strides along the (right-aligned) dims
};
struct EwIr {
  std::vector<EwIrNode> nodes;
  std::vector<EwIrView> views;
  int64_t shape[FS_MAX_RANK] = {1, 1, 1, 1};    // right-aligned: leading extents 1
  int rank = 0;
  int64_t n = 0;
  int n_outputs = 0;
};

// ---- kernel generation (Section 5: the stitched op is emitted as code, compiled, cached) ----

// HIP source of one kernel computing the whole group; pure text, no GPU or compiler involved.
std::string ew_emit_source(const EwIr& ir, int* width, int* unroll, std::string* kernel_name);
// Several independent groups (each with its own shape) as one kernel: group q owns a run of
// blocks[q] consecutive workgroups of `wg` threads, its views start after those of the groups
// before it in Args::in, its outputs keep their ordinals of the whole list.
std::string ew_emit_packed(const std::vector<const EwIr*>& parts, int wg, std::vector<int>* widths, std::vector<int>* blocks,
                           std::string* kernel_name);
// Compile with the run-time compiler (works on a machine without a GPU).  Results are cached
// per process by source text.  False + message if the compiler is unavailable or fails.
bool ew_compile_source(const std::string& source, std::vector<char>* code_object, std::string* err);
// While on (per thread), ew_compile_source succeeds without compiling: plans made then can be
// inspected but not launched.  Used by the fusion planner to ask "can this group be generated".
void codegen_set_dry_run(bool on);
// Code objects on disk (directory from FS_KERNEL_CACHE_DIR unless set here; NULL or "" turns it off),
// the per-process cache emptied (the files stay), and how often a kernel was compiled, found in
// memory, found on disk.
void codegen_cache_dir(const char* dir);
void codegen_cache_drop_memory();
void codegen_cache_stats(int64_t* compiled, int64_t* from_memory, int64_t* from_disk);

// A loaded kernel (module handle and function), bound to the device current at load time.
struct EwModule {
  void* module = nullptr;
  void* function = nullptr;
  int device = -1;
};
int ew_module_launch(EwModule* m, const std::vector<char>& code_object, const std::string& kernel_name,
                     const void* args, size_t args_bytes, int grid, int block, void* stream, std::string* err);
void ew_module_release(EwModule* m);

}  // namespace fs
