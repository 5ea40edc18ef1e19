// Host-side description of what the recogniser found in a fusion group and what a
// stitched kernel needs to run it.  Plain data passed from the matcher to the
// launchers; no GPU types.
#pragma once
#include <stdint.h>
#include <string>

namespace fs {

enum Dtype : int { DT_F32 = 0, DT_F16 = 1, DT_BF16 = 2 };
inline int dtype_size(int dt) { return dt == DT_F32 ? 4 : 2; }
inline const char* dtype_name(int dt) { return dt == DT_F32 ? "f32" : dt == DT_F16 ? "f16" : "bf16"; }

struct LaunchOpts {
  int wg_size = 0;
  int rows_per_wave = 0;
  int grid = 0;
  bool codegen = true;     // schedules that generate their kernel at run time may do so
};

// ---- schedule 1: elementwise prologue -> row reduce(s) -> broadcast -> epilogue ------
enum RowCore : int { CORE_LAYERNORM = 0, CORE_SOFTMAX = 1 };

struct RowSpec {
  int core = 0;
  int64_t rows = 0, cols = 0;
  int dtype = DT_F32;          // storage dtype of every parameter and of the output
  // parameter ordinals (index into fs_launch's inputs[]), -1 = absent
  int in_x = -1;               // main [rows, cols] operand (LayerNorm input / scores)
  int in_bias = -1;            // [cols], added before the GELU (prologue present if gelu)
  int in_res = -1;             // [rows, cols], added after the GELU
  int in_gamma = -1, in_beta = -1;   // [cols]
  int in_mask = -1;            // softmax additive mask
  bool gelu = false;           // r = c_half*h*(1 + tanh(k0*(h + k1*h^3))) with h = x (+ bias)
  float gelu_half = 0.5f, gelu_k0 = 0.f, gelu_k1 = 0.f;
  float eps = 0.f;             // LayerNorm
  float scale = 1.f;           // softmax: z = scale*x + mask
  // mask row = i0*ms[0] + i1*ms[1] + i2*ms[2] where (i0,i1,i2) are the leading indices of
  // the score row r = (i0*d1 + i1)*d2 + i2; a full mask has d1 = d2 = 1 and ms[0] = 1
  int64_t mask_d1 = 1, mask_d2 = 1;
  int64_t mask_stride[3] = {1, 0, 0};
};

// ---- schedule 1+2 packed: LayerNorm backward (row path for dx, column path for the
// parameter gradients over the same register-resident rows) -----------------------------
struct LnBwdSpec {
  int64_t rows = 0, cols = 0;
  int in_dy = -1, in_x = -1, in_gamma = -1, in_mean = -1, in_rstd = -1;
  int out_dx = -1, out_dgamma = -1, out_dbeta = -1;   // output ordinals, -1 = not produced
};

// ---- schedule 3: batched dot -> scale -> (+ mask) -> (causal mask) -> row softmax -> batched dot
// -> (x gate) -> (+ residual); optional second output: the log-sum-exp of every score row ----------
struct AttnSpec {
  int64_t batch = 0, sq = 0, sk = 0, dim = 0;   // query length, key length, head dim
  int dtype = DT_F16;          // storage dtype of q, k, v, gate, residual and o
  int in_q = -1, in_k = -1, in_v = -1;
  float scale = 1.f;
  bool causal = false;
  float fill = 0.f;            // value of masked scores (-inf allowed)
  int in_mask = -1;            // fp32 parameter added to the scaled scores, -1 = none; element (b, i, j) at
  int64_t mask_sb = 0, mask_sq = 0;   //   b * mask_sb + i * mask_sq + j  (0 strides: broadcast over batch / over query rows)
  int in_gate = -1, in_res = -1;      // [batch, sq, dim] parameters of the epilogue O * gate + res, -1 = absent
  int out_o = 0, out_lse = -1;        // output ordinals; lse [batch, sq] fp32
};

}  // namespace fs
