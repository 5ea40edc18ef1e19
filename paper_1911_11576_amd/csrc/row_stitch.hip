// Host side of schedule 1: geometry selection, template-notation description and launch
// (the kernel template lives in row_stitch_impl.h, instantiated per dtype).
#include "row_stitch_impl.h"

namespace fs {
namespace {

constexpr int kKs[] = {1, 2, 3, 4, 6, 8};

int pick_K(int nvec) {
  const int need = (nvec + 63) / 64;
  for (int k : kKs) if (k >= need) return k;
  return -1;
}

int pick_L(int nvec) {
  if (nvec >= 64) return 64;
  int L = 8;
  while (L < nvec) L *= 2;
  return L;
}

int max_U(int K, int V) { return K * V <= 8 ? 4 : K * V <= 16 ? 2 : 1; }

}  // namespace

bool row_stitch_plan(const RowSpec& sp, const LaunchOpts& opt, RowLaunch* out, std::string* err) {
  const int V = 16 / dtype_size(sp.dtype);
  if (sp.cols % V != 0) { *err = "row schedule: cols must be a multiple of the 16-byte vector width"; return false; }
  const int64_t nvec = sp.cols / V;
  // one wavefront holds a whole row in registers: at most 32 fp32 values per lane
  if (sp.cols > 2048) { *err = "row schedule: row longer than one wavefront's register tile (cols > 2048)"; return false; }
  if (sp.rows >= (int64_t)1 << 31) { *err = "row schedule: rows >= 2^31"; return false; }
  RowLaunch rl;
  rl.K = pick_K((int)nvec);
  rl.L = pick_L((int)nvec);
  rl.wg = opt.wg_size ? opt.wg_size : 256;
  if (rl.wg < 64 || rl.wg > 512 || rl.wg % 64) { *err = "row schedule: wg_size must be a multiple of 64 in [64,512]"; return false; }
  // default row groups in flight per wavefront: two while a lane holds at most 32 bytes of
  // a row, else one (measured: more only costs registers)
  const int kv = rl.K * V;
  int U = opt.rows_per_wave ? opt.rows_per_wave : (kv <= 8 ? 2 : 1);
  if (U < 1 || U > 8) { *err = "rows_per_wave out of range [1,8]"; return false; }
  const int mu = max_U(rl.K, V);
  rl.U = U >= 4 && mu >= 4 ? 4 : U >= 2 && mu >= 2 ? 2 : 1;
  const int G = 64 / rl.L;
  const int64_t n_groups = (sp.rows + G - 1) / G;
  const int64_t n_iters = (n_groups + rl.U - 1) / rl.U;
  const int waves = rl.wg / 64;
  int64_t grid = (n_iters + waves - 1) / waves;
  if (opt.grid > 0 && opt.grid < grid) grid = opt.grid;
  if (grid > 0x7fffffff) grid = 0x7fffffff;
  rl.grid = (int)grid;
  const bool mask_bcast = !(sp.mask_d1 == 1 && sp.mask_d2 == 1 && sp.mask_stride[0] == 1);
  rl.variant = sp.core == CORE_LAYERNORM ? (sp.gelu ? 1 : 0) : (sp.in_mask < 0 ? 2 : mask_bcast ? 4 : 3);
  *out = rl;
  return true;
}

std::string row_stitch_describe(const RowSpec& sp, const RowLaunch& rl) {
  // one schedule per reduction and per output, in the template notation of Section 5.2:
  // rows are tiled GRID then WARP (U row groups of 64/L rows per wavefront), columns are
  // WARP-parallel with K vectors per lane; nothing carries the S attribute
  char buf[512];
  const int G = 64 / rl.L;
  const char* r1 = sp.core == CORE_LAYERNORM ? "reduce_mean" : "reduce_max";
  const char* r2 = sp.core == CORE_LAYERNORM ? "reduce_var" : "reduce_sum";
  snprintf(buf, sizeof buf,
           "%s[GRID-WARP_%d,WARP]; %s[GRID-WARP_%d,WARP]; out[GRID-WARP_%d,WARP-THREAD_%d]; "
           "cta_num=%d, cta_size=%d",
           r1, rl.U * G, r2, rl.U * G, rl.U * G, rl.K * (16 / dtype_size(sp.dtype)), rl.grid, rl.wg);
  return buf;
}

void row_fill_args(const RowSpec& sp, const void* const* in, void* const* out, RowArgs* pa) {
  RowArgs& a = *pa;
  a.x = in[sp.in_x];
  a.res = sp.in_res >= 0 ? in[sp.in_res] : nullptr;
  a.bias = sp.in_bias >= 0 ? in[sp.in_bias] : nullptr;
  a.gamma = sp.in_gamma >= 0 ? in[sp.in_gamma] : nullptr;
  a.beta = sp.in_beta >= 0 ? in[sp.in_beta] : nullptr;
  a.mask = sp.in_mask >= 0 ? in[sp.in_mask] : nullptr;
  a.y = out[0];
  a.rows = sp.rows;
  a.cols = (int)sp.cols;
  a.nvec = (int)(sp.cols / (16 / dtype_size(sp.dtype)));
  a.scale = sp.scale; a.eps = sp.eps; a.inv_n = (float)(1.0 / (double)sp.cols);
  // c*h*(1 + tanh(k0*(h + k1*h^3))) == 2c*h / (1 + exp2(h*(a0 + a1*h^2))), a0 = -2*k0*log2(e)
  a.g_mul = 2.f * sp.gelu_half;
  a.g_a0 = (float)(-2.0 * (double)sp.gelu_k0 * 1.4426950408889634);
  a.g_a1 = (float)(-2.0 * (double)sp.gelu_k0 * 1.4426950408889634 * (double)sp.gelu_k1);
  a.mask_d1 = FastDiv::make((uint32_t)sp.mask_d1); a.mask_d2 = FastDiv::make((uint32_t)sp.mask_d2);
  a.ms0 = sp.mask_stride[0]; a.ms1 = sp.mask_stride[1]; a.ms2 = sp.mask_stride[2];
}

int row_stitch_launch(const RowSpec& sp, const RowLaunch& rl, const void* const* in, void* const* out,
                      void* stream, std::string* err) {
  if (sp.rows == 0 || sp.cols == 0) return 0;
  RowArgs a{};
  row_fill_args(sp, in, out, &a);
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e;
  switch (sp.dtype) {
    case DT_F32: e = row_launch_f32(a, rl, s); break;
    case DT_F16: e = row_launch_f16(a, rl, s); break;
    default: e = row_launch_bf16(a, rl, s); break;
  }
  if (e != hipSuccess) { *err = std::string("row_stitch launch: ") + hipGetErrorString(e); return -1; }
  return 0;
}

}  // namespace fs
