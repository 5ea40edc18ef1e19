// Host side of schedule 3: geometry, LDS budget, template-notation description and launch (the kernel
// template lives in attn_stitch_impl.h, instantiated per dtype).
#include "attn_stitch_impl.h"

namespace fs {

// LDS budget per workgroup: the volume constraint of shared-memory planning.  72 KB of the
// 160 KB a CU has keeps two workgroups resident (the largest case, 128 keys of 128 values, needs 69 632).
static constexpr int64_t kLdsBudget = 72 * 1024;

static int pow2_tiles(int64_t len) {
  const int need = (int)((len + 15) / 16);
  return need <= 1 ? 1 : need <= 2 ? 2 : need <= 4 ? 4 : 8;
}

bool attn_stitch_plan(const AttnSpec& sp, const LaunchOpts& opt, AttnLaunch* out, int* status, std::string* err) {
  *status = FS_ERR_UNSUPPORTED;
  if (sp.dim != 32 && sp.dim != 64 && sp.dim != 128) { *err = "attention schedule: head dim must be 32, 64 or 128"; return false; }
  if (sp.sq > 128 || sp.sk > 128) { *err = "attention schedule: fine-grained dots only (query and key lengths <= 128)"; return false; }
  if (sp.sk == 0 && sp.sq > 0 && sp.batch > 0) { *err = "attention schedule: softmax over zero keys"; return false; }
  if (sp.batch > 0x7fffffff) { *err = "attention schedule: batch too large"; return false; }
  AttnLaunch l;
  l.nq = pow2_tiles(sp.sq);
  l.nk = pow2_tiles(sp.sk);
  l.wg = 64 * l.nq;
  if (opt.wg_size && opt.wg_size != l.wg) { *err = "attention schedule: wg_size is fixed at 64 per 16 query rows"; *status = FS_ERR_INVALID; return false; }
  l.grid = (int)sp.batch;
  l.lds_bytes = attn_lds_bytes(l.nk, (int)sp.dim);
  if (l.lds_bytes > kLdsBudget) {
    char buf[160];
    snprintf(buf, sizeof buf, "attention schedule: needs %lld bytes of LDS per workgroup, budget is %lld",
             (long long)l.lds_bytes, (long long)kLdsBudget);
    *err = buf;
    *status = FS_ERR_LDS;
    return false;
  }
  *out = l;
  *status = FS_OK;
  return true;
}

std::string attn_stitch_describe(const AttnSpec& sp, const AttnLaunch& l) {
  char buf[640];
  snprintf(buf, sizeof buf,
           "dot_1[GRID,WARP_16,CTA]; %ssoftmax[GRID,WARP_16,WARP]; %sdot_2[GRID,WARP_16,CTA]S; %s%s"
           "cta_num=%d, cta_size=%d, lds=%lld",
           sp.in_mask >= 0 ? "add_mask[GRID,WARP_16,WARP-THREAD_4]; " : "",
           sp.out_lse >= 0 ? "logsumexp[GRID,WARP_16,WARP]; " : "",
           sp.in_gate >= 0 ? "multiply_gate[GRID,WARP_16,CTA-THREAD_4]; " : "",
           sp.in_res >= 0 ? "add_residual[GRID,WARP_16,CTA-THREAD_4]; " : "",
           l.grid, l.wg, (long long)l.lds_bytes);
  return buf;
}

int attn_stitch_launch(const AttnSpec& sp, const AttnLaunch& l, const void* const* in, void* const* out,
                       void* stream, std::string* err) {
  if (sp.batch == 0 || sp.sq == 0) return 0;
  AttnArgs a{};
  a.q = in[sp.in_q]; a.k = in[sp.in_k]; a.v = in[sp.in_v]; a.o = out[sp.out_o];
  a.mask = sp.in_mask >= 0 ? static_cast<const float*>(in[sp.in_mask]) : nullptr;
  a.mask_sb = sp.mask_sb; a.mask_sq = sp.mask_sq;
  a.mask_vec = (sp.sk % 4 == 0 && sp.mask_sb % 4 == 0 && sp.mask_sq % 4 == 0) ? 1 : 0;
  a.gate = sp.in_gate >= 0 ? in[sp.in_gate] : nullptr;
  a.res = sp.in_res >= 0 ? in[sp.in_res] : nullptr;
  a.lse = sp.out_lse >= 0 ? static_cast<float*>(out[sp.out_lse]) : nullptr;
  a.batch = (int)sp.batch; a.sq = (int)sp.sq; a.sk = (int)sp.sk; a.dim = (int)sp.dim;
  a.scale = sp.scale; a.fill = sp.fill; a.causal = sp.causal ? 1 : 0;
  a.skip_masked_tiles = sp.causal && sp.fill == -INFINITY;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const hipError_t e = sp.dtype == DT_F16 ? attn_launch_f16(a, l.nq, l.nk, s) : attn_launch_bf16(a, l.nq, l.nk, s);
  if (e != hipSuccess) { *err = std::string("attn_stitch launch: ") + hipGetErrorString(e); return -1; }
  return 0;
}

}  // namespace fs
