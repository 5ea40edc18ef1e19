// Schedule 3 (block composition around a fine-grained batched GEMM, paper Section 5.1):
//   S = Q K^T  ->  scale  ->  (causal mask)  ->  row softmax  ->  P (16-bit)  ->  O = P V
// as one kernel, one workgroup per batch element.  The two dots are the only dense
// contractions of the group and run on MFMA (v_mfma_f32_16x16x32 f16/bf16, fp32
// accumulate); everything between them is thread-composed on the accumulator registers,
// the row max/sum are 16-lane DPP all-reduces, and P is handed from the first dot's
// accumulator layout to the second dot's operand layout through LDS (the `S` attribute),
// as is V (transposed on the way in) and O (so the final store is 16 bytes per lane).
//
// Wavefront w owns query rows 16w..16w+15.  Operand fragments of Q and K are read from
// global memory directly in MFMA layout (lane (c,g) = (l%16, l/16) holds 8 consecutive
// k-values of row c starting at 8g: one 16-byte load).  With a causal mask of -inf,
// key tiles right of the diagonal contribute exactly zero and are skipped.
#include "dev_common.h"
#include "launchers.h"
#include "../../include/fs.h"

namespace fs {

struct AttnArgs {
  const void* q; const void* k; const void* v; void* o;
  int batch, seq, dim;
  float scale, fill;
  int causal, skip_masked_tiles;
};

template <typename T> struct Mfma;
template <> struct Mfma<f16_t> {
  static __device__ __forceinline__ f32x4 run(u32x4 a, u32x4 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
  }
  static __device__ __forceinline__ uint16_t cvt(float f) { return (uint16_t)f32_to_f16(f); }
};
template <> struct Mfma<bf16_t> {
  static __device__ __forceinline__ f32x4 run(u32x4 a, u32x4 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  }
  static __device__ __forceinline__ uint16_t cvt(float f) { return (uint16_t)f32_to_bf16(f); }
};

// NT: 16-row tiles along the sequence (workgroup = NT wavefronts); D: head dim
template <typename T, int NT, int D>
__global__ __launch_bounds__(64 * NT) void attn_stitch_kernel(const AttnArgs a) {
  constexpr int KS = D / 32;                 // k-steps of the first dot
  constexpr int NTP = NT < 2 ? 2 : NT;       // key tiles padded to whole 32-key steps
  constexpr int SP = NTP * 16 + 8;           // padded row length of Vt and P (halves)
  constexpr int DP = D + 8;                  // padded row length of the O staging tile
  constexpr int WROW = SP > DP ? SP : DP;
  extern __shared__ uint16_t smem[];
  uint16_t* vt = smem;                                   // [D][SP]   V transposed
  uint16_t* pw = smem + D * SP + (threadIdx.x >> 6) * 16 * WROW;   // [16][WROW] per wavefront
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int c = lane & 15, g = lane >> 4;
  const int b = blockIdx.x;
  const int seq = a.seq;
  const uint16_t* qb = static_cast<const uint16_t*>(a.q) + (int64_t)b * seq * D;
  const uint16_t* kb = static_cast<const uint16_t*>(a.k) + (int64_t)b * seq * D;
  const uint16_t* vb = static_cast<const uint16_t*>(a.v) + (int64_t)b * seq * D;
  uint16_t* ob = static_cast<uint16_t*>(a.o) + (int64_t)b * seq * D;
  const int q0 = 16 * w;
  const bool active = q0 < seq;
  // key tiles this wavefront needs: all that hold a valid key, cut at the diagonal when
  // masked scores are exactly -inf
  int tiles = (seq + 15) / 16;
  if (a.skip_masked_tiles && w + 1 < tiles) tiles = w + 1;

  // ---- stage V transposed into LDS (all wavefronts), zero-filling keys >= seq ----------
  constexpr int CH = D / 8;                  // 16-byte chunks per row
  for (int ci = threadIdx.x; ci < NTP * 16 * CH; ci += 64 * NT) {
    const int key = ci / CH, d0 = (ci % CH) * 8;
    u32x4 t = {0u, 0u, 0u, 0u};
    if (key < seq) t = *reinterpret_cast<const u32x4*>(vb + (int64_t)key * D + d0);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      vt[(d0 + 2 * j) * SP + key] = (uint16_t)(t[j] & 0xFFFFu);
      vt[(d0 + 2 * j + 1) * SP + key] = (uint16_t)(t[j] >> 16);
    }
  }

  f32x4 acc[NT];
  if (active) {
    // ---- first dot: S tile kt = Q(16 x D) . K_kt^T ---------------------------------------
    u32x4 qf[KS];
    const int qrow = min(q0 + c, seq - 1);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      qf[ks] = *reinterpret_cast<const u32x4*>(qb + (int64_t)qrow * D + ks * 32 + 8 * g);
#pragma unroll
    for (int kt = 0; kt < NT; ++kt) {
      acc[kt] = f32x4{0.f, 0.f, 0.f, 0.f};
      if (kt < tiles) {
        const int krow = min(kt * 16 + c, seq - 1);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          const u32x4 kf = *reinterpret_cast<const u32x4*>(kb + (int64_t)krow * D + ks * 32 + 8 * g);
          acc[kt] = Mfma<T>::run(qf[ks], kf, acc[kt]);
        }
      }
    }
    // ---- scale, mask, softmax on the accumulators: lane holds S[q0+4g+i][16kt+c] ----------
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int qi = q0 + 4 * g + i;
      float mx = -INFINITY;
#pragma unroll
      for (int kt = 0; kt < NT; ++kt) {
        const int key = kt * 16 + c;
        float z = acc[kt][i] * a.scale;
        if (a.causal && key > qi) z = a.fill;
        if (key >= seq || kt >= tiles) z = -INFINITY;
        acc[kt][i] = z;
        mx = fmaxf(mx, z);
      }
      mx = group_allreduce<MaxOp, 16>(mx);
      float s = 0.f;
#pragma unroll
      for (int kt = 0; kt < NT; ++kt) {
        const float e = __expf(acc[kt][i] - mx);
        acc[kt][i] = e;
        s += e;
      }
      s = group_allreduce<SumOp, 16>(s);
      const float inv = 1.f / s;
#pragma unroll
      for (int kt = 0; kt < NTP; ++kt) {
        const float p = kt < NT ? acc[kt < NT ? kt : 0][i] * inv : 0.f;
        pw[(4 * g + i) * WROW + kt * 16 + c] = Mfma<T>::cvt(p);   // P rounded to the dot's dtype
      }
    }
  }
  __syncthreads();   // Vt complete; P of this wavefront visible to all its lanes

  if (active) {
    // ---- second dot: O(16 x D) = P(16 x keys) . V -----------------------------------------
    f32x4 o[D / 16];
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt) o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    const int ksteps = (tiles + 1) / 2;
#pragma unroll
    for (int kk = 0; kk < NTP / 2; ++kk) {
      if (kk < ksteps) {
        const u32x4 pa = *reinterpret_cast<const u32x4*>(pw + c * WROW + kk * 32 + 8 * g);
#pragma unroll
        for (int dt = 0; dt < D / 16; ++dt) {
          const u32x4 vf = *reinterpret_cast<const u32x4*>(vt + (dt * 16 + c) * SP + kk * 32 + 8 * g);
          o[dt] = Mfma<T>::run(pa, vf, o[dt]);
        }
      }
    }
    // ---- O through the wavefront's LDS tile so that each lane stores 16 bytes ---------------
    // (every lane's reads of P above are complete before the tile is overwritten: LDS
    // operations of one wavefront execute in order)
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt)
#pragma unroll
      for (int i = 0; i < 4; ++i) pw[(4 * g + i) * WROW + dt * 16 + c] = Mfma<T>::cvt(o[dt][i]);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int ci = lane; ci < 16 * CH; ci += 64) {
      const int r = ci / CH, d0 = (ci % CH) * 8;
      if (q0 + r < seq)
        *reinterpret_cast<u32x4*>(ob + (int64_t)(q0 + r) * D + d0) =
            *reinterpret_cast<const u32x4*>(pw + r * WROW + d0);
    }
  }
}

namespace {

int64_t attn_lds_bytes(int NT, int D) {
  const int NTP = NT < 2 ? 2 : NT;
  const int SP = NTP * 16 + 8, DP = D + 8, WROW = SP > DP ? SP : DP;
  return 2 * ((int64_t)D * SP + (int64_t)NT * 16 * WROW);
}

template <typename T, int NT, int D>
hipError_t launch_one(const AttnArgs& a, hipStream_t s) {
  hipLaunchKernelGGL((attn_stitch_kernel<T, NT, D>), dim3(a.batch), dim3(64 * NT),
                     (size_t)attn_lds_bytes(NT, D), s, a);
  return hipGetLastError();
}

template <typename T, int NT>
hipError_t launch_D(const AttnArgs& a, hipStream_t s) {
  switch (a.dim) {
    case 32: return launch_one<T, NT, 32>(a, s);
    case 64: return launch_one<T, NT, 64>(a, s);
    default: return launch_one<T, NT, 128>(a, s);
  }
}

template <typename T>
hipError_t launch_NT(const AttnArgs& a, int nt, hipStream_t s) {
  switch (nt) {
    case 1: return launch_D<T, 1>(a, s);
    case 2: return launch_D<T, 2>(a, s);
    case 4: return launch_D<T, 4>(a, s);
    default: return launch_D<T, 8>(a, s);
  }
}

}  // namespace

// LDS budget per workgroup: the volume constraint of shared-memory planning.  64 KB of the
// 160 KB a CU has keeps at least two workgroups resident.
static constexpr int64_t kLdsBudget = 64 * 1024;

bool attn_stitch_plan(const AttnSpec& sp, const LaunchOpts& opt, AttnLaunch* out, int* status, std::string* err) {
  *status = FS_ERR_UNSUPPORTED;
  if (sp.dim != 32 && sp.dim != 64 && sp.dim != 128) { *err = "attention schedule: head dim must be 32, 64 or 128"; return false; }
  if (sp.seq > 128) { *err = "attention schedule: fine-grained dots only (sequence <= 128)"; return false; }
  if (sp.batch > 0x7fffffff) { *err = "attention schedule: batch too large"; return false; }
  AttnLaunch l;
  const int need = (int)((sp.seq + 15) / 16);
  l.tiles = need <= 1 ? 1 : need <= 2 ? 2 : need <= 4 ? 4 : 8;
  l.wg = 64 * l.tiles;
  if (opt.wg_size && opt.wg_size != l.wg) { *err = "attention schedule: wg_size is fixed at 64 per 16 query rows"; *status = FS_ERR_INVALID; return false; }
  l.grid = (int)sp.batch;
  l.lds_bytes = attn_lds_bytes(l.tiles, (int)sp.dim);
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
  char buf[512];
  snprintf(buf, sizeof buf,
           "dot_1[GRID,WARP_16,CTA]; softmax[GRID,WARP_16,WARP]S; dot_2[GRID,WARP_16,CTA]S; "
           "cta_num=%d, cta_size=%d, lds=%lld",
           l.grid, l.wg, (long long)l.lds_bytes);
  (void)sp;
  return buf;
}

int attn_stitch_launch(const AttnSpec& sp, const AttnLaunch& l, const void* const* in, void* const* out,
                       void* stream, std::string* err) {
  if (sp.batch == 0 || sp.seq == 0) return 0;
  AttnArgs a{};
  a.q = in[sp.in_q]; a.k = in[sp.in_k]; a.v = in[sp.in_v]; a.o = out[0];
  a.batch = (int)sp.batch; a.seq = (int)sp.seq; a.dim = (int)sp.dim;
  a.scale = sp.scale; a.fill = sp.fill; a.causal = sp.causal ? 1 : 0;
  a.skip_masked_tiles = sp.causal && sp.fill == -INFINITY;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const hipError_t e = sp.dtype == DT_F16 ? launch_NT<f16_t>(a, l.tiles, s) : launch_NT<bf16_t>(a, l.tiles, s);
  if (e != hipSuccess) { *err = std::string("attn_stitch launch: ") + hipGetErrorString(e); return -1; }
  return 0;
}

}  // namespace fs
