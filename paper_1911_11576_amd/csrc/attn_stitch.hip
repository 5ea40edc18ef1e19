// Schedule 3 (block composition around a fine-grained batched GEMM, paper Section 5.1):
//   S = Q K^T  ->  scale  ->  (causal mask)  ->  row softmax  ->  P (16-bit)  ->  O = P V
// as one kernel, one workgroup per batch element.  The two dots are the only dense
// contractions of the group and run on MFMA (v_mfma_f32_16x16x32 f16/bf16, fp32
// accumulate); everything between them is thread-composed on the accumulator registers.
//
// Wavefront w owns query rows 16w..16w+15 and computes the scores TRANSPOSED: tile kt is
// K_kt (16 keys x D) . Q^T, so lane (c,g) = (l%16, l/16) holds S[q0+c][16kt+4g+i], i < 4 - every
// score a lane holds belongs to ONE query row.  The softmax is then a register reduction plus two
// cross-row steps (lanes c, c+16, c+32, c+48), and the normalised probabilities already sit in the
// second dot's B-operand layout: O^T = V^T . P^T contracts over keys, and the order of the keys
// inside a 32-key step is free as long as both operands use the same one, so k-slot 8g+4h+i of
// step kk is key 32kk+16h+4g+i - the scores of tiles 2kk and 2kk+1 that lane g holds.  P never
// leaves the registers.  V is the only operand that goes through LDS (the `S` attribute):
// transposed on the way in, keys stored in that slot order, read back as 16-byte A fragments.
// O^T leaves the accumulators as four consecutive head-dim values per lane and tile; one row swap
// between lane pairs makes that eight, so the final store is 16 bytes per lane.
//
// Operand fragments of Q and K are read from global memory directly in MFMA layout (8
// consecutive k-values of row c starting at 8g: one 16-byte load).  With a causal mask of -inf,
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
  static __device__ __forceinline__ uint32_t pack(float lo, float hi) { return pack2_f16(lo, hi); }
};
template <> struct Mfma<bf16_t> {
  static __device__ __forceinline__ f32x4 run(u32x4 a, u32x4 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  }
  static __device__ __forceinline__ uint32_t pack(float lo, float hi) { return pack2_bf16(lo, hi); }
};

// the value of lanes c, c+16, c+32, c+48 combined, in all four
template <class Op> __device__ __forceinline__ float rows_allreduce(float v) {
  uint32_t u = __builtin_bit_cast(uint32_t, v);
  auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  v = Op::apply(as_f32(r[0]), as_f32(r[1]));
  u = __builtin_bit_cast(uint32_t, v);
  r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return Op::apply(as_f32(r[0]), as_f32(r[1]));
}

// the value of the lane whose index differs in bit log2(CH): the lane that holds the other key of a
// pair when CH lanes share one key (CH = 16-byte chunks per row of V)
template <int CH> __device__ __forceinline__ uint32_t pair_exchange(uint32_t x) {
  if constexpr (CH == 8) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x128, 0xF, 0xF, false);   // row_ror:8
  } else {
    return (uint32_t)__builtin_amdgcn_ds_bpermute((int)(((threadIdx.x & 63) ^ CH) << 2), (int)x);
  }
}

// NT: 16-row tiles along the sequence (workgroup = NT wavefronts); D: head dim
template <typename T, int NT, int D>
__global__ __launch_bounds__(64 * NT) void attn_stitch_kernel(const AttnArgs a) {
  constexpr int KS = D / 32;                 // k-steps of the first dot
  constexpr int NTP = NT < 2 ? 2 : NT;       // key tiles padded to whole 32-key steps
  constexpr int SP = NTP * 16 + 8;           // padded row length of Vt (halves)
  constexpr int SWM = (2 * NTP < 8 ? 2 * NTP : 8) - 1;   // granules of a row that the swizzle permutes
  extern __shared__ uint16_t smem[];
  uint16_t* vt = smem;                       // [D][SP]   V transposed, keys in k-slot order
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

  // ---- every global load of the wavefront is issued before the first use: Q, all K tiles, then its
  // share of V (for the LDS transpose).  Loads behind run-time conditions would each wait out a
  // full memory latency in turn; rows beyond seq are clamped to the last row and masked later.
  constexpr int CH = D / 8;                  // 16-byte chunks per row
  constexpr int NV = NTP * 16 * CH / (64 * NT);
  static_assert(NV * 64 * NT == NTP * 16 * CH, "V chunks divide evenly over the workgroup");
  u32x4 qf[KS], kf[NT][KS], vreg[NV];
  {
    const int qrow = min(q0 + c, seq - 1);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      qf[ks] = *reinterpret_cast<const u32x4*>(qb + (int64_t)qrow * D + ks * 32 + 8 * g);
#pragma unroll
    for (int kt = 0; kt < NT; ++kt) {
      const int krow = min(kt * 16 + c, seq - 1);
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        if (kt < tiles) kf[kt][ks] = *reinterpret_cast<const u32x4*>(kb + (int64_t)krow * D + ks * 32 + 8 * g);   // same for the whole wavefront
      }
    }
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int ci = threadIdx.x + i * 64 * NT;
      const int key = min(ci / CH, seq - 1), d0 = (ci % CH) * 8;
      vreg[i] = *reinterpret_cast<const u32x4*>(vb + (int64_t)key * D + d0);
    }
  }

  u32x4 pb[NTP / 2];                         // P^T, the second dot's B fragments
  if (active) {
    // ---- first dot, transposed: tile kt = K_kt(16 x D) . Q^T -----------------------------
    f32x4 acc[NT];
#pragma unroll
    for (int kt = 0; kt < NT; ++kt) {
      acc[kt] = f32x4{0.f, 0.f, 0.f, 0.f};
      if (kt < tiles) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) acc[kt] = Mfma<T>::run(kf[kt][ks], qf[ks], acc[kt]);
      }
    }
    // ---- scale, mask, softmax of query row q0+c: the lane holds S[q0+c][16kt+4g+i] ---------
    const int qi = q0 + c;
    float mx = -INFINITY;
#pragma unroll
    for (int kt = 0; kt < NT; ++kt)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int key = kt * 16 + 4 * g + i;
        float z = acc[kt][i] * a.scale;
        if (a.causal && key > qi) z = a.fill;
        if (key >= seq || kt >= tiles) z = -INFINITY;
        acc[kt][i] = z;
        mx = fmaxf(mx, z);
      }
    mx = rows_allreduce<MaxOp>(mx);
    float sum = 0.f;
#pragma unroll
    for (int kt = 0; kt < NT; ++kt)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float e = __expf(acc[kt][i] - mx);
        acc[kt][i] = e;
        sum += e;
      }
    sum = rows_allreduce<SumOp>(sum);
    const float inv = 1.f / sum;
    // P rounded to the dot's dtype, packed in k-slot order: slots 4h+i of step kk <- tile 2kk+h
#pragma unroll
    for (int kk = 0; kk < NTP / 2; ++kk)
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int kt = 2 * kk + h;
        float p[4] = {0.f, 0.f, 0.f, 0.f};
        if (kt < NT) {
#pragma unroll
          for (int i = 0; i < 4; ++i) p[i] = acc[kt < NT ? kt : 0][i] * inv;
        }
        pb[kk][2 * h] = Mfma<T>::pack(p[0], p[1]);
        pb[kk][2 * h + 1] = Mfma<T>::pack(p[2], p[3]);
      }
  }
  // ---- V transposed into LDS (all wavefronts), zero-filling keys >= seq; key 32kk+16h+4g+i of
  // a 32-key step sits at slot 8g+4h+i.  Two things keep the stores off each other's banks: the
  // lanes of keys 2n and 2n+1 first trade half of their eight values, so that each stores whole
  // 32-bit words (both keys of one row) instead of 16-bit halves, and the 16-byte granule of a
  // slot is xor-ed with the row's group of eight (row / 8), which spreads the eight row groups a
  // store instruction touches over all banks.  (Stored piecewise the kernel spent as many cycles
  // in bank conflicts as in everything else the LDS did, by the counters.) ---------------------
  uint32_t* vt32 = reinterpret_cast<uint32_t*>(smem);
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int ci = threadIdx.x + i * 64 * NT;
    const int key = ci / CH, dg = ci % CH, d0 = dg * 8;
    const int slot = ((key & ~31) | ((key & 12) << 1) | ((key & 16) >> 2) | (key & 3)) ^ ((dg & SWM) << 3);
    const u32x4 t = key < seq ? vreg[i] : u32x4{0u, 0u, 0u, 0u};
    const bool odd = (key & 1) != 0;
    // the even key's lane ends up with rows d0 .. d0+3 of both keys, the odd key's with d0+4 .. d0+7
    const uint32_t rx = pair_exchange<CH>(odd ? t[0] : t[2]), ry = pair_exchange<CH>(odd ? t[1] : t[3]);
    const uint32_t ex = odd ? rx : t[0], ey = odd ? ry : t[1];     // the even key's two value pairs
    const uint32_t ox = odd ? t[2] : rx, oy = odd ? t[3] : ry;     // the odd key's
    uint32_t* w0 = vt32 + (((d0 + (odd ? 4 : 0)) * SP + (slot & ~1)) >> 1);
    w0[0 * (SP / 2)] = (ex & 0xFFFFu) | (ox << 16);
    w0[1 * (SP / 2)] = (ex >> 16) | (ox & 0xFFFF0000u);
    w0[2 * (SP / 2)] = (ey & 0xFFFFu) | (oy << 16);
    w0[3 * (SP / 2)] = (ey >> 16) | (oy & 0xFFFF0000u);
  }
  __syncthreads();   // Vt complete

  if (active) {
    // ---- second dot, transposed: O^T(D x 16) = V^T(D x keys) . P^T ---------------------------
    f32x4 o[D / 16];
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt) o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    const int ksteps = (tiles + 1) / 2;
#pragma unroll
    for (int kk = 0; kk < NTP / 2; ++kk) {
      if (kk < ksteps) {
#pragma unroll
        for (int dt = 0; dt < D / 16; ++dt) {
          const int sw = (2 * dt + (c >> 3)) & SWM;          // the row's granule swizzle, as stored
          const u32x4 vf = *reinterpret_cast<const u32x4*>(vt + (dt * 16 + c) * SP + 8 * ((kk * 4 + g) ^ sw));
          o[dt] = Mfma<T>::run(vf, pb[kk], o[dt]);
        }
      }
    }
    // ---- the lane holds O[q0+c][16dt+4g+i], i < 4: 8 bytes per tile.  Lanes g and g^1 trade
    // one tile of a pair (dt, dt+1) so that each ends up with 8 consecutive values, 16 bytes: after
    // the row swap lane g holds d = 32(dt/2) + 16(g&1) + 8(g>>1) .. +7 ------------------------
    uint16_t* orow = ob + (int64_t)min(q0 + c, seq - 1) * D + 16 * (g & 1) + 8 * (g >> 1);
#pragma unroll
    for (int dp = 0; dp < D / 32; ++dp) {
      const uint32_t a0 = Mfma<T>::pack(o[2 * dp][0], o[2 * dp][1]), a1 = Mfma<T>::pack(o[2 * dp][2], o[2 * dp][3]);
      const uint32_t b0 = Mfma<T>::pack(o[2 * dp + 1][0], o[2 * dp + 1][1]), b1 = Mfma<T>::pack(o[2 * dp + 1][2], o[2 * dp + 1][3]);
      // odd rows of the first operand trade places with even rows of the second
      const auto r0 = __builtin_amdgcn_permlane16_swap(a0, b0, false, false);
      const auto r1 = __builtin_amdgcn_permlane16_swap(a1, b1, false, false);
      if (q0 + c < seq) *reinterpret_cast<u32x4*>(orow + dp * 32) = u32x4{r0[0], r1[0], r0[1], r1[1]};
    }
  }
}

namespace {

int64_t attn_lds_bytes(int NT, int D) {
  const int NTP = NT < 2 ? 2 : NT;
  const int SP = NTP * 16 + 8;
  return 2 * (int64_t)D * SP;
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
           "dot_1[GRID,WARP_16,CTA]; softmax[GRID,WARP_16,WARP]; dot_2[GRID,WARP_16,CTA]S; "
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
