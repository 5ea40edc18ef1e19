// Schedule 3 (block composition around a fine-grained batched GEMM, paper Section 5.1; the
// dot -> elementwise -> reduce -> dot shape with several outputs of the motivating example,
// Section 3.1):
//   S = Q K^T -> scale -> (+ additive mask or bias) -> (causal mask) -> row softmax -> P (16-bit)
//     -> O = P V -> (x gate) -> (+ residual) -> store;   optional second output: log-sum-exp per row
// as one kernel, one workgroup per batch element.  The two dots are the only dense
// contractions of the group and run on MFMA (v_mfma_f32_16x16x32 f16/bf16, fp32
// accumulate); everything around them is thread-composed on the accumulator registers.
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
// O^T leaves the accumulators as four consecutive head-dim values per lane and tile (where the
// epilogue operands are read, 8 bytes each); one row swap between lane pairs makes that eight, so
// the final store is 16 bytes per lane.
//
// Operand fragments of Q and K are read from global memory directly in MFMA layout (8
// consecutive k-values of row c starting at 8g: one 16-byte load).  With a causal mask of -inf,
// key tiles right of the diagonal contribute exactly zero and are skipped.  Query and key
// lengths are independent (each up to 128).
#pragma once
#include "dev_common.h"
#include "launchers.h"
#include "../../include/fs.h"

namespace fs {

struct AttnArgs {
  const void* q; const void* k; const void* v; void* o;
  const float* mask;            // additive, fp32: element (b, i, j) at mask[b*mask_sb + i*mask_sq + j]; NULL = none
  const void* gate;             // [B, Sq, D] in the dot dtype, multiplies O; NULL = none
  const void* res;              // [B, Sq, D] in the dot dtype, added after the gate; NULL = none
  float* lse;                   // [B, Sq] fp32: max + log(sum) of every score row; NULL = not produced
  int64_t mask_sb, mask_sq;
  int batch, sq, sk, dim;
  float scale, fill;
  int causal, skip_masked_tiles, mask_vec;   // mask_vec: four mask values of a lane are one aligned 16-byte load
};

template <typename T> struct Mfma;
template <> struct Mfma<f16_t> {
  static __device__ __forceinline__ f32x4 run(u32x4 a, u32x4 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
  }
  static __device__ __forceinline__ uint32_t pack(float lo, float hi) { return pack2_f16(lo, hi); }
  static __device__ __forceinline__ float lo(uint32_t w) { return f16_to_f32(w & 0xFFFFu); }
  static __device__ __forceinline__ float hi(uint32_t w) { return f16_to_f32(w >> 16); }
};
template <> struct Mfma<bf16_t> {
  static __device__ __forceinline__ f32x4 run(u32x4 a, u32x4 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  }
  static __device__ __forceinline__ uint32_t pack(float lo, float hi) { return pack2_bf16(lo, hi); }
  static __device__ __forceinline__ float lo(uint32_t w) { return as_f32(w << 16); }
  static __device__ __forceinline__ float hi(uint32_t w) { return as_f32(w & 0xFFFF0000u); }
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

// NQ: 16-row tiles of queries (workgroup = NQ wavefronts); NK: 16-key tiles; D: head dim;
// X: the group has a mask, an epilogue operand or a second output (without any of them those paths
// are compiled out: on the bare dot-softmax-dot group their run-time tests alone cost 0.15 us of 6)
template <typename T, int NQ, int NK, int D, bool X>
__global__ __launch_bounds__(64 * NQ) void attn_stitch_kernel(const AttnArgs a) {
  constexpr int KS = D / 32;                 // k-steps of the first dot
  constexpr int NKP = NK < 2 ? 2 : NK;       // key tiles padded to whole 32-key steps
  constexpr int SP = NKP * 16 + 8;           // padded row length of Vt (halves)
  constexpr int SWM = (2 * NKP < 8 ? 2 * NKP : 8) - 1;   // granules of a row that the swizzle permutes
  extern __shared__ uint16_t smem[];
  uint16_t* vt = smem;                       // [D][SP]   V transposed, keys in k-slot order
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int c = lane & 15, g = lane >> 4;
  const int b = blockIdx.x;
  const int sq = a.sq, sk = a.sk;
  const uint16_t* qb = static_cast<const uint16_t*>(a.q) + (int64_t)b * sq * D;
  const uint16_t* kb = static_cast<const uint16_t*>(a.k) + (int64_t)b * sk * D;
  const uint16_t* vb = static_cast<const uint16_t*>(a.v) + (int64_t)b * sk * D;
  uint16_t* ob = static_cast<uint16_t*>(a.o) + (int64_t)b * sq * D;
  const int q0 = 16 * w;
  const bool active = q0 < sq;
  const int qi = q0 + c;                     // the lane's query row
  const int qrow = min(qi, sq - 1);
  // key tiles this wavefront needs: all that hold a valid key, cut at the diagonal when
  // masked scores are exactly -inf
  int tiles = (sk + 15) / 16;
  if (a.skip_masked_tiles && w + 1 < tiles) tiles = w + 1;

  // ---- every global load of the wavefront is issued before the first use: Q, all K tiles, its
  // share of V (for the LDS transpose), the mask values of its scores and the epilogue operands.
  // Loads behind run-time conditions would each wait out a full memory latency in turn; rows
  // beyond the lengths are clamped to the last row and masked later.
  constexpr int CH = D / 8;                  // 16-byte chunks per row
  constexpr int VTOT = NKP * 16 * CH;        // chunks of the (padded) V tile
  constexpr int NV = (VTOT + 64 * NQ - 1) / (64 * NQ);
  u32x4 qf[KS], kf[NK][KS], vreg[NV];
  f32x4 mk[NK];
  u32x2 gt[D / 16], rs[D / 16];
  {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      qf[ks] = *reinterpret_cast<const u32x4*>(qb + (int64_t)qrow * D + ks * 32 + 8 * g);
#pragma unroll
    for (int kt = 0; kt < NK; ++kt) {
      const int krow = min(kt * 16 + c, sk - 1);
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        if (kt < tiles) kf[kt][ks] = *reinterpret_cast<const u32x4*>(kb + (int64_t)krow * D + ks * 32 + 8 * g);   // same for the whole wavefront
      }
    }
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int ci = min((int)threadIdx.x + i * 64 * NQ, VTOT - 1);
      const int key = min(ci / CH, sk - 1), d0 = (ci % CH) * 8;
      vreg[i] = *reinterpret_cast<const u32x4*>(vb + (int64_t)key * D + d0);
    }
    if (X && a.mask) {
      const float* mrow = a.mask + (int64_t)b * a.mask_sb + (int64_t)qrow * a.mask_sq;
#pragma unroll
      for (int kt = 0; kt < NK; ++kt) {
        const int key0 = kt * 16 + 4 * g;
        mk[kt] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (kt < tiles) {
          if (a.mask_vec) {
            if (key0 < sk) mk[kt] = *reinterpret_cast<const f32x4*>(mrow + key0);
          } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) if (key0 + i < sk) mk[kt][i] = mrow[key0 + i];
          }
        }
      }
    }
    if (X && a.gate) {
      const uint16_t* p = static_cast<const uint16_t*>(a.gate) + ((int64_t)b * sq + qrow) * D + 4 * g;
#pragma unroll
      for (int dt = 0; dt < D / 16; ++dt) gt[dt] = *reinterpret_cast<const u32x2*>(p + dt * 16);
    }
    if (X && a.res) {
      const uint16_t* p = static_cast<const uint16_t*>(a.res) + ((int64_t)b * sq + qrow) * D + 4 * g;
#pragma unroll
      for (int dt = 0; dt < D / 16; ++dt) rs[dt] = *reinterpret_cast<const u32x2*>(p + dt * 16);
    }
  }

  u32x4 pb[NKP / 2];                         // P^T, the second dot's B fragments
  if (active) {
    // ---- first dot, transposed: tile kt = K_kt(16 x D) . Q^T -----------------------------
    f32x4 acc[NK];
#pragma unroll
    for (int kt = 0; kt < NK; ++kt) {
      acc[kt] = f32x4{0.f, 0.f, 0.f, 0.f};
      if (kt < tiles) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) acc[kt] = Mfma<T>::run(kf[kt][ks], qf[ks], acc[kt]);
      }
    }
    // ---- scale, mask, softmax of query row q0+c: the lane holds S[q0+c][16kt+4g+i] ---------
    float mx = -INFINITY;
#pragma unroll
    for (int kt = 0; kt < NK; ++kt)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int key = kt * 16 + 4 * g + i;
        float z = acc[kt][i] * a.scale;
        if (X && a.mask) z += mk[kt][i];
        if (a.causal && key > qi) z = a.fill;
        if (key >= sk || kt >= tiles) z = -INFINITY;
        acc[kt][i] = z;
        mx = fmaxf(mx, z);
      }
    mx = rows_allreduce<MaxOp>(mx);
    float sum = 0.f;
#pragma unroll
    for (int kt = 0; kt < NK; ++kt)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float e = __expf(acc[kt][i] - mx);
        acc[kt][i] = e;
        sum += e;
      }
    sum = rows_allreduce<SumOp>(sum);
    const float inv = 1.f / sum;
    if (X && a.lse && g == 0 && qi < sq) a.lse[(int64_t)b * sq + qi] = mx + logf(sum);
    // P rounded to the dot's dtype, packed in k-slot order: slots 4h+i of step kk <- tile 2kk+h
#pragma unroll
    for (int kk = 0; kk < NKP / 2; ++kk)
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int kt = 2 * kk + h;
        float p[4] = {0.f, 0.f, 0.f, 0.f};
        if (kt < NK) {
#pragma unroll
          for (int i = 0; i < 4; ++i) p[i] = acc[kt < NK ? kt : 0][i] * inv;
        }
        pb[kk][2 * h] = Mfma<T>::pack(p[0], p[1]);
        pb[kk][2 * h + 1] = Mfma<T>::pack(p[2], p[3]);
      }
  }
  // ---- V transposed into LDS (all wavefronts), zero-filling keys >= sk; key 32kk+16h+4g+i of
  // a 32-key step sits at slot 8g+4h+i.  Two things keep the stores off each other's banks: the
  // lanes of keys 2n and 2n+1 first trade half of their eight values, so that each stores whole
  // 32-bit words (both keys of one row) instead of 16-bit halves, and the 16-byte granule of a
  // slot is xor-ed with the row's group of eight (row / 8), which spreads the eight row groups a
  // store instruction touches over all banks. ------------------------------------------------
  uint32_t* vt32 = reinterpret_cast<uint32_t*>(smem);
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int cu = (int)threadIdx.x + i * 64 * NQ;       // chunks beyond the tile exist only where the workgroup has more
    const int ci = min(cu, VTOT - 1);                    // lanes than the tile has chunks: they take part in the exchange, not in the store
    const int key = ci / CH, dg = ci % CH, d0 = dg * 8;
    const int slot = ((key & ~31) | ((key & 12) << 1) | ((key & 16) >> 2) | (key & 3)) ^ ((dg & SWM) << 3);
    const u32x4 t = key < sk ? vreg[i] : u32x4{0u, 0u, 0u, 0u};
    const bool odd = (key & 1) != 0;
    // the even key's lane ends up with rows d0 .. d0+3 of both keys, the odd key's with d0+4 .. d0+7
    const uint32_t rx = pair_exchange<CH>(odd ? t[0] : t[2]), ry = pair_exchange<CH>(odd ? t[1] : t[3]);
    const uint32_t ex = odd ? rx : t[0], ey = odd ? ry : t[1];     // the even key's two value pairs
    const uint32_t ox = odd ? t[2] : rx, oy = odd ? t[3] : ry;     // the odd key's
    if (cu < VTOT) {
      uint32_t* w0 = vt32 + (((d0 + (odd ? 4 : 0)) * SP + (slot & ~1)) >> 1);
      w0[0 * (SP / 2)] = (ex & 0xFFFFu) | (ox << 16);
      w0[1 * (SP / 2)] = (ex >> 16) | (ox & 0xFFFF0000u);
      w0[2 * (SP / 2)] = (ey & 0xFFFFu) | (oy << 16);
      w0[3 * (SP / 2)] = (ey >> 16) | (oy & 0xFFFF0000u);
    }
  }
  __syncthreads();   // Vt complete

  if (active) {
    // ---- second dot, transposed: O^T(D x 16) = V^T(D x keys) . P^T ---------------------------
    f32x4 o[D / 16];
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt) o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    const int ksteps = (tiles + 1) / 2;
#pragma unroll
    for (int kk = 0; kk < NKP / 2; ++kk) {
      if (kk < ksteps) {
#pragma unroll
        for (int dt = 0; dt < D / 16; ++dt) {
          const int sw = (2 * dt + (c >> 3)) & SWM;          // the row's granule swizzle, as stored
          const u32x4 vf = *reinterpret_cast<const u32x4*>(vt + (dt * 16 + c) * SP + 8 * ((kk * 4 + g) ^ sw));
          o[dt] = Mfma<T>::run(vf, pb[kk], o[dt]);
        }
      }
    }
    // ---- epilogue on the accumulators: the lane holds O[q0+c][16dt+4g+i], i < 4 -----------------
    if (X && a.gate) {
#pragma unroll
      for (int dt = 0; dt < D / 16; ++dt) {
        o[dt][0] *= Mfma<T>::lo(gt[dt][0]); o[dt][1] *= Mfma<T>::hi(gt[dt][0]);
        o[dt][2] *= Mfma<T>::lo(gt[dt][1]); o[dt][3] *= Mfma<T>::hi(gt[dt][1]);
      }
    }
    if (X && a.res) {
#pragma unroll
      for (int dt = 0; dt < D / 16; ++dt) {
        o[dt][0] += Mfma<T>::lo(rs[dt][0]); o[dt][1] += Mfma<T>::hi(rs[dt][0]);
        o[dt][2] += Mfma<T>::lo(rs[dt][1]); o[dt][3] += Mfma<T>::hi(rs[dt][1]);
      }
    }
    // ---- 8 bytes per tile.  Lanes g and g^1 trade
    // one tile of a pair (dt, dt+1) so that each ends up with 8 consecutive values, 16 bytes: after
    // the row swap lane g holds d = 32(dt/2) + 16(g&1) + 8(g>>1) .. +7 ------------------------
    uint16_t* orow = ob + (int64_t)qrow * D + 16 * (g & 1) + 8 * (g >> 1);
#pragma unroll
    for (int dp = 0; dp < D / 32; ++dp) {
      const uint32_t a0 = Mfma<T>::pack(o[2 * dp][0], o[2 * dp][1]), a1 = Mfma<T>::pack(o[2 * dp][2], o[2 * dp][3]);
      const uint32_t b0 = Mfma<T>::pack(o[2 * dp + 1][0], o[2 * dp + 1][1]), b1 = Mfma<T>::pack(o[2 * dp + 1][2], o[2 * dp + 1][3]);
      // odd rows of the first operand trade places with even rows of the second
      const auto r0 = __builtin_amdgcn_permlane16_swap(a0, b0, false, false);
      const auto r1 = __builtin_amdgcn_permlane16_swap(a1, b1, false, false);
      if (qi < sq) *reinterpret_cast<u32x4*>(orow + dp * 32) = u32x4{r0[0], r1[0], r0[1], r1[1]};
    }
  }
}

inline int64_t attn_lds_bytes(int NK, int D) {
  const int NKP = NK < 2 ? 2 : NK;
  const int SP = NKP * 16 + 8;
  return 2 * (int64_t)D * SP;
}

template <typename T, int NQ, int NK, int D>
hipError_t attn_launch_one(const AttnArgs& a, hipStream_t s) {
  const bool extras = a.mask || a.gate || a.res || a.lse;
  if (extras) hipLaunchKernelGGL((attn_stitch_kernel<T, NQ, NK, D, true>), dim3(a.batch), dim3(64 * NQ), (size_t)attn_lds_bytes(NK, D), s, a);
  else hipLaunchKernelGGL((attn_stitch_kernel<T, NQ, NK, D, false>), dim3(a.batch), dim3(64 * NQ), (size_t)attn_lds_bytes(NK, D), s, a);
  return hipGetLastError();
}

template <typename T, int NQ, int NK>
hipError_t attn_launch_D(const AttnArgs& a, hipStream_t s) {
  switch (a.dim) {
    case 32: return attn_launch_one<T, NQ, NK, 32>(a, s);
    case 64: return attn_launch_one<T, NQ, NK, 64>(a, s);
    default: return attn_launch_one<T, NQ, NK, 128>(a, s);
  }
}

template <typename T, int NQ>
hipError_t attn_launch_NK(const AttnArgs& a, int nk, hipStream_t s) {
  switch (nk) {
    case 1: return attn_launch_D<T, NQ, 1>(a, s);
    case 2: return attn_launch_D<T, NQ, 2>(a, s);
    case 4: return attn_launch_D<T, NQ, 4>(a, s);
    default: return attn_launch_D<T, NQ, 8>(a, s);
  }
}

template <typename T>
hipError_t attn_launch_dtype(const AttnArgs& a, int nq, int nk, hipStream_t s) {
  switch (nq) {
    case 1: return attn_launch_NK<T, 1>(a, nk, s);
    case 2: return attn_launch_NK<T, 2>(a, nk, s);
    case 4: return attn_launch_NK<T, 4>(a, nk, s);
    default: return attn_launch_NK<T, 8>(a, nk, s);
  }
}

hipError_t attn_launch_f16(const AttnArgs& a, int nq, int nk, hipStream_t s);
hipError_t attn_launch_bf16(const AttnArgs& a, int nq, int nk, hipStream_t s);

}  // namespace fs
