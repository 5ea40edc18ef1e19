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
// leaves the registers.  V goes through LDS as stored (row-major, 16-byte stores) and comes back
// transposed: the transposing LDS read of gfx950 (ds_read_b64_tr_b16) hands lane c of a 16-lane
// group column c of a 4 x 16 tile whose four rows the group's lanes address in fours, which is the
// A fragment of four consecutive keys at head-dim 16dt + c; two reads make the eight k-slots.
// O^T leaves the accumulators as four consecutive head-dim values per lane and tile (where the
// epilogue operands are read, 8 bytes each); one row swap between lane pairs makes that eight, so
// the final store is 16 bytes per lane.
//
// Operand fragments of Q are read from global memory directly in MFMA layout (8 consecutive
// k-values of row c starting at 8g: one 16-byte load).  K is read the same way, every 16-key tile
// by ONE wavefront, and handed to the others through LDS (row-major, rows padded by 16 bytes so
// that eight lanes' 16-byte accesses fall on different banks): every wavefront loading every tile
// it needs keeps the texture path busy with the same lines up to four times over, which costs 0.4 us
// of 5 on 512 x 64 x 64 x 64.  With a causal mask of -inf, key tiles right of the diagonal contribute
// exactly zero and are skipped.  Query and key lengths are independent (each up to 128).
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

template <int N> struct TileCount { static constexpr int value = N; };   // a compile-time count handed to a generic lambda

// NQ: 16-row tiles of queries (workgroup = NQ wavefronts); NK: 16-key tiles; D: head dim;
// X: the group has a mask, an epilogue operand or a second output (without any of them those paths
// are compiled out: on the bare dot-softmax-dot group their run-time tests alone cost 0.15 us of 6);
// E: the lengths are exactly 16 NQ queries and 16 NK keys (NK >= 2), so no row is clamped and no key
// or query is tested against a length.
// With two wavefronts per SIMD and a memory phase of one round trip, the kernel's time follows its
// instruction count: everything that is the same for a whole wavefront (its first query row, the
// number of key tiles it needs, whether a tile touches the causal diagonal or the end of the keys)
// is kept in scalar registers and decided by scalar branches, and only tiles that a mask can touch
// pay for the comparisons.
template <typename T, int NQ, int NK, int D, bool X, bool E>
__global__ __launch_bounds__(64 * NQ) void attn_stitch_kernel(const AttnArgs a) {
  constexpr int KS = D / 32;                 // k-steps of the first dot
  constexpr int NKP = NK < 2 ? 2 : NK;       // key tiles padded to whole 32-key steps
  constexpr int VP = D + (D == 64 ? 8 : 16); // padded row length of V in LDS (halves): the four rows of a
                                             // transposing read fall on different banks
  constexpr int KP = D + 8;                  // padded row length of K in LDS (halves)
  constexpr int KT = (NK + NQ - 1) / NQ;     // key tiles a wavefront loads for the workgroup
  extern __shared__ uint16_t smem[];
  uint16_t* ksh = smem;                      // [NK * 16][KP]  K as stored
  uint16_t* vsh = smem + NK * 16 * KP;       // [NKP * 16][VP]  V as stored, keys beyond the last zero
  const int lane = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));    // the same in the whole wavefront
  const int c = lane & 15, g = lane >> 4;
  const int b = blockIdx.x;
  const int sq = E ? 16 * NQ : a.sq, sk = E ? 16 * NK : a.sk;
  const uint16_t* qb = static_cast<const uint16_t*>(a.q) + (int64_t)b * sq * D;
  const uint16_t* kb = static_cast<const uint16_t*>(a.k) + (int64_t)b * sk * D;
  const uint16_t* vb = static_cast<const uint16_t*>(a.v) + (int64_t)b * sk * D;
  uint16_t* ob = static_cast<uint16_t*>(a.o) + (int64_t)b * sq * D;
  const int q0 = 16 * w;
  const bool active = E || q0 < sq;
  const int qi = q0 + c;                     // the lane's query row
  const int qrow = E ? qi : min(qi, sq - 1);
  // key tiles this wavefront needs: all that hold a valid key, cut at the diagonal when
  // masked scores are exactly -inf
  int tiles = (sk + 15) / 16;
  int wg_tiles = tiles;                      // ... and the workgroup as a whole
  if (a.skip_masked_tiles && NQ < wg_tiles) wg_tiles = NQ;
  if (a.skip_masked_tiles && w + 1 < tiles) tiles = w + 1;

  // ---- every global load of the wavefront is issued before the first use: Q, its share of K and
  // of V (for LDS), the mask values of its scores and the epilogue operands.
  // Loads behind run-time conditions would each wait out a full memory latency in turn; rows
  // beyond the lengths are clamped to the last row and masked later.
  constexpr int CH = D / 8;                  // 16-byte chunks per row
  constexpr int VTOT = NKP * 16 * CH;        // chunks of the (padded) V tile
  constexpr int NV = (VTOT + 64 * NQ - 1) / (64 * NQ);
  constexpr bool VFULL = VTOT % (64 * NQ) == 0;   // every lane has a chunk in every round
  u32x4 qf[KS], kf[KT][KS], vreg[NV];
  f32x4 mk[NK];
  u32x2 gt[D / 16], rs[D / 16];
  {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      qf[ks] = *reinterpret_cast<const u32x4*>(qb + (int64_t)qrow * D + ks * 32 + 8 * g);
#pragma unroll
    for (int j = 0; j < KT; ++j) {
      const int kt = w + j * NQ;               // the same for the whole wavefront
      const int krow = E ? kt * 16 + c : min(kt * 16 + c, sk - 1);
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        if (kt < wg_tiles) kf[j][ks] = *reinterpret_cast<const u32x4*>(kb + (int64_t)krow * D + ks * 32 + 8 * g);
      }
    }
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int ci = VFULL ? (int)threadIdx.x + i * 64 * NQ : min((int)threadIdx.x + i * 64 * NQ, VTOT - 1);
      const int key = E ? ci / CH : min(ci / CH, sk - 1), d0 = (ci % CH) * 8;
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
  // the loads stay here: left alone, the compiler moves some down to their use, behind the wait for
  // others - a second memory round trip.  (The empty statement claims to read and write memory.)
  asm volatile("" ::: "memory");

  // ---- K into LDS as loaded ------------------------------------------------------------------
#pragma unroll
  for (int j = 0; j < KT; ++j) {
    const int kt = w + j * NQ;
    if (kt < wg_tiles) {
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) *reinterpret_cast<u32x4*>(ksh + (kt * 16 + c) * KP + ks * 32 + 8 * g) = kf[j][ks];
    }
  }
  // ---- V into LDS as loaded (all wavefronts), zero-filling keys >= sk ---------------------------
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int cu = (int)threadIdx.x + i * 64 * NQ;       // chunks beyond the tile exist only where the workgroup has
    const int ci = VFULL ? cu : min(cu, VTOT - 1);       // more lanes than the tile has chunks
    const int key = ci / CH, d0 = (ci % CH) * 8;
    const u32x4 t = (E || key < sk) ? vreg[i] : u32x4{0u, 0u, 0u, 0u};
    if (VFULL || cu < VTOT) *reinterpret_cast<u32x4*>(vsh + key * VP + d0) = t;
  }
  __syncthreads();   // K and V complete

  // the A fragment of the second dot for 32-key step kk and head-dim tile dt: keys 32kk+16h+4g+i at
  // k-slot 4h+i, head-dim 16dt+c.  Lane c addresses row (c / 4) and columns 4 (c % 4) .. +3 of the tile.
  const uint16_t* vlane = vsh + (4 * g + (c >> 2)) * VP + 4 * (c & 3);
  auto vfrag = [&](int kk, int dt) {
    typedef short s16x4 __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    const uint16_t* p = vlane + 32 * kk * VP + 16 * dt;
    const u32x2 lo = __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p)));
    const u32x2 hi = __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 16 * VP)));
    return u32x4{lo[0], lo[1], hi[0], hi[1]};
  };
  // ---- everything behind the barrier as a function of TL, the number of key tiles the wavefront needs (the
  // same for the whole wavefront, so which instance runs is a scalar branch): straight-line code per count.
  // With the count a run-time bound of unrolled loops the compiler merged the paths register by register -
  // on 128 x 128 x 64, 497 of 1266 instructions were moves - and held 212 registers.
  auto work = [&](auto tl_c) __attribute__((always_inline)) {
    constexpr int TL = decltype(tl_c)::value;
    constexpr int KST = (TL + 1) / 2;           // 32-key steps of the second dot
    // ---- first dot, transposed: tile kt = K_kt(16 x D) . Q^T -----------------------------
    // (the LDS reads of up to eight fragments first, then their matrix instructions: one latency per
    // batch, not one per tile)
    f32x4 acc[TL];
    constexpr int CT = KS >= 8 ? 1 : 8 / KS;     // key tiles per batch
#pragma unroll
    for (int k0 = 0; k0 < TL; k0 += CT) {
      u32x4 kfr[CT][KS];
#pragma unroll
      for (int j = 0; j < CT; ++j) {
        if (k0 + j < TL) {
#pragma unroll
          for (int ks = 0; ks < KS; ++ks)
            kfr[j][ks] = *reinterpret_cast<const u32x4*>(ksh + ((k0 + j) * 16 + c) * KP + ks * 32 + 8 * g);
        }
      }
#pragma unroll
      for (int j = 0; j < CT; ++j) {
        if (k0 + j < TL) {
          acc[k0 + j] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) acc[k0 + j] = Mfma<T>::run(kfr[j][ks], qf[ks], acc[k0 + j]);
        }
      }
    }
    // the first 32-key step of V^T for the second dot: its LDS latency passes under the softmax
    // (where registers allow)
    constexpr bool PRE = D <= 64;
    u32x4 vpre[PRE ? D / 16 : 1];
    if constexpr (PRE) {
#pragma unroll
      for (int dt = 0; dt < D / 16; ++dt) vpre[dt] = vfrag(0, dt);
    }
    // ---- scale, mask, softmax of query row q0+c: the lane holds S[q0+c][16kt+4g+i].  The scores
    // are kept in units of log 2 (scale, mask and fill times log2 e), so that the exponential is the
    // hardware's base-2 one without a multiplication per score. ------------------------------------
    constexpr float kLog2e = 1.4426950408889634f, kLn2 = 0.6931471805599453f;
    const float sc2 = a.scale * kLog2e;
    const float fill2 = a.fill == -INFINITY ? -INFINITY : fmaxf(a.fill * kLog2e, -3.0e38f);
    float mx = -INFINITY;
#pragma unroll
    for (int kt = 0; kt < TL; ++kt) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float z = acc[kt][i] * sc2;
        if (X && a.mask) z = fmaf(mk[kt][i], kLog2e, z);
        acc[kt][i] = z;
      }
      if (a.causal && 16 * kt + 15 > q0) {             // the tile holds keys right of some row's diagonal
#pragma unroll
        for (int i = 0; i < 4; ++i) if (kt * 16 + 4 * g + i > qi) acc[kt][i] = fill2;
      }
      if (!E && 16 * kt + 15 >= sk) {                  // the tile runs past the last key
#pragma unroll
        for (int i = 0; i < 4; ++i) if (kt * 16 + 4 * g + i >= sk) acc[kt][i] = -INFINITY;
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) mx = fmaxf(mx, acc[kt][i]);
    }
    mx = rows_allreduce<MaxOp>(mx);
    float sum = 0.f;
#pragma unroll
    for (int kt = 0; kt < TL; ++kt)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float e = __builtin_amdgcn_exp2f(acc[kt][i] - mx);
        acc[kt][i] = e;
        sum += e;
      }
    sum = rows_allreduce<SumOp>(sum);
    const float inv = __builtin_amdgcn_rcpf(sum);
    if (X && a.lse && g == 0 && qi < sq) a.lse[(int64_t)b * sq + qi] = (mx + __builtin_amdgcn_logf(sum)) * kLn2;
    // P rounded to the dot's dtype, packed in k-slot order: slots 4h+i of step kk <- tile 2kk+h
    u32x4 pb[KST];                              // P^T, the second dot's B fragments
#pragma unroll
    for (int kk = 0; kk < KST; ++kk)
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int kt = 2 * kk + h;
        float p[4] = {0.f, 0.f, 0.f, 0.f};
        if (kt < TL) {
#pragma unroll
          for (int i = 0; i < 4; ++i) p[i] = acc[kt < TL ? kt : 0][i] * inv;
        }
        pb[kk][2 * h] = Mfma<T>::pack(p[0], p[1]);
        pb[kk][2 * h + 1] = Mfma<T>::pack(p[2], p[3]);
      }

    // ---- second dot, transposed: O^T(D x 16) = V^T(D x keys) . P^T ---------------------------
    f32x4 o[D / 16];
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt) {
      if constexpr (PRE) o[dt] = Mfma<T>::run(vpre[dt], pb[0], f32x4{0.f, 0.f, 0.f, 0.f});
      else o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
#pragma unroll
    for (int kk = PRE ? 1 : 0; kk < KST; ++kk) {
#pragma unroll
      for (int dt = 0; dt < D / 16; ++dt) o[dt] = Mfma<T>::run(vfrag(kk, dt), pb[kk], o[dt]);
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
      if (E || qi < sq) *reinterpret_cast<u32x4*>(orow + dp * 32) = u32x4{r0[0], r1[0], r0[1], r1[1]};
    }
  };
  if (active) {
    switch (tiles) {
      case 1: work(TileCount<1>{}); break;
      case 2: if constexpr (NK >= 2) work(TileCount<2>{}); break;
      case 3: if constexpr (NK >= 4) work(TileCount<3>{}); break;
      case 4: if constexpr (NK >= 4) work(TileCount<4>{}); break;
      case 5: if constexpr (NK >= 8) work(TileCount<5>{}); break;
      case 6: if constexpr (NK >= 8) work(TileCount<6>{}); break;
      case 7: if constexpr (NK >= 8) work(TileCount<7>{}); break;
      case 8: if constexpr (NK >= 8) work(TileCount<8>{}); break;
      default: break;
    }
  }
}

inline int64_t attn_lds_bytes(int NK, int D) {
  const int NKP = NK < 2 ? 2 : NK;
  const int VP = D + (D == 64 ? 8 : 16);
  return 2 * ((int64_t)NKP * 16 * VP + (int64_t)NK * 16 * (D + 8));
}

template <typename T, int NQ, int NK, int D>
hipError_t attn_launch_one(const AttnArgs& a, hipStream_t s) {
  const bool extras = a.mask || a.gate || a.res || a.lse;
  const bool exact = NK >= 2 && a.sq == 16 * NQ && a.sk == 16 * NK;
  const dim3 grid(a.batch), wg(64 * NQ);
  const size_t lds = (size_t)attn_lds_bytes(NK, D);
  if (lds > 64 * 1024) {     // more dynamic LDS than a kernel may use unasked
    const void* f = extras ? reinterpret_cast<const void*>(attn_stitch_kernel<T, NQ, NK, D, true, false>)
                           : reinterpret_cast<const void*>(attn_stitch_kernel<T, NQ, NK, D, false, false>);
    const hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    if constexpr (NK >= 2) {
      const void* fe = extras ? reinterpret_cast<const void*>(attn_stitch_kernel<T, NQ, NK, D, true, true>)
                              : reinterpret_cast<const void*>(attn_stitch_kernel<T, NQ, NK, D, false, true>);
      const hipError_t e2 = hipFuncSetAttribute(fe, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      if (e2 != hipSuccess) return e2;
    }
  }
  if constexpr (NK >= 2) {
    if (exact) {
      if (extras) hipLaunchKernelGGL((attn_stitch_kernel<T, NQ, NK, D, true, true>), grid, wg, lds, s, a);
      else hipLaunchKernelGGL((attn_stitch_kernel<T, NQ, NK, D, false, true>), grid, wg, lds, s, a);
      return hipGetLastError();
    }
  }
  if (extras) hipLaunchKernelGGL((attn_stitch_kernel<T, NQ, NK, D, true, false>), grid, wg, lds, s, a);
  else hipLaunchKernelGGL((attn_stitch_kernel<T, NQ, NK, D, false, false>), grid, wg, lds, s, a);
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
