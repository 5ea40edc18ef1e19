// Device-side building blocks shared by the stitched kernels: 16-byte vector access
// for the three storage dtypes and wave64 all-reduce over lane groups.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fs {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

// Bit reinterpretation through a by-value parameter.  (Applying __builtin_bit_cast
// directly to a vector element expression such as t[i] reads element 0 for every i.)
__device__ __forceinline__ float as_f32(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ uint32_t as_u32(float f) { return __builtin_bit_cast(uint32_t, f); }

struct bf16_t { uint16_t bits; };   // storage-only tags: all arithmetic is fp32
struct f16_t { uint16_t bits; };

__device__ __forceinline__ float bf16_to_f32(uint32_t b) { return as_f32(b << 16); }
__device__ __forceinline__ uint32_t f32_to_bf16(float f) {
  return (uint32_t)__builtin_bit_cast(uint16_t, (__bf16)f);   // round to nearest even
}
__device__ __forceinline__ float f16_to_f32(uint32_t b) {
  return (float)__builtin_bit_cast(_Float16, (uint16_t)b);
}
__device__ __forceinline__ uint32_t f32_to_f16(float f) {
  return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)f);
}
// two fp32 -> one packed 32-bit word (lo in bits 0..15), round to nearest even: a single
// v_cvt_pk_{bf16,f16}_f32
__device__ __forceinline__ uint32_t pack2_bf16(float lo, float hi) {
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
__device__ __forceinline__ uint32_t pack2_f16(float lo, float hi) {
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2));
}

// One 16-byte vector of T <-> V fp32 values.
template <typename T> struct Vec;

template <> struct Vec<float> {
  static constexpr int V = 4;
  static constexpr uint32_t kOneBits = 0x3F800000u;
  static __device__ __forceinline__ u32x4 load_raw(const float* p) {
    return *reinterpret_cast<const u32x4*>(p);
  }
  static __device__ __forceinline__ void unpack(u32x4 t, float (&o)[4]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) o[i] = as_f32(t[i]);
  }
  static __device__ __forceinline__ void load(const float* p, float (&o)[4]) { unpack(load_raw(p), o); }
  static __device__ __forceinline__ void store(float* p, const float (&v)[4]) {
    f32x4 t = {v[0], v[1], v[2], v[3]};
    *reinterpret_cast<f32x4*>(p) = t;
  }
  static __device__ __forceinline__ float load1(const float* p) { return *p; }
  static __device__ __forceinline__ void store1(float* p, float v) { *p = v; }
};

template <> struct Vec<bf16_t> {
  static constexpr int V = 8;
  static constexpr uint32_t kOneBits = 0x3F80u;
  static __device__ __forceinline__ u32x4 load_raw(const bf16_t* p) {
    return *reinterpret_cast<const u32x4*>(p);
  }
  static __device__ __forceinline__ void unpack(u32x4 t, float (&o)[8]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      o[2 * i] = as_f32(t[i] << 16);
      o[2 * i + 1] = as_f32(t[i] & 0xFFFF0000u);
    }
  }
  static __device__ __forceinline__ void load(const bf16_t* p, float (&o)[8]) { unpack(load_raw(p), o); }
  static __device__ __forceinline__ void store(bf16_t* p, const float (&v)[8]) {
    u32x4 t;
#pragma unroll
    for (int i = 0; i < 4; ++i) t[i] = pack2_bf16(v[2 * i], v[2 * i + 1]);
    *reinterpret_cast<u32x4*>(p) = t;
  }
  static __device__ __forceinline__ float load1(const bf16_t* p) { return bf16_to_f32(p->bits); }
  static __device__ __forceinline__ void store1(bf16_t* p, float v) { p->bits = (uint16_t)f32_to_bf16(v); }
};

template <> struct Vec<f16_t> {
  static constexpr int V = 8;
  static constexpr uint32_t kOneBits = 0x3C00u;
  static __device__ __forceinline__ u32x4 load_raw(const f16_t* p) {
    return *reinterpret_cast<const u32x4*>(p);
  }
  static __device__ __forceinline__ void unpack(u32x4 t, float (&o)[8]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      o[2 * i] = f16_to_f32(t[i] & 0xFFFFu);
      o[2 * i + 1] = f16_to_f32(t[i] >> 16);
    }
  }
  static __device__ __forceinline__ void load(const f16_t* p, float (&o)[8]) { unpack(load_raw(p), o); }
  static __device__ __forceinline__ void store(f16_t* p, const float (&v)[8]) {
    u32x4 t;
#pragma unroll
    for (int i = 0; i < 4; ++i) t[i] = pack2_f16(v[2 * i], v[2 * i + 1]);
    *reinterpret_cast<u32x4*>(p) = t;
  }
  static __device__ __forceinline__ float load1(const f16_t* p) { return f16_to_f32(p->bits); }
  static __device__ __forceinline__ void store1(f16_t* p, float v) { p->bits = (uint16_t)f32_to_f16(v); }
};

// Streaming access for tensors that are touched exactly once: nontemporal 16-byte loads
// and stores keep them from displacing reusable lines in L2 / the memory-side cache and
// measurably raise achieved HBM bandwidth on gfx950 (plain copy: about +7%).
__device__ __forceinline__ u32x4 stream_load16(const void* p) {
  return __builtin_nontemporal_load(static_cast<const u32x4*>(p));
}
__device__ __forceinline__ void stream_store16(void* p, u32x4 v) {
  __builtin_nontemporal_store(v, static_cast<u32x4*>(p));
}
template <typename T> __device__ __forceinline__ u32x4 pack16(const float (&v)[Vec<T>::V]);
template <> __device__ __forceinline__ u32x4 pack16<float>(const float (&v)[4]) {
  u32x4 t;
#pragma unroll
  for (int i = 0; i < 4; ++i) t[i] = as_u32(v[i]);
  return t;
}
template <> __device__ __forceinline__ u32x4 pack16<bf16_t>(const float (&v)[8]) {
  u32x4 t;
#pragma unroll
  for (int i = 0; i < 4; ++i) t[i] = pack2_bf16(v[2 * i], v[2 * i + 1]);
  return t;
}
template <> __device__ __forceinline__ u32x4 pack16<f16_t>(const float (&v)[8]) {
  u32x4 t;
#pragma unroll
  for (int i = 0; i < 4; ++i) t[i] = pack2_f16(v[2 * i], v[2 * i + 1]);
  return t;
}

// ---- wave64 all-reduce over aligned groups of L lanes (L a power of two) -----------
// Steps inside a 16-lane DPP row are DPP permutes (quad swaps, half mirror, mirror);
// the two cross-row steps use the gfx950 permlane16/32 swaps, so no step goes through
// LDS.  Every lane of the wave must be active.
struct SumOp { static __device__ __forceinline__ float apply(float a, float b) { return a + b; } };
struct MaxOp { static __device__ __forceinline__ float apply(float a, float b) { return fmaxf(a, b); } };

template <int CTRL> __device__ __forceinline__ float dpp_move(float v) {
  return __builtin_bit_cast(
      float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, false));
}

template <class Op, int L> __device__ __forceinline__ float group_allreduce(float v) {
  static_assert(L == 1 || L == 2 || L == 4 || L == 8 || L == 16 || L == 32 || L == 64, "L");
  if (L >= 2) v = Op::apply(v, dpp_move<0xB1>(v));    // quad_perm [1,0,3,2]
  if (L >= 4) v = Op::apply(v, dpp_move<0x4E>(v));    // quad_perm [2,3,0,1]
  if (L >= 8) v = Op::apply(v, dpp_move<0x141>(v));   // row_half_mirror
  if (L >= 16) v = Op::apply(v, dpp_move<0x140>(v));  // row_mirror
  if (L >= 32) {
    uint32_t u = __builtin_bit_cast(uint32_t, v);
    auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    v = Op::apply(as_f32(r[0]), as_f32(r[1]));
  }
  if (L >= 64) {
    uint32_t u = __builtin_bit_cast(uint32_t, v);
    auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    v = Op::apply(as_f32(r[0]), as_f32(r[1]));
  }
  return v;
}

}  // namespace fs
