// Device-side helpers shared by the libsparq kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sparq {

constexpr int kWave = 64;
constexpr float kLog2e = 1.4426950408889634f;

// ---- 16-bit storage formats: exact widening to fp32, round-to-nearest-even narrowing ----
struct F16 {
  static __device__ __forceinline__ float lo(uint32_t w) {
    return (float)__builtin_bit_cast(_Float16, (uint16_t)(w & 0xffffu));
  }
  static __device__ __forceinline__ float hi(uint32_t w) {
    return (float)__builtin_bit_cast(_Float16, (uint16_t)(w >> 16));
  }
  static __device__ __forceinline__ float widen(uint16_t c) { return (float)__builtin_bit_cast(_Float16, c); }
  static __device__ __forceinline__ uint16_t narrow(float x) { return __builtin_bit_cast(uint16_t, (_Float16)x); }
};

struct BF16 {
  static __device__ __forceinline__ float lo(uint32_t w) { return __uint_as_float(w << 16); }
  static __device__ __forceinline__ float hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
  static __device__ __forceinline__ float widen(uint16_t c) { return __uint_as_float((uint32_t)c << 16); }
  static __device__ __forceinline__ uint16_t narrow(float x) {
    uint32_t u = __float_as_uint(x);
    u += 0x7fffu + ((u >> 16) & 1u);   // finite inputs only
    return (uint16_t)(u >> 16);
  }
};

template <class T>
__device__ __forceinline__ void unpack8(const uint4& v, float (&f)[8]) {
  f[0] = T::lo(v.x); f[1] = T::hi(v.x); f[2] = T::lo(v.y); f[3] = T::hi(v.y);
  f[4] = T::lo(v.z); f[5] = T::hi(v.z); f[6] = T::lo(v.w); f[7] = T::hi(v.w);
}

// 16 bytes of cache data: every such load in this library reads what the launch uses once (rows of Kt, K and V,
// sorted keys), so it is marked non-temporal: the line is not kept in L2 or in the memory-side cache on account of
// this read.  Measured against plain loads: the decode step 6-10 % faster on every many-head workload (config 2
// 52.8 -> 47.6 us, config 4 157.3 -> 147.4, config 5 243.6 -> 222.1), 1-3 % slower only where the query heads of
// a KV group select for themselves in the one-launch kernel and find each other's rows in L2.
__device__ __forceinline__ uint4 load16(const void* p) {
  typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
  const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}

// ---- order-preserving map fp32 -> uint32 (larger float <=> larger key; -0 == +0) ----
// Every finite float maps to a key >= 0x00800000, so key 0 is below all of them.
__device__ __forceinline__ uint32_t float_to_key(float x) {
  uint32_t u = __float_as_uint(x);
  if (u == 0x80000000u) u = 0u;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float key_to_float(uint32_t k) {
  return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

// 2^x as the hardware's one instruction.  exp2f() wraps it in range scaling so that results below 2^-126 come
// out as denormals; a softmax weight that small adds nothing to a sum whose largest term is 1.
__device__ __forceinline__ float exp2_weight(float x) { return __builtin_amdgcn_exp2f(x); }

// ---- wave64 primitives (DPP: no LDS traffic, a few cycles each) ----
template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false));
}
__device__ __forceinline__ float lane_f(float v, int lane) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}
// Butterfly all-reduce over aligned groups of N lanes (N = 8 or 16): xor 1 and xor 2 by quad
// permutes, then half-row mirror and row mirror, which act as xor 4 / xor 8 once the quads (halves)
// are uniform.  Every step adds a pair commutatively, so all lanes of a group end with the same bits.
template <int N>
__device__ __forceinline__ float group_sum(float v) {
  v += dpp_f<0xB1>(v);                  // quad_perm [1,0,3,2]
  v += dpp_f<0x4E>(v);                  // quad_perm [2,3,0,1]
  v += dpp_f<0x141>(v);                 // row_half_mirror
  if (N >= 16) v += dpp_f<0x140>(v);    // row_mirror
  return v;
}
template <int N>
__device__ __forceinline__ float group_max(float v) {
  v = fmaxf(v, dpp_f<0xB1>(v));
  v = fmaxf(v, dpp_f<0x4E>(v));
  v = fmaxf(v, dpp_f<0x141>(v));
  if (N >= 16) v = fmaxf(v, dpp_f<0x140>(v));
  return v;
}
// reductions over the whole wave: the result is wave-uniform
__device__ __forceinline__ float wave_sum(float v) {
  v = group_sum<16>(v);
  return (lane_f(v, 0) + lane_f(v, 16)) + (lane_f(v, 32) + lane_f(v, 48));
}
__device__ __forceinline__ float wave_max(float v) {
  v = group_max<16>(v);
  return fmaxf(fmaxf(lane_f(v, 0), lane_f(v, 16)), fmaxf(lane_f(v, 32), lane_f(v, 48)));
}
// sum over aligned groups of LPR lanes (8, 16 or 32), same value in every lane of a group
template <int LPR>
__device__ __forceinline__ float lanes_sum(float v) {
  if (LPR == 8) return group_sum<8>(v);
  v = group_sum<16>(v);
  if (LPR == 32) v += __shfl_xor(v, 16);
  return v;
}
// inclusive prefix sum across the 64 lanes with DPP row shifts and row broadcasts
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_or_zero(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xf, false);
}
__device__ __forceinline__ uint32_t wave_scan_incl(uint32_t v) {
  v += dpp_or_zero<0x111, 0xf>(v);   // row_shr:1
  v += dpp_or_zero<0x112, 0xf>(v);   // row_shr:2
  v += dpp_or_zero<0x114, 0xf>(v);   // row_shr:4
  v += dpp_or_zero<0x118, 0xf>(v);   // row_shr:8   -> scan inside each row of 16
  v += dpp_or_zero<0x142, 0xa>(v);   // row_bcast:15 into rows 1 and 3
  v += dpp_or_zero<0x143, 0xc>(v);   // row_bcast:31 into rows 2 and 3
  return v;
}

// exp2 that maps (-inf) - (-inf) situations to weight 0 instead of NaN
__device__ __forceinline__ float weight_exp2(float m, float m_ref) {
  return (m == -INFINITY) ? 0.0f : exp2f(m - m_ref);
}

}  // namespace sparq
