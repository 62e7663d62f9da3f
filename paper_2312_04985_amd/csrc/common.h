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

__device__ __forceinline__ uint4 load16(const void* p) { return *reinterpret_cast<const uint4*>(p); }

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

// ---- wave64 primitives ----
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
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
