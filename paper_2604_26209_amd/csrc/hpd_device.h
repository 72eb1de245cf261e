// Small device helpers: bf16 <-> fp32 conversion and vector loads.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hpd {

struct bf16_t {
  uint16_t bits;
};

__device__ __forceinline__ float bf16_bits_to_float(uint32_t bits) {
  return __uint_as_float(bits << 16);
}

// round-to-nearest-even; NaN stays NaN
__device__ __forceinline__ uint32_t float_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}

__device__ __forceinline__ float to_float(float x) { return x; }
__device__ __forceinline__ float to_float(bf16_t x) { return bf16_bits_to_float(x.bits); }

template <typename T>
__device__ __forceinline__ T from_float(float f);
template <>
__device__ __forceinline__ float from_float<float>(float f) { return f; }
template <>
__device__ __forceinline__ bf16_t from_float<bf16_t>(float f) {
  bf16_t r;
  r.bits = (uint16_t)float_to_bf16_bits(f);
  return r;
}

// Elements of a bf16 cache.  The stored value is the bf16 value (a rotated key rounded to bf16,
// round to nearest even: the precision of the cache; a value element as the caller gave it),
// and it is written in IEEE half format: the same 2 bytes per element, exact for
// 2^-14 <= |x| <= 65504 (bf16 has 8 significant bits, half has 11), within 2^-25 absolute below
// that, saturating above.  Both products of the attention then run on the half-precision matrix
// instruction, which takes the query and the softmax weights with 11 significant bits instead
// of 8.  Every kernel that writes or reads a pool goes through these.
__device__ __forceinline__ uint32_t cache_bits_pair(float a, float b) {
  // a, b hold bf16 values: the conversion towards zero is exact in the normal range of half
  // and saturates at the largest finite half
  return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(a, b));
}
__device__ __forceinline__ float cache_bits_to_float(uint32_t bits) {
  return (float)__builtin_bit_cast(_Float16, (uint16_t)bits);
}
template <typename T>
__device__ __forceinline__ T cache_from_float(float f);
template <>
__device__ __forceinline__ float cache_from_float<float>(float f) { return f; }
template <>
__device__ __forceinline__ bf16_t cache_from_float<bf16_t>(float f) {
  bf16_t r;
  r.bits = (uint16_t)cache_bits_pair(bf16_bits_to_float(float_to_bf16_bits(f)), 0.f);
  return r;
}
__device__ __forceinline__ float cache_to_float(float x) { return x; }
__device__ __forceinline__ float cache_to_float(bf16_t x) { return cache_bits_to_float(x.bits); }
// two bf16 values (the halves of w) as cache elements
__device__ __forceinline__ uint32_t cache_bits_from_bf16_pair(uint32_t w) {
  return cache_bits_pair(__uint_as_float(w << 16), __uint_as_float(w & 0xffff0000u));
}

// Rotation of one (first-half, second-half) channel pair.  Every kernel that rotates a key
// or a query uses this exact sequence so that all of them round identically.
__device__ __forceinline__ void rope_pair(float x1, float x2, float c, float s, float& r1, float& r2) {
  r1 = __fmaf_rn(x1, c, -__fmul_rn(x2, s));
  r2 = __fmaf_rn(x2, c, __fmul_rn(x1, s));
}

// 8 consecutive elements (16-byte aligned for bf16, 32-byte for fp32) to fp32
__device__ __forceinline__ void load8(const float* p, float out[8]) {
  const float4 a = *reinterpret_cast<const float4*>(p);
  const float4 b = *reinterpret_cast<const float4*>(p + 4);
  out[0] = a.x; out[1] = a.y; out[2] = a.z; out[3] = a.w;
  out[4] = b.x; out[5] = b.y; out[6] = b.z; out[7] = b.w;
}
__device__ __forceinline__ void load8(const bf16_t* p, float out[8]) {
  const uint4 a = *reinterpret_cast<const uint4*>(p);
  out[0] = bf16_bits_to_float(a.x & 0xffffu); out[1] = bf16_bits_to_float(a.x >> 16);
  out[2] = bf16_bits_to_float(a.y & 0xffffu); out[3] = bf16_bits_to_float(a.y >> 16);
  out[4] = bf16_bits_to_float(a.z & 0xffffu); out[5] = bf16_bits_to_float(a.z >> 16);
  out[6] = bf16_bits_to_float(a.w & 0xffffu); out[7] = bf16_bits_to_float(a.w >> 16);
}
// 8 consecutive elements of a pool
__device__ __forceinline__ void load8_cache(const float* p, float out[8]) { load8(p, out); }
__device__ __forceinline__ void load8_cache(const bf16_t* p, float out[8]) {
  const uint4 a = *reinterpret_cast<const uint4*>(p);
  out[0] = cache_bits_to_float(a.x & 0xffffu); out[1] = cache_bits_to_float(a.x >> 16);
  out[2] = cache_bits_to_float(a.y & 0xffffu); out[3] = cache_bits_to_float(a.y >> 16);
  out[4] = cache_bits_to_float(a.z & 0xffffu); out[5] = cache_bits_to_float(a.z >> 16);
  out[6] = cache_bits_to_float(a.w & 0xffffu); out[7] = cache_bits_to_float(a.w >> 16);
}

}  // namespace hpd
