// Device-side helpers shared by the kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "vf_internal.h"

namespace vf {

// fp32 -> bf16 bits, round-to-nearest-even (NaN stays NaN): the conversion instruction of this GPU
// (v_cvt_pk_bf16_f32).  A run over all 2^32 inputs gave the bits of the integer form
//   u + 0x7fff + ((u >> 16) & 1) >> 16,  NaN -> (u >> 16) | 0x40
// for every one of them, at a seventh of the instructions.
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  const __bf16 h = static_cast<__bf16>(f);
  return __builtin_bit_cast(bf16_t, h);
}
// two values, packed low | high << 16
__device__ __forceinline__ uint32_t f32x2_to_bf16x2(float lo, float hi) {
  typedef __bf16 vf_bf16x2 __attribute__((ext_vector_type(2)));
  typedef float vf_f32x2c __attribute__((ext_vector_type(2)));
  const vf_f32x2c v = {lo, hi};
  const vf_bf16x2 h = __builtin_convertvector(v, vf_bf16x2);
  return __builtin_bit_cast(uint32_t, h);
}
__device__ __forceinline__ float bf16_to_f32(bf16_t h) { return __uint_as_float(((uint32_t)h) << 16); }
__device__ __forceinline__ float round_bf16(float f) { return bf16_to_f32(f32_to_bf16(f)); }

__device__ __forceinline__ float load_f(const float* p) { return *p; }
__device__ __forceinline__ float load_f(const bf16_t* p) { return bf16_to_f32(*p); }
__device__ __forceinline__ void store_f(float* p, float v) { *p = v; }
__device__ __forceinline__ void store_f(bf16_t* p, float v) { *p = f32_to_bf16(v); }
// two consecutive elements at an address aligned for the pair
__device__ __forceinline__ void store_f2(float* p, float a, float b) { *reinterpret_cast<float2*>(p) = make_float2(a, b); }
__device__ __forceinline__ void store_f2(bf16_t* p, float a, float b) {
  *reinterpret_cast<uint32_t*>(p) = (uint32_t)f32_to_bf16(a) | ((uint32_t)f32_to_bf16(b) << 16);
}

// Accesses with the non-temporal hint, for data that is read or written once and not used again soon.
typedef float vf_f32x4 __attribute__((ext_vector_type(4)));
typedef float vf_f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t vf_u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 load4_stream(const float* p) {
  const vf_f32x4 r = __builtin_nontemporal_load(reinterpret_cast<const vf_f32x4*>(p));
  return float4{r[0], r[1], r[2], r[3]};
}
__device__ __forceinline__ float2 load2_stream(const float* p) {
  const vf_f32x2 r = __builtin_nontemporal_load(reinterpret_cast<const vf_f32x2*>(p));
  return float2{r[0], r[1]};
}
__device__ __forceinline__ void store16_stream(void* p, uint4 v) {
  const vf_u32x4 r = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(r, reinterpret_cast<vf_u32x4*>(p));
}

__device__ __forceinline__ void grad_store(const GradOut& g, int64_t p, float v) {
  float old = g.accumulate ? g.dst[p] : 0.f;
  g.dst[p] = fmaf(g.alpha, v, old);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

}  // namespace vf
