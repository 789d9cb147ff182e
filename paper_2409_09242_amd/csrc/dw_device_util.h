// Small device helpers shared by the kernel translation units of libdw.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dw {

// fp32 -> bfloat16 bit pattern, round to nearest even (no NaN handling: the callers' values are finite)
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// 16-byte accesses with the non-temporal policy: for data that streams through once (optimizer state, gradients) and
// must not displace lines that are reused (the centre, sign bits, other blocks' operand panels)
typedef float dw_f32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 nt_load4(const float* p) {
  const dw_f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const dw_f32x4*>(p));
  return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ float4 nt_load4(const float4* p) { return nt_load4(reinterpret_cast<const float*>(p)); }
__device__ __forceinline__ void nt_store4(float* p, float4 x) {
  const dw_f32x4 v = {x.x, x.y, x.z, x.w};
  __builtin_nontemporal_store(v, reinterpret_cast<dw_f32x4*>(p));
}
__device__ __forceinline__ void nt_store4(float4* p, float4 x) { nt_store4(reinterpret_cast<float*>(p), x); }

}  // namespace dw
