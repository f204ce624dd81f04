// Device-side scalar helpers: SiLU and its derivative, bf16 rounding, matrix-core vector types.
#pragma once

#include <hip/hip_runtime.h>

namespace hgnn {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

// silu(t) = t / (1 + exp(-t)); exp through the hardware 2^x, reciprocal through v_rcp_f32
__device__ __forceinline__ float silu_f(float t) {
  const float e = __expf(-t);
  return t * __builtin_amdgcn_rcpf(1.0f + e);
}
// silu'(t) = s (1 + t (1 - s)),  s = sigmoid(t)
__device__ __forceinline__ float dsilu_f(float t) {
  const float e = __expf(-t);
  const float s = __builtin_amdgcn_rcpf(1.0f + e);
  return s * (1.0f + t * (1.0f - s));
}
__device__ __forceinline__ void silu_both(float t, float& y, float& dy) {
  const float e = __expf(-t);
  const float s = __builtin_amdgcn_rcpf(1.0f + e);
  y = t * s;
  dy = fmaf(y, 1.0f - s, s);   // s (1 + t (1 - s))
}

// float -> bf16, round to nearest even, through the packed hardware conversion (v_cvt_pk_bf16_f32)
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned pack_bf16x2(float lo, float hi) {
  const f32x2_t v = {lo, hi};
  const bf16x2_t b = __builtin_convertvector(v, bf16x2_t);
  return *reinterpret_cast<const unsigned*>(&b);
}
__device__ __forceinline__ unsigned f2bf_bits(float x) { return pack_bf16x2(x, 0.f) & 0xffffu; }

}  // namespace hgnn
