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

// fp32 operands on the bf16 matrix cores: x = hi + mid + lo with three bf16 terms (each the rounded remainder of the
// one before, so |mid| <= 2^-8 |x|, |lo| <= 2^-16 |x| and the sum is x to within 2^-25 |x|). A product then takes the
// six partial products hi.hi + hi.mid + mid.hi + hi.lo + mid.mid + lo.hi; the three that are left out are below
// 2^-23 |x||y| together, the size of the rounding of an fp32 product. The matrix cores run bf16 sixteen times as
// fast as fp32, so the six products cost three eighths of the one.
typedef unsigned u32x4_t_ __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void split_bf16x3(const float (&x)[8], bf16x8_t (&o)[3]) {
  u32x4_t_ w[3];
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const float x0 = x[2 * t], x1 = x[2 * t + 1];
    const unsigned h = pack_bf16x2(x0, x1);
    const float r0 = x0 - __uint_as_float(h << 16), r1 = x1 - __uint_as_float(h & 0xffff0000u);
    const unsigned m = pack_bf16x2(r0, r1);
    const float s0 = r0 - __uint_as_float(m << 16), s1 = r1 - __uint_as_float(m & 0xffff0000u);
    w[0][t] = h;
    w[1][t] = m;
    w[2][t] = pack_bf16x2(s0, s1);
  }
#pragma unroll
  for (int q = 0; q < 3; ++q) o[q] = __builtin_bit_cast(bf16x8_t, w[q]);
}
// acc += (a as three terms) x (b as three terms), smallest partial products first
__device__ __forceinline__ f32x16_t mfma_bf16x3(const bf16x8_t (&a)[3], const bf16x8_t (&b)[3], f32x16_t acc) {
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[2], b[0], acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[1], b[1], acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0], b[2], acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[1], b[0], acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0], b[1], acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0], b[0], acc, 0, 0, 0);
  return acc;
}

}  // namespace hgnn
