// Small device helpers for gfx950 kernels (wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

namespace tcmv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// round-to-nearest-even fp32 -> bf16 (hardware conversion on gfx950)
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  __bf16 b = (__bf16)f;
  return __builtin_bit_cast(uint16_t, b);
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  f32x2 v = {lo, hi};
  bf16x2 r = __builtin_convertvector(v, bf16x2);
  return __builtin_bit_cast(uint32_t, r);
}

// GELU, erf form: x/2 * (1 + erf(x / sqrt 2))
__device__ __forceinline__ float gelu_erf(float x) { return 0.5f * x * (1.0f + erff(x * 0.70710678118654752f)); }

// GELU for bf16 outputs: gelu(x) = max(x, 0) - |x| * Phi(-|x|), with the lower tail of the normal distribution
// evaluated as 2^G(|x|), G a polynomial of degree 5 fitted to log2 Phi(-a) on [0, 5.5] (|error| <= 3.6e-4, so the
// tail is accurate in RELATIVE terms: 2.5e-4).  Beyond 5.5 the argument of G is held: the result is then off by at
// most |x| * Phi(-5.5) < 2e-8 * |x|.  Absolute error of the product <= 3.5e-5; after rounding to bf16 the
// result is within one bf16 unit in the last place of the rounded exact value (or within 2^-22 of it where that is
// larger), for every x in [-10, 10].  5 fused multiply-adds, one exp2 and three other vector instructions.
__device__ __forceinline__ float gelu_bf16(float x) {
  const float a = fminf(fabsf(x), 5.5f);
  float t = fmaf(-0.00023325323f, a, 0.004869808f);
  t = fmaf(t, a, -0.044599235f);
  t = fmaf(t, a, -0.46968046f);
  t = fmaf(t, a, -1.1462616f);
  t = fmaf(t, a, -1.0003588f);
  const float tail = __builtin_amdgcn_exp2f(t);     // Phi(-|x|)
  return fmaf(-fabsf(x), tail, fmaxf(x, 0.0f));
}

// compile-time loop: f(std::integral_constant<int, 0>) ... f(<N-1>)
template <int I, int N, class F>
__device__ __forceinline__ void static_for_impl(F& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for_impl<I + 1, N>(f);
  }
}
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) { static_for_impl<0, N>(f); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

}  // namespace tcmv
