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

// GELU for bf16 outputs.  x * Phi(x) with Phi(x) = 1 / (1 + exp(-p(x))), p an odd polynomial of
// degree 5 fitted (minimax over [-10, 10]) to the logit of the normal distribution function:
// |error| of the product <= 2.6e-5, two orders below the bf16 rounding of the result, in 7
// vector and 2 transcendental instructions.  The polynomial is evaluated on x clamped to
// [-8, 8] (beyond that Phi is 0 or 1 to 1e-12 and the fitted polynomial would turn over).
__device__ __forceinline__ float gelu_fast(float x) {
  const float xc = __builtin_amdgcn_fmed3f(x, -8.0f, 8.0f);
  const float x2 = xc * xc;
  // -log2(e) * (1.59501577 + 0.07401129 x^2 - 0.00070303 x^4)
  float t = fmaf(1.0142630e-3f, x2, -1.0677572e-1f);
  t = fmaf(t, x2, -2.3011213f);
  const float e = __builtin_amdgcn_exp2f(t * xc);
  return x * __builtin_amdgcn_rcpf(1.0f + e);
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
