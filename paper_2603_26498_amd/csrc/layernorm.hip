// LayerNorm (or RMSNorm) over the last dimension, one wavefront per row (gfx950, wave64).
//
// The row (fp32) is read once with 16-byte loads and kept in registers; the
// mean and the centred sum of squares are reduced across the wave in fp32 (two
// passes over registers, no second trip to memory); the result is written as
// bf16 or fp32.  HBM-bound: 4*d bytes read + 2*d (or 4*d) bytes written per row.
#include "tcmv_internal.h"
#include "device_utils.h"

namespace tcmv {

template <int NV, bool OUT_BF16, bool RMS>
__global__ __launch_bounds__(256) void layernorm_kernel(const float* x, const float* __restrict__ gamma,
                                                        const float* __restrict__ beta, void* y,
                                                        int64_t rows, int d, float eps) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const int nvec = d >> 2;
  const float4* xr = reinterpret_cast<const float4*>(x + row * d);
  float4 v[NV];
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    const int i = lane + 64 * j;
    v[j] = (i < nvec) ? xr[i] : make_float4(0.f, 0.f, 0.f, 0.f);
    s += (v[j].x + v[j].y) + (v[j].z + v[j].w);
  }
  const float mean = RMS ? 0.f : wave_sum(s) / (float)d;
  float q = 0.f;
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    const int i = lane + 64 * j;
    if (i < nvec) {
      v[j].x -= mean; v[j].y -= mean; v[j].z -= mean; v[j].w -= mean;
      q += (v[j].x * v[j].x + v[j].y * v[j].y) + (v[j].z * v[j].z + v[j].w * v[j].w);
    }
  }
  const float rstd = 1.0f / sqrtf(wave_sum(q) / (float)d + eps);
  const float4* g4 = reinterpret_cast<const float4*>(gamma);
  const float4* b4 = reinterpret_cast<const float4*>(beta);
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    const int i = lane + 64 * j;
    if (i < nvec) {
      const float4 g = g4[i], b = RMS ? make_float4(0.f, 0.f, 0.f, 0.f) : b4[i];
      float4 o;
      o.x = v[j].x * rstd * g.x + b.x;
      o.y = v[j].y * rstd * g.y + b.y;
      o.z = v[j].z * rstd * g.z + b.z;
      o.w = v[j].w * rstd * g.w + b.w;
      if (OUT_BF16) {
        uint2 p;
        p.x = pack_bf16x2(o.x, o.y);
        p.y = pack_bf16x2(o.z, o.w);
        reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(y) + row * d)[i] = p;
      } else {
        reinterpret_cast<float4*>(reinterpret_cast<float*>(y) + row * d)[i] = o;
      }
    }
  }
}

template <bool OUT_BF16, bool RMS>
static hipError_t launch_ln_t(const float* x, const float* g, const float* b, void* y, int64_t rows, int d, float eps,
                              hipStream_t s) {
  dim3 grid((unsigned)((rows + 3) / 4)), block(256);
  const int nv = (d / 4 + 63) / 64;
#define TCMV_LN_CASE(N)                                                                                   \
  case N:                                                                                                 \
    hipLaunchKernelGGL((layernorm_kernel<N, OUT_BF16, RMS>), grid, block, 0, s, x, g, b, y, rows, d, eps); \
    break;
  switch (nv) {
    TCMV_LN_CASE(1) TCMV_LN_CASE(2) TCMV_LN_CASE(3) TCMV_LN_CASE(4)
    TCMV_LN_CASE(5) TCMV_LN_CASE(6) TCMV_LN_CASE(7) TCMV_LN_CASE(8)
    default: return hipErrorInvalidValue;
  }
#undef TCMV_LN_CASE
  return hipGetLastError();
}

// Reference for the bandwidth-bound kernels: n_in 16-byte words read once, n_out 16-byte words written once, no
// other work - what a kernel that moves these bytes can reach at best at this size.
__global__ __launch_bounds__(256) void stream_ref_kernel(const uint4* __restrict__ in, uint4* __restrict__ out,
                                                         size_t n_in, size_t n_out) {
  const size_t tid = (size_t)blockIdx.x * 256 + threadIdx.x, nt = (size_t)gridDim.x * 256;
  uint4 acc = {0u, 0u, 0u, 0u};
  for (size_t i = tid; i < n_in; i += nt) {
    const uint4 v = in[i];
    acc.x ^= v.x; acc.y ^= v.y; acc.z ^= v.z; acc.w ^= v.w;
  }
  for (size_t i = tid; i < n_out; i += nt) out[i] = acc;
}

hipError_t launch_stream_ref(const void* in, size_t in_bytes, void* out, size_t out_bytes, hipStream_t s) {
  if (in_bytes % 16 || out_bytes % 16 || reinterpret_cast<uintptr_t>(in) % 16 || reinterpret_cast<uintptr_t>(out) % 16)
    return hipErrorInvalidValue;
  if (in_bytes + out_bytes == 0) return hipSuccess;
  hipLaunchKernelGGL(stream_ref_kernel, dim3(2048), dim3(256), 0, s, reinterpret_cast<const uint4*>(in),
                     reinterpret_cast<uint4*>(out), in_bytes / 16, out_bytes / 16);
  return hipGetLastError();
}

hipError_t launch_layernorm(const float* x, const float* g, const float* b, void* y, int64_t rows, int d, float eps,
                            int out_bf16, hipStream_t s, int rms) {
  if (rows == 0) return hipSuccess;
  if (d % 4 || d <= 0 || d > 2048) return hipErrorInvalidValue;
  if (rms) return out_bf16 ? launch_ln_t<true, true>(x, g, b, y, rows, d, eps, s) : launch_ln_t<false, true>(x, g, b, y, rows, d, eps, s);
  return out_bf16 ? launch_ln_t<true, false>(x, g, b, y, rows, d, eps, s) : launch_ln_t<false, false>(x, g, b, y, rows, d, eps, s);
}

}  // namespace tcmv
