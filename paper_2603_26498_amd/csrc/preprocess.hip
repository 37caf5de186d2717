// Resize + normalise + patchify in one pass (gfx950).
//
// One workgroup produces one patch row (token).  Every output element is decoded
// to (channel, frame-in-group, patch row, patch column), fetched from the raw
// uint8 frame (directly, or through a 4-tap integer bilinear resample) and mapped
// through a 3x256 table of already-rounded normalised values, so the result is
// bit-exact by construction.  Stores are coalesced: consecutive lanes write
// consecutive element pairs of the row, padding columns included.
#include "tcmv_internal.h"
#include "device_utils.h"

namespace tcmv {

constexpr int kMaxPatch = 32;
constexpr int kFracBits = 11;
constexpr int kOne = 1 << kFracBits;

// Source taps of one destination index: half-pixel centres, clamp at the edge,
// weight of the second tap in 1/2048 units.
__device__ __forceinline__ void axis_tap(int i, int n_src, int n_dst, int& i0, int& i1, int& fr) {
  int num = (2 * i + 1) * n_src - n_dst;
  if (num < 0) num = 0;
  const int den = 2 * n_dst;
  int a = num / den;
  int f = ((num - a * den) * kOne + n_dst) / den;
  if (a >= n_src - 1) { a = n_src - 1; i1 = a; f = 0; } else { i1 = a + 1; }
  i0 = a; fr = f;
}

template <int P_, int TP_>
__global__ __launch_bounds__(256) void preprocess_kernel(PreprocArgs a) {
  const int P = P_ ? P_ : a.patch;
  const int TP = TP_ ? TP_ : a.tpatch;
  const int64_t r = blockIdx.x;
  const int item = a.prow_item[r];
  const int thw = a.prow_thw[r];
  const ItemDev it = a.items[item];
  const int t = thw >> 16, ph = (thw >> 8) & 255, pw = thw & 255;

  __shared__ int tap_r0[kMaxPatch], tap_r1[kMaxPatch], tap_fy[kMaxPatch];
  __shared__ int tap_c0[kMaxPatch], tap_c1[kMaxPatch], tap_fx[kMaxPatch];
  if (it.resized) {
    const int i = threadIdx.x;
    if (i < P) {
      axis_tap(ph * P + i, it.src_h, it.dst_h, tap_r0[i], tap_r1[i], tap_fy[i]);
    } else if (i >= 64 && i < 64 + P) {
      axis_tap(pw * P + (i - 64), it.src_w, it.dst_w, tap_c0[i - 64], tap_c1[i - 64], tap_fx[i - 64]);
    }
    __syncthreads();
  }

  const size_t frame_stride = (size_t)it.src_h * it.src_w * 3;
  const int row_stride = it.src_w * 3;
  const int pp = P * P;

  auto fetch = [&](int k) -> float {
    if (k >= a.k) return 0.0f;
    const int px = k % P;
    const int py = (k / P) % P;
    const int tt = (k / pp) % TP;
    const int c = k / (pp * TP);
    const int f = (it.n_frames == 1) ? 0 : t * TP + tt;
    const uint8_t* fr = it.frames + (size_t)f * frame_stride + c;
    int v;
    if (!it.resized) {
      v = fr[(size_t)(ph * P + py) * row_stride + (pw * P + px) * 3];
    } else {
      const int r0 = tap_r0[py], r1 = tap_r1[py], fy = tap_fy[py];
      const int c0 = tap_c0[px], c1 = tap_c1[px], fx = tap_fx[px];
      const uint32_t p00 = fr[(size_t)r0 * row_stride + c0 * 3];
      const uint32_t p01 = fr[(size_t)r0 * row_stride + c1 * 3];
      const uint32_t p10 = fr[(size_t)r1 * row_stride + c0 * 3];
      const uint32_t p11 = fr[(size_t)r1 * row_stride + c1 * 3];
      const uint32_t acc = p00 * (uint32_t)((kOne - fx) * (kOne - fy)) + p01 * (uint32_t)(fx * (kOne - fy)) +
                           p10 * (uint32_t)((kOne - fx) * fy) + p11 * (uint32_t)(fx * fy) +
                           (1u << (2 * kFracBits - 1));
      v = (int)(acc >> (2 * kFracBits));
    }
    return a.lut[c * 256 + v];
  };

  const int pairs = a.k_pad >> 1;
  if (a.out_bf16) {
    uint32_t* out = reinterpret_cast<uint32_t*>(a.patches) + (size_t)r * pairs;
    for (int k2 = threadIdx.x; k2 < pairs; k2 += 256) {
      const float x0 = fetch(2 * k2), x1 = fetch(2 * k2 + 1);
      // table entries are exactly representable in bf16: truncation is exact
      out[k2] = (__float_as_uint(x0) >> 16) | (__float_as_uint(x1) & 0xFFFF0000u);
    }
  } else {
    float2* out = reinterpret_cast<float2*>(a.patches) + (size_t)r * pairs;
    for (int k2 = threadIdx.x; k2 < pairs; k2 += 256) {
      out[k2] = make_float2(fetch(2 * k2), fetch(2 * k2 + 1));
    }
  }
}

hipError_t launch_preprocess(const PreprocArgs& a, hipStream_t s) {
  if (a.rows == 0) return hipSuccess;
  dim3 grid((unsigned)a.rows), block(256);
  if (a.patch == 14 && a.tpatch == 2) {
    hipLaunchKernelGGL((preprocess_kernel<14, 2>), grid, block, 0, s, a);
  } else if (a.patch == 14 && a.tpatch == 1) {
    hipLaunchKernelGGL((preprocess_kernel<14, 1>), grid, block, 0, s, a);
  } else if (a.patch == 16 && a.tpatch == 1) {
    hipLaunchKernelGGL((preprocess_kernel<16, 1>), grid, block, 0, s, a);
  } else {
    hipLaunchKernelGGL((preprocess_kernel<0, 0>), grid, block, 0, s, a);
  }
  return hipGetLastError();
}

}  // namespace tcmv
