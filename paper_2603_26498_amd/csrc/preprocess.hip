// Resize + normalise + patchify in one pass (gfx950).
//
// A patch row is 3*tpatch*patch runs of `patch` consecutive pixels of one channel of
// one source line, followed by zero padding.  Two kernels share that decomposition:
//
//  * strip kernel: a workgroup takes up to
//    16 horizontally adjacent patches of one patch line, copies their tpatch*patch
//    source line segments into LDS with coalesced 4-byte loads (every source byte is
//    read from HBM exactly once, all loads of a thread in flight together), then
//    produces the patch rows from LDS, normalising through a 3x256 table of already-rounded
//    values or, for bf16 output where the host has verified that it gives the same 768 values,
//    by one fused multiply-add and the hardware's bf16 conversion; on the bf16 path a wave takes whole rows and its lanes write
//    consecutive dwords (element pairs) of a row, on the fp32 path a thread writes runs;
//    resampled requests go the same way, except that the LDS lines are not copied but
//    computed: the strip's destination pixels, blended from their four source taps;
//  * run kernel (frames that are not 4-byte aligned, patch sizes without a compiled
//    strip kernel, window-major token order): one thread per run, reading its pixels
//    (or the four bilinear taps of each) straight from global memory.
//
// Integer / table arithmetic only: the result is bit-exact by construction.
#include "tcmv_internal.h"
#include "device_utils.h"
#include <type_traits>

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

template <int P_, int TP_, bool BF16>
__global__ __launch_bounds__(256) void preprocess_kernel(PreprocArgs a, int runs_per_row, int data_runs) {
  const int P = P_ ? P_ : a.patch;
  const int TP = TP_ ? TP_ : a.tpatch;
  __shared__ float lut[768];
  for (int i = threadIdx.x; i < 768; i += 256) lut[i] = a.lut[i];
  __syncthreads();
  const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t ri = gid / runs_per_row;                 // index into the list of rows handled here
  if (ri >= a.n_run_rows) return;
  const int64_t r = a.run_rows[ri];                      // patch row (token)
  const int run = (int)(gid - ri * runs_per_row);
  const int k0 = run * P;                                // first element of the run inside the row
  typedef typename std::conditional<BF16, uint16_t, float>::type out_t;
  out_t* out = reinterpret_cast<out_t*>(a.patches) + (size_t)r * a.k_pad + k0;
  auto emit = [&](int i, float x) {
    if (BF16) reinterpret_cast<uint16_t*>(out)[i] = (uint16_t)(__float_as_uint(x) >> 16);   // table entries are exact in bf16
    else reinterpret_cast<float*>(out)[i] = x;
  };
  if (run >= data_runs) {                                // padding columns
    const int n = min(P, a.k_pad - k0);
    for (int i = 0; i < n; ++i) emit(i, 0.f);
    return;
  }
  const int item = a.prow_item[r];
  const int thw = a.prow_thw[r];
  const ItemDev it = a.items[item];
  const int t = thw >> 16, ph = (thw >> 8) & 255, pw = thw & 255;
  const int py = run % P;
  const int tt = (run / P) % TP;
  const int c = run / (P * TP);
  const int f = (it.n_frames == 1) ? 0 : t * TP + tt;
  const uint8_t* fr = it.frames + (size_t)f * it.src_h * it.src_w * 3 + c;
  const int row_stride = it.src_w * 3;
  const float* lc = lut + c * 256;
  float x[P_ ? P_ : kMaxPatch];
  if (!it.resized) {
    const uint8_t* src = fr + (size_t)(ph * P + py) * row_stride + (size_t)(pw * P) * 3;
#pragma unroll
    for (int i = 0; i < (P_ ? P_ : kMaxPatch); ++i)
      if (i < P) x[i] = lc[src[3 * i]];
  } else {
    int r0, r1, fy;
    axis_tap(ph * P + py, it.src_h, it.dst_h, r0, r1, fy);
    const uint8_t* l0 = fr + (size_t)r0 * row_stride;
    const uint8_t* l1 = fr + (size_t)r1 * row_stride;
#pragma unroll
    for (int i = 0; i < (P_ ? P_ : kMaxPatch); ++i)
      if (i < P) {
        int c0, c1, fx;
        axis_tap(pw * P + i, it.src_w, it.dst_w, c0, c1, fx);
        const uint32_t p00 = l0[c0 * 3], p01 = l0[c1 * 3], p10 = l1[c0 * 3], p11 = l1[c1 * 3];
        const uint32_t acc = p00 * (uint32_t)((kOne - fx) * (kOne - fy)) + p01 * (uint32_t)(fx * (kOne - fy)) +
                             p10 * (uint32_t)((kOne - fx) * fy) + p11 * (uint32_t)(fx * fy) +
                             (1u << (2 * kFracBits - 1));
        x[i] = lc[acc >> (2 * kFracBits)];
      }
  }
  if (BF16 && (P_ % 2 == 0) && P_ > 0) {                 // even run length: 4-byte stores of bf16 pairs
    uint32_t* o2 = reinterpret_cast<uint32_t*>(out);
#pragma unroll
    for (int i = 0; i < P_ / 2; ++i)
      o2[i] = (__float_as_uint(x[2 * i]) >> 16) | (__float_as_uint(x[2 * i + 1]) & 0xFFFF0000u);
  } else {
#pragma unroll
    for (int i = 0; i < (P_ ? P_ : kMaxPatch); ++i)
      if (i < P) emit(i, x[i]);
  }
}

// Strip kernel: see the file comment.  Only instantiated for compile-time patch sizes.
// RES: the strips of this launch are resampled ones (they need tap tables in LDS; the copy instantiation does
//      without them, which lets one more workgroup live on a compute unit).
// AFF: the normalised bf16 value is computed - one fused multiply-add and the hardware's round-to-nearest-even
//      conversion, which the host has checked against all 768 table entries - instead of looked up: no table
//      in LDS, no bank conflicts between lanes that hold different pixel values.
template <int P_, int TP_, bool BF16, bool AFF, bool RES>
__global__ __launch_bounds__(256) void preprocess_strip_kernel(PreprocArgs a, int first, int runs_per_row, int data_runs) {
  constexpr int P = P_ ? P_ : 1, TP = TP_ ? TP_ : 1;
  constexpr int SEG = kStripTokens * P * 3;              // bytes of one line segment (multiple of 4)
  static_assert(SEG % 4 == 0, "segment size");
  __shared__ float lut[AFF ? 1 : 768];
  // lanes that work on neighbouring lines read the same byte offset of each: the line stride is an odd number
  // of dwords so that those reads fall into different banks
  __shared__ __attribute__((aligned(16))) uint8_t seg[TP * P][SEG + 4];
  const PreStrip sp = a.strips[first + blockIdx.x];
  const int ntok = sp.ntok;
  const int nbytes = ntok * P * 3;
  const bool still = sp.flags & kStripStill;                       // a still image is its own second frame
  const int nlines = still ? P : TP * P;
  if constexpr (!AFF)
    for (int i = threadIdx.x; i < 768; i += 256) lut[i] = a.lut[i];
  if constexpr (!RES) {
    // source line segments -> LDS, 4 bytes per lane, then the (at most 3) tail bytes of each line.  All loads
    // of a thread are issued before the first is used (a fixed-count loop over the full strip width, lanes
    // beyond the strip's own width masked off), so a workgroup has its whole input in flight at once.
    const int ndw = nbytes >> 2;
    {
      constexpr int NDW = SEG / 4;                         // dwords of a full-width line segment
      constexpr int NL = (TP * P * NDW + 255) / 256;       // loads per thread
      uint32_t v[NL];
#pragma unroll
      for (int j = 0; j < NL; ++j) {
        const int i = threadIdx.x + 256 * j;
        const int line = i / NDW, dw = i - line * NDW;
        v[j] = 0u;
        if (line < nlines && dw < ndw) {
          const uint8_t* src = sp.src + (size_t)(line / P) * sp.frame_stride + (size_t)(line % P) * sp.row_stride;
          v[j] = reinterpret_cast<const uint32_t*>(src)[dw];
        }
      }
#pragma unroll
      for (int j = 0; j < NL; ++j) {
        const int i = threadIdx.x + 256 * j;
        const int line = i / NDW, dw = i - line * NDW;
        if (line < nlines && dw < ndw) reinterpret_cast<uint32_t*>(seg[line])[dw] = v[j];
      }
    }
    const int ntail = nbytes & 3;
    for (int i = threadIdx.x; i < nlines * ntail; i += 256) {
      const int line = i / ntail, b = (ndw << 2) + (i - line * ntail);
      seg[line][b] = sp.src[(size_t)(line / P) * sp.frame_stride + (size_t)(line % P) * sp.row_stride + b];
    }
  } else if constexpr (RES) {
    // Resampled request: the strip's destination pixels are computed into the same LDS lines (as the uint8
    // values a resized frame would hold), so everything after this point is shared with the copy case.
    // Taps and weights of the strip's columns and lines are worked out once per workgroup; a thread then
    // takes destination pixels with lanes running along the line (neighbouring lanes read neighbouring
    // source pixels) and blends the three channels of each with the same four weights.
    __shared__ int col_c0[kStripTokens * P], col_c1[kStripTokens * P], col_fx[kStripTokens * P];
    __shared__ int line_r0[TP * P], line_r1[TP * P], line_fy[TP * P];
    const ItemDev it = a.items[sp.item];
    const int row_stride = it.src_w * 3;
    const int npx = ntok * P;
    for (int x = threadIdx.x; x < npx; x += 256) {
      int c0, c1, fx;
      axis_tap(sp.pw0 * P + x, it.src_w, it.dst_w, c0, c1, fx);
      col_c0[x] = c0 * 3; col_c1[x] = c1 * 3; col_fx[x] = fx;
    }
    for (int l = threadIdx.x; l < nlines; l += 256) {
      int r0, r1, fy;
      axis_tap(sp.ph * P + l % P, it.src_h, it.dst_h, r0, r1, fy);
      line_r0[l] = r0; line_r1[l] = r1; line_fy[l] = fy;
    }
    __syncthreads();
    for (int i = threadIdx.x; i < nlines * npx; i += 256) {
      const int line = i / npx, x = i - line * npx;
      const int f = still ? 0 : sp.t * TP + line / P;
      const uint8_t* fr = it.frames + (size_t)f * it.src_h * it.src_w * 3;
      const uint8_t* l0 = fr + (size_t)line_r0[line] * row_stride;
      const uint8_t* l1 = fr + (size_t)line_r1[line] * row_stride;
      const int c0 = col_c0[x], c1 = col_c1[x], fx = col_fx[x], fy = line_fy[line];
      const uint32_t w00 = (uint32_t)((kOne - fx) * (kOne - fy)), w01 = (uint32_t)(fx * (kOne - fy));
      const uint32_t w10 = (uint32_t)((kOne - fx) * fy), w11 = (uint32_t)(fx * fy);
#pragma unroll
      for (int c = 0; c < 3; ++c) {
        const uint32_t acc = (uint32_t)l0[c0 + c] * w00 + (uint32_t)l0[c1 + c] * w01 + (uint32_t)l1[c0 + c] * w10 +
                             (uint32_t)l1[c1 + c] * w11 + (1u << (2 * kFracBits - 1));
        seg[line][x * 3 + c] = (uint8_t)(acc >> (2 * kFracBits));
      }
    }
  }
  __syncthreads();
  // patch row of token (t, ph, pw): raster order, or merge-group-major order
  const int64_t row_base = sp.row_base;
  auto row_of = [&](int tok) -> int64_t { return (a.merge == 2) ? row_base + (tok >> 1) * 4 + (tok & 1) : row_base + tok; };
  typedef typename std::conditional<BF16, uint16_t, float>::type out_t;
  if constexpr (BF16 && P % 2 == 0) {
    // bf16: a lane produces pairs of neighbouring elements (dwords of a patch row) and consecutive lanes
    // produce consecutive dwords, so every store instruction writes whole cache lines; the padding columns
    // are dwords like the others.  A wave takes whole tokens, so a lane meets the same dwords of every row
    // it works on and decodes them (channel, frame, line, pixel pair) once.
    constexpr int KP = (3 * TP * P * P + 63) / 64 * 64;  // == a.k_pad (checked by the launcher)
    constexpr int PAIRS = KP / 2;                        // dwords per patch row
    constexpr int DP = 3 * TP * P * P / 2;               // of which carry pixels
    constexpr int HP = P / 2;                            // pairs per run
    constexpr int NJ = (PAIRS + 63) / 64;                // dwords per lane and row
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int soff[NJ], lbase[NJ];                             // byte offset of the pair's first pixel in seg (token 0), table row
    float sc[NJ], of[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int e = lane + 64 * j;
      soff[j] = -1; lbase[j] = 0;
      if (e < DP) {
        const int run = e / HP, i = e - run * HP;
        const int py = run % P, tt = (run / P) % TP, c = run / (P * TP);
        soff[j] = ((still ? 0 : tt) * P + py) * (SEG + 4) + c + 6 * i;
        lbase[j] = c * 256;
      }
      if constexpr (AFF) {
        // padding dwords read byte 0 of the strip and multiply it by zero: the loop below has no branches, so the
        // LDS reads of all dwords of a row are in flight together
        const int c = lbase[j] >> 8;
        sc[j] = soff[j] >= 0 ? a.aff_scale[c] : 0.f;
        of[j] = soff[j] >= 0 ? a.aff_off[c] : 0.f;
        soff[j] = max(soff[j], 0);
      }
    }
    const uint8_t* seg0 = &seg[0][0];
    for (int tok = wave; tok < ntok; tok += 4) {
      const uint8_t* sb = seg0 + tok * P * 3;
      uint32_t* orow = reinterpret_cast<uint32_t*>(reinterpret_cast<uint16_t*>(a.patches) + (size_t)row_of(tok) * KP);
      if constexpr (AFF) {
        uint32_t b0[NJ], b1[NJ];
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
          const uint8_t* px = sb + soff[j];
          b0[j] = px[0]; b1[j] = px[3];
        }
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
          const int e = lane + 64 * j;
          const uint32_t val = pack_bf16x2(__builtin_fmaf((float)b0[j], sc[j], of[j]), __builtin_fmaf((float)b1[j], sc[j], of[j]));
          if (64 * j + 63 < PAIRS || e < PAIRS) orow[e] = val;
        }
      } else {
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
          const int e = lane + 64 * j;
          if (e < PAIRS) {
            uint32_t val = 0u;
            if (soff[j] >= 0) {
              const uint8_t* px = sb + soff[j];
              val = (__float_as_uint(lut[lbase[j] + px[0]]) >> 16) | (__float_as_uint(lut[lbase[j] + px[3]]) & 0xFFFF0000u);
            }
            orow[e] = val;
          }
        }
      }
    }
  } else {
    for (int q = threadIdx.x; q < ntok * runs_per_row; q += 256) {
      const int tok = q / runs_per_row, run = q - tok * runs_per_row;
      const int k0 = run * P;
      out_t* out = reinterpret_cast<out_t*>(a.patches) + (size_t)row_of(tok) * a.k_pad + k0;
      if (run >= data_runs) {                            // padding columns
        const int n = min(P, a.k_pad - k0);
        for (int i = 0; i < n; ++i) out[i] = (out_t)0;
        continue;
      }
      const int py = run % P, tt = (run / P) % TP, c = run / (P * TP);
      const uint8_t* src = seg[(still ? 0 : tt) * P + py] + tok * P * 3 + c;
      const float* lc = lut + c * 256;
#pragma unroll
      for (int i = 0; i < P; ++i) {
        const float x = lc[src[3 * i]];
        if (BF16) reinterpret_cast<uint16_t*>(out)[i] = (uint16_t)(__float_as_uint(x) >> 16);
        else reinterpret_cast<float*>(out)[i] = x;
      }
    }
  }
}

template <int P_, int TP_>
static void launch_pp(const PreprocArgs& a, hipStream_t s) {
  const int P = a.patch;
  const int data_runs = 3 * a.tpatch * P;
  const int runs_per_row = data_runs + (a.k_pad - a.k + P - 1) / P;
  if (a.n_run_rows > 0) {
    const int64_t threads = a.n_run_rows * runs_per_row;
    dim3 grid((unsigned)((threads + 255) / 256)), block(256);
    if (a.out_bf16) hipLaunchKernelGGL((preprocess_kernel<P_, TP_, true>), grid, block, 0, s, a, runs_per_row, data_runs);
    else hipLaunchKernelGGL((preprocess_kernel<P_, TP_, false>), grid, block, 0, s, a, runs_per_row, data_runs);
  }
  if (a.n_strips > 0 && P_ != 0) {
    auto go = [&](auto res, int first, int count) {
      constexpr bool RES = decltype(res)::value;
      if (count <= 0) return;
      dim3 grid((unsigned)count), block(256);
      if (a.out_bf16 && a.affine && P_ % 2 == 0)
        hipLaunchKernelGGL((preprocess_strip_kernel<P_, TP_, true, true, RES>), grid, block, 0, s, a, first, runs_per_row, data_runs);
      else if (a.out_bf16)
        hipLaunchKernelGGL((preprocess_strip_kernel<P_, TP_, true, false, RES>), grid, block, 0, s, a, first, runs_per_row, data_runs);
      else
        hipLaunchKernelGGL((preprocess_strip_kernel<P_, TP_, false, false, RES>), grid, block, 0, s, a, first, runs_per_row, data_runs);
    };
    go(std::false_type{}, 0, a.n_copy_strips);
    go(std::true_type{}, a.n_copy_strips, a.n_strips - a.n_copy_strips);
  }
}

// patch sizes with a compiled strip kernel (the host plans strips only for these)
bool preprocess_has_strip_kernel(int patch, int tpatch) {
  return (patch == 14 && (tpatch == 1 || tpatch == 2)) || (patch == 16 && tpatch == 1);
}

hipError_t launch_preprocess(const PreprocArgs& a, hipStream_t s) {
  if (a.rows == 0) return hipSuccess;
  if (a.n_strips > 0 && !preprocess_has_strip_kernel(a.patch, a.tpatch)) return hipErrorInvalidValue;
  if (a.n_copy_strips < 0 || a.n_copy_strips > a.n_strips) return hipErrorInvalidValue;
  // the bf16 strip kernel writes dwords of rows of (K rounded up to 64) elements
  if (a.n_strips > 0 && a.out_bf16 && (a.k_pad != (a.k + 63) / 64 * 64 || reinterpret_cast<uintptr_t>(a.patches) % 16))
    return hipErrorInvalidValue;
  if (a.patch > kMaxPatch || a.rows * (int64_t)(3 * a.tpatch * a.patch + a.k_pad) > (1LL << 38)) return hipErrorInvalidValue;
  if (a.patch == 14 && a.tpatch == 2) launch_pp<14, 2>(a, s);
  else if (a.patch == 14 && a.tpatch == 1) launch_pp<14, 1>(a, s);
  else if (a.patch == 16 && a.tpatch == 1) launch_pp<16, 1>(a, s);
  else launch_pp<0, 0>(a, s);
  return hipGetLastError();
}

}  // namespace tcmv
