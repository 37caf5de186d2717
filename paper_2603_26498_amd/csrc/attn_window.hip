// Attention inside short windows (at most 64 tokens) on bf16 MFMA (gfx950).
//
// A windowed encoder layer has thousands of tiny attention problems (a window of 8 x 8
// patches is 64 tokens): 64 x 64 scores per head are a few microseconds of matrix work,
// the layer is bound by reading q, k, v and writing the output once.  What counts is
// therefore many resident workgroups and whole-line memory accesses, not the key loop of
// the long-sequence kernel (whose three-stage K/V ring leaves two workgroups per CU).
//
// One workgroup of two waves = one window and one head; a wave owns 32 query rows.  K
// (64 rows) and V^T (head_dim rows x 64 keys, already transposed and zero beyond the
// window) are staged once in 23 KB of LDS, six workgroups fit a CU.  As in the
// long-sequence kernel the scores are computed transposed, S^T = K * Q^T, so a lane holds
// one query column: all 64 scores of a query sit in the registers of two lanes, the
// softmax is the plain one (maximum, exponentials, no running statistics), and the
// probabilities, packed to bf16 in place, are the B operand of O^T += V^T * P^T.  The
// queries arrive multiplied by softmax scale * log2(e).  Workgroups that follow each
// other handle the heads of one window, so the lines of q and k they share are fetched once;
// the output tile leaves through LDS, 16 bytes per lane along a row.
#include "tcmv_internal.h"
#include "device_utils.h"

namespace tcmv {

namespace {
constexpr int kWinKeys = 64;
}

template <int DH>
__global__ __launch_bounds__(128) void attn_window_kernel(AttnArgs a) {
  constexpr int KS = DH / 16;                      // MFMA k-steps of the score product
  constexpr int DHP = (DH + 31) / 32 * 32;         // V^T rows incl. padding
  constexpr int MT = DHP / 32;                     // 32-row tiles of O^T
  constexpr bool ONES = (DH % 32) == 16;           // a padding row of ones yields the denominator
  constexpr int KCH = DH / 8;                      // 16-byte chunks per K row
  constexpr int KSTR = (KCH | 1) * 16;             // K row stride in LDS: odd number of chunks, conflict-free fragment reads
  __shared__ __attribute__((aligned(16))) uint8_t sk[kWinKeys * KSTR];
  __shared__ __attribute__((aligned(16))) uint8_t sv[DHP * 128];

  const int total = a.n_work * a.heads;
  const int chunk = (total + 7) >> 3;
  const int p = (int)(blockIdx.x & 7) * chunk + (int)(blockIdx.x >> 3);   // consecutive p on one XCD
  if (p >= total) return;
  const int wi = p / a.heads, head = p - wi * a.heads;
  const AttnWork w = a.work[wi];
  const int n = w.seg_len;                         // 1..64 keys = queries of the window
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr = lane & 31, lg = lane >> 5;
  const uint16_t* Q = reinterpret_cast<const uint16_t*>(a.q);
  const uint16_t* K = reinterpret_cast<const uint16_t*>(a.k);
  const uint16_t* VT = reinterpret_cast<const uint16_t*>(a.v);

  // K rows of the window (zeros beyond it), 16 bytes per lane along the row
  for (int i = tid; i < kWinKeys * KCH; i += 128) {
    const int r = i / KCH, c = i - r * KCH;
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (r < n) v = *reinterpret_cast<const uint4*>(K + (size_t)(w.seg_start + r) * a.ldqk + head * DH + c * 8);
    *reinterpret_cast<uint4*>(sk + r * KSTR + c * 16) = v;
  }
  // V^T rows of the head: 64 keys = 128 bytes each, chunks XOR-swizzled by (row/2)%8 so that 16 consecutive
  // rows reading the same logical chunk fall into different bank groups.  The buffer holds the keys of a group
  // of 16 in quarter order 0,2,1,3: chunk 2G+g is what the lanes of half-wave g contribute to k-step G.
  for (int i = tid; i < DHP * 8; i += 128) {
    const int r = i >> 3, c = i & 7;
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (r < DH) v = *reinterpret_cast<const uint4*>(VT + (size_t)(head * DH + r) * a.ldv + w.v0 + c * 8);
    else if (ONES && r == DH) v = make_uint4(0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u);
    *reinterpret_cast<uint4*>(sv + r * 128 + ((c ^ ((r >> 1) & 7)) << 4)) = v;
  }
  // query fragments (B operand of S^T = K Q^T); rows beyond the window repeat its last row and are not stored
  const int qi = wave * 32 + lr;
  const int qc = qi < n ? qi : n - 1;
  bf16x8 qf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks)
    qf[ks] = *reinterpret_cast<const bf16x8*>(Q + (size_t)(w.q0 + qc) * a.ldqk + head * DH + (2 * ks + lg) * 8);
  __syncthreads();
  // (in a window of at most 32 tokens the second wave computes on repeated rows and stores nothing)

  // scores: two blocks of 32 keys; a lane holds query lr and keys 32*kb + 8*(v/4) + 4*lg + v%4
  f32x16 s[2];
#pragma unroll
  for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
    for (int v = 0; v < 16; ++v) s[kb][v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const bf16x8 kf = *reinterpret_cast<const bf16x8*>(sk + (32 * kb + lr) * KSTR + (2 * ks + lg) * 16);
      s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], s[kb], 0, 0, 0);
    }
  }
  float m = -INFINITY;
#pragma unroll
  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int key = 32 * kb + 8 * (v >> 2) + 4 * lg + (v & 3);
      if (key >= n) s[kb][v] = -INFINITY;
      m = fmaxf(m, s[kb][v]);
    }
  m = fmaxf(m, __shfl_xor(m, 32, 64));             // the other half-wave holds the other keys of the same query
  // probabilities, rounded to bf16 where they enter the product; the denominator sums the rounded values
  bf16x8 pf[4];
  float l = 0.f;
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    uint32_t pk[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float p0 = __builtin_amdgcn_exp2f(s[g >> 1][8 * (g & 1) + 2 * j] - m);
      const float p1 = __builtin_amdgcn_exp2f(s[g >> 1][8 * (g & 1) + 2 * j + 1] - m);
      pk[j] = pack_bf16x2(p0, p1);
      if (!ONES) l += __uint_as_float(pk[j] << 16) + __uint_as_float(pk[j] & 0xFFFF0000u);
    }
    union { uint32_t u[4]; bf16x8 v; } cv;
    cv.u[0] = pk[0]; cv.u[1] = pk[1]; cv.u[2] = pk[2]; cv.u[3] = pk[3];
    pf[g] = cv.v;
  }
  // O^T += V^T P^T: rows = head dimensions, columns = queries
  f32x16 o[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
    for (int v = 0; v < 16; ++v) o[mt][v] = 0.f;
    const int row = 32 * mt + lr;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const bf16x8 vf = *reinterpret_cast<const bf16x8*>(sv + row * 128 + (((2 * g + lg) ^ ((row >> 1) & 7)) << 4));
      o[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[g], o[mt], 0, 0, 0);
    }
  }
  if (ONES) {
    constexpr int r = DH % 32;                     // row of the ones line inside its tile (16): held by the lower half-wave
    l = __shfl(o[DH / 32][4 * (r / 8)], lr, 64);
  } else {
    l += __shfl_xor(l, 32, 64);
  }
  const float inv = 1.0f / l;
  // The output leaves through LDS so that lanes run along the rows (16 bytes each, whole 2*DH-byte row pieces per
  // store) instead of writing 8-byte pieces of 32 different rows: each wave puts its 32 x DH tile (bf16) into its
  // half of the K buffer, which nobody reads any more once both waves are past their scores.
  __syncthreads();
  uint8_t* so = sk + wave * 32 * KSTR;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int vq = 0; vq < 4; ++vq) {
      const int dh0 = mt * 32 + 8 * vq + 4 * lg;
      if (dh0 < DH) {
        uint2 pk;
        pk.x = pack_bf16x2(o[mt][4 * vq] * inv, o[mt][4 * vq + 1] * inv);
        pk.y = pack_bf16x2(o[mt][4 * vq + 2] * inv, o[mt][4 * vq + 3] * inv);
        *reinterpret_cast<uint2*>(so + lr * KSTR + dh0 * 2) = pk;
      }
    }
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // the wave reads back only what it wrote itself
  for (int i = lane; i < 32 * KCH; i += 64) {
    const int r = i / KCH, c = i - r * KCH;
    if (wave * 32 + r < n) {
      const uint4 v = *reinterpret_cast<const uint4*>(so + r * KSTR + c * 16);
      *reinterpret_cast<uint4*>(reinterpret_cast<uint16_t*>(a.out) + (size_t)(w.q0 + wave * 32 + r) * a.ldo + head * DH + c * 8) = v;
    }
  }
}

// Every work item must be a whole window of at most 64 tokens (q0 == seg_start, nq == seg_len <= 64) and the
// queries must already carry the softmax scale; the caller guarantees both.
hipError_t launch_attn_window_bf16(const AttnArgs& a, hipStream_t s) {
  if (a.n_work == 0 || a.heads == 0) return hipSuccess;
  if (!a.prescaled || a.ldqk % 8 || a.ldv % 8 || a.ldo % 8 || reinterpret_cast<uintptr_t>(a.out) % 16) return hipErrorInvalidValue;
  const int64_t total = (int64_t)a.n_work * a.heads;
  if (total > (1 << 30)) return hipErrorInvalidValue;
  const unsigned grid = (unsigned)(((total + 7) / 8) * 8);
  switch (a.dh) {
    case 32: hipLaunchKernelGGL(attn_window_kernel<32>, dim3(grid), dim3(128), 0, s, a); break;
    case 64: hipLaunchKernelGGL(attn_window_kernel<64>, dim3(grid), dim3(128), 0, s, a); break;
    case 80: hipLaunchKernelGGL(attn_window_kernel<80>, dim3(grid), dim3(128), 0, s, a); break;
    case 96: hipLaunchKernelGGL(attn_window_kernel<96>, dim3(grid), dim3(128), 0, s, a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace tcmv
