// C = epilogue(A * W^T + bias) on bf16 MFMA (gfx950), fp32 accumulation.
//
// A [m, k] and W [n, k] are both contiguous along k, so both operands are staged
// the same way: 16-byte global loads -> registers -> LDS tile of 64 k-elements
// per row (128 bytes), with the 16-byte chunk index XOR-swizzled by the row so
// that the per-lane 16-byte MFMA operand reads (32 rows x same chunk) spread over
// all banks.  LDS is double buffered and the next tile's global loads are issued
// before the current tile's MFMAs.  Each wave owns a (BM/WM) x (BN/WN) sub-tile
// built from v_mfma_f32_32x32x16_bf16.
//
// The MFMA is issued with W as the row operand and A as the column operand, so
// the accumulator holds C^T: a lane owns ONE output row (token) and, per 32x32
// tile, four groups of four consecutive output columns.  The epilogue therefore
// works on 4-wide vectors: one 16-byte read-modify-write for the fp32 residual,
// one 8-byte store for bf16 outputs, a float4 of bias / position values; and the
// transposed-V store of the QKV projection has consecutive lanes on consecutive
// tokens (64-byte segments).
//
// Workgroups are numbered so that the eight XCDs (workgroup id mod 8) each walk
// a contiguous range of tiles: neighbouring tiles share A rows or W rows in the
// XCD's own L2.
#include "tcmv_internal.h"
#include "device_utils.h"
#include <cstdlib>

namespace tcmv {

template <int BM, int BN, int WM, int WN, int EPI>
__global__ __launch_bounds__(WM* WN * 64) void gemm_bf16_kernel(GemmArgs g) {
  constexpr int NT = WM * WN * 64;
  constexpr int BK = 64;
  constexpr int TM = BM / WM, TN = BN / WN, MI = TM / 32, NI = TN / 32;
  constexpr int A_CH = BM * 8 / NT, B_CH = BN * 8 / NT;
  static_assert(BM * 8 % NT == 0 && BN * 8 % NT == 0, "tile/threads mismatch");
  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
  constexpr int A_BYTES = BM * 128, B_BYTES = BN * 128, STAGE = A_BYTES + B_BYTES;

  const int tiles_n = (g.n + BN - 1) / BN;
  const int tiles_m = (int)((g.m + BM - 1) / BM);
  const int total = tiles_m * tiles_n;
  const int chunk = (total + 7) >> 3;
  const int p = (int)(blockIdx.x & 7) * chunk + (int)(blockIdx.x >> 3);
  if (p >= total) return;
  const int tm = p / tiles_n, tn = p - tm * tiles_n;
  const int64_t m0 = (int64_t)tm * BM;
  const int n0 = tn * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const uint16_t* A = reinterpret_cast<const uint16_t*>(g.a);
  const uint16_t* W = reinterpret_cast<const uint16_t*>(g.w);

  uint4 ra[A_CH], rb[B_CH];
  auto load_tiles = [&](int kt) {
#pragma unroll
    for (int i = 0; i < A_CH; ++i) {
      const int c = tid + i * NT, row = c >> 3, cc = c & 7;
      const int64_t gr = m0 + row;
      ra[i] = (gr < g.m) ? *reinterpret_cast<const uint4*>(A + (size_t)gr * g.lda + (size_t)kt * BK + cc * 8)
                         : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < B_CH; ++i) {
      const int c = tid + i * NT, row = c >> 3, cc = c & 7;
      const int gn = n0 + row;
      rb[i] = (gn < g.n) ? *reinterpret_cast<const uint4*>(W + (size_t)gn * g.k + (size_t)kt * BK + cc * 8)
                         : make_uint4(0, 0, 0, 0);
    }
  };
  auto store_tiles = [&](int buf) {
    uint8_t* sa = smem + buf * STAGE;
    uint8_t* sb = sa + A_BYTES;
#pragma unroll
    for (int i = 0; i < A_CH; ++i) {
      const int c = tid + i * NT, row = c >> 3, cc = c & 7;
      *reinterpret_cast<uint4*>(sa + row * 128 + ((cc ^ (row & 7)) << 4)) = ra[i];
    }
#pragma unroll
    for (int i = 0; i < B_CH; ++i) {
      const int c = tid + i * NT, row = c >> 3, cc = c & 7;
      *reinterpret_cast<uint4*>(sb + row * 128 + ((cc ^ (row & 7)) << 4)) = rb[i];
    }
  };

  f32x16 acc[MI][NI];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;

  const int nk = g.k / BK;
  load_tiles(0);
  store_tiles(0);
  __syncthreads();
  const int lr = lane & 31, lg = lane >> 5;
  for (int kt = 0; kt < nk; ++kt) {
    if (kt + 1 < nk) load_tiles(kt + 1);
    const uint8_t* sa = smem + (kt & 1) * STAGE;
    const uint8_t* sb = sa + A_BYTES;
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      bf16x8 af[MI], bfr[NI];
      const int ch = kk * 2 + lg;
#pragma unroll
      for (int mi = 0; mi < MI; ++mi) {
        const int row = wm * TM + mi * 32 + lr;
        af[mi] = *reinterpret_cast<const bf16x8*>(sa + row * 128 + ((ch ^ (row & 7)) << 4));
      }
#pragma unroll
      for (int ni = 0; ni < NI; ++ni) {
        const int row = wn * TN + ni * 32 + lr;
        bfr[ni] = *reinterpret_cast<const bf16x8*>(sb + row * 128 + ((ch ^ (row & 7)) << 4));
      }
#pragma unroll
      for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
          acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[ni], af[mi], acc[mi][ni], 0, 0, 0);
    }
    if (kt + 1 < nk) store_tiles((kt + 1) & 1);
    __syncthreads();
  }

  // ---- epilogue: lane holds row (lane & 31) and columns 8*(v/4) + 4*(lane>>5) + v%4 of each 32x32 tile
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) {
    const int64_t row = m0 + wm * TM + mi * 32 + lr;
    if (row >= g.m) continue;
    int64_t dst = row;
    int pi = 0, vc = 0;
    if (EPI == EPI_EMBED) {
      if (g.dst_row) dst = g.dst_row[row];
      if (g.pos_idx) pi = g.pos_idx[row];
    }
    if (EPI == EPI_QKV) vc = g.vcol[row];
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
#pragma unroll
      for (int vq = 0; vq < 4; ++vq) {
        const int col = n0 + wn * TN + ni * 32 + 8 * vq + 4 * lg;
        if (col >= g.n) continue;
        float4 val = make_float4(acc[mi][ni][4 * vq], acc[mi][ni][4 * vq + 1], acc[mi][ni][4 * vq + 2],
                                 acc[mi][ni][4 * vq + 3]);
        if (g.bias) {
          const float4 b4 = *reinterpret_cast<const float4*>(g.bias + col);
          val.x += b4.x; val.y += b4.y; val.z += b4.z; val.w += b4.w;
        }
        if (EPI == EPI_STORE || EPI == EPI_GELU || (EPI == EPI_QKV && col < g.split)) {
          if (EPI == EPI_GELU) {
            val.x = gelu_fast(val.x); val.y = gelu_fast(val.y); val.z = gelu_fast(val.z); val.w = gelu_fast(val.w);
          }
          uint2 pk;
          pk.x = pack_bf16x2(val.x, val.y);
          pk.y = pack_bf16x2(val.z, val.w);
          *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(g.c) + (size_t)row * g.ldc + col) = pk;
        } else if (EPI == EPI_RESID) {
          float4* c = reinterpret_cast<float4*>(reinterpret_cast<float*>(g.c) + (size_t)row * g.ldc + col);
          float4 old = *c;
          old.x += val.x; old.y += val.y; old.z += val.z; old.w += val.w;
          *c = old;
        } else if (EPI == EPI_EMBED) {
          if (g.pos_kind == 1) {
            const float4 p0 = *reinterpret_cast<const float4*>(g.pos0 + (size_t)pi * g.n + col);
            val.x += p0.x; val.y += p0.y; val.z += p0.z; val.w += p0.w;
          } else if (g.pos_kind == 2) {
            const float4 p0 = *reinterpret_cast<const float4*>(g.pos0 + (size_t)(pi & 0xFFFF) * g.n + col);
            const float4 p1 = *reinterpret_cast<const float4*>(g.pos1 + (size_t)(pi >> 16) * g.n + col);
            val.x += p0.x + p1.x; val.y += p0.y + p1.y; val.z += p0.z + p1.z; val.w += p0.w + p1.w;
          }
          *reinterpret_cast<float4*>(reinterpret_cast<float*>(g.c) + (size_t)dst * g.ldc + col) = val;
        } else if (EPI == EPI_QKV) {
          uint16_t* vt = reinterpret_cast<uint16_t*>(g.vt) + (size_t)(col - g.split) * g.ldvt + vc;
          vt[0] = f32_to_bf16(val.x);
          vt[g.ldvt] = f32_to_bf16(val.y);
          vt[2 * g.ldvt] = f32_to_bf16(val.z);
          vt[3 * g.ldvt] = f32_to_bf16(val.w);
        }
      }
    }
  }
}

template <int BM, int BN, int WM, int WN>
static hipError_t launch_cfg(const GemmArgs& a, hipStream_t s) {
  const int tiles_n = (a.n + BN - 1) / BN;
  const int64_t tiles_m = (a.m + BM - 1) / BM;
  const int64_t total = tiles_m * tiles_n;
  if (total <= 0) return hipSuccess;
  if (total > (1 << 30)) return hipErrorInvalidValue;
  const unsigned grid = (unsigned)(((total + 7) / 8) * 8);
  const size_t lds = 2 * (size_t)(BM + BN) * 128;
  dim3 block(WM * WN * 64);
#define TCMV_GEMM_CASE(E)                                                                              \
  case E: {                                                                                            \
    auto kern = gemm_bf16_kernel<BM, BN, WM, WN, E>;                                                   \
    if (lds > 64 * 1024) {                                                                             \
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                          \
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);        \
      if (e != hipSuccess) return e;                                                                   \
    }                                                                                                  \
    hipLaunchKernelGGL(kern, dim3(grid), block, lds, s, a);                                            \
    break;                                                                                             \
  }
  switch (a.epi) {
    TCMV_GEMM_CASE(EPI_STORE) TCMV_GEMM_CASE(EPI_GELU) TCMV_GEMM_CASE(EPI_RESID)
    TCMV_GEMM_CASE(EPI_EMBED) TCMV_GEMM_CASE(EPI_QKV)
    default: return hipErrorInvalidValue;
  }
#undef TCMV_GEMM_CASE
  return hipGetLastError();
}

hipError_t launch_gemm_bf16(const GemmArgs& a, hipStream_t s) {
  if (a.m == 0 || a.n == 0) return hipSuccess;
  if (a.k <= 0 || a.k % 64 || a.lda % 8 || a.n <= 0 || a.n % 8 || a.ldc % 4) return hipErrorInvalidValue;
  if (a.epi == EPI_QKV && (a.split % 4)) return hipErrorInvalidValue;
  static const int big = []{ const char* e = getenv("TCMV_GEMM_BIG"); return e ? atoi(e) : 0; }();
  if (big == 1) return launch_cfg<256, 256, 2, 2>(a, s);
  if (big == 2) return launch_cfg<256, 128, 2, 2>(a, s);
  if (big == 3) return launch_cfg<256, 256, 2, 4>(a, s);
  if (big == 4) return launch_cfg<256, 256, 4, 2>(a, s);
  if (big == 5) return launch_cfg<128, 256, 2, 2>(a, s);
  if (big == 6) return launch_cfg<256, 128, 4, 2>(a, s);
  return launch_cfg<128, 128, 2, 2>(a, s);
}

}  // namespace tcmv
